// Row gather + per-bag sum pooling: pooled[b, :] = sum over the bag's occurrences
// of the row of that occurrence's key.  A group of LPR lanes owns one bag; each lane
// carries float4 columns (lane*4 + k*LPR*4).  Also records, per occurrence, the bag
// it belongs to (needed by the push).
#pragma once

#include "common.cuh"
#include "table.cuh"

namespace hps {

constexpr int kPoolThreads = 256;

template <int LPR>
__global__ void __launch_bounds__(kPoolThreads)
pool_bags(TableView t, const i32* __restrict__ offsets, u32 n_bags,
          const i32* __restrict__ inverse, const u32* __restrict__ rows,
          float* __restrict__ pooled, i32* __restrict__ bag_of) {
  constexpr int kMaxCols = 4;   // float4 columns per lane: dim <= LPR * 16
  const u32 b = (blockIdx.x * kPoolThreads + threadIdx.x) / LPR;
  const u32 sub = threadIdx.x % LPR;
  if (b >= n_bags) return;
  if (load_error(t.st) != 0) return;
  const u32 dim4 = t.dim >> 2;
  float4 acc[kMaxCols];
#pragma unroll
  for (int c = 0; c < kMaxCols; ++c) acc[c] = make_float4(0.f, 0.f, 0.f, 0.f);
  const i32 lo = offsets[b], hi = offsets[b + 1];
  for (i32 i = lo; i < hi; ++i) {
    const u32 r = rows[inverse[i]];
    if (sub == 0) bag_of[i] = (i32)b;
    if (r == kNoRow) continue;
    const float4* row = reinterpret_cast<const float4*>(t.w + (u64)r * t.dim);
#pragma unroll
    for (int c = 0; c < kMaxCols; ++c) {
      const u32 col = sub + c * LPR;
      if (col < dim4) {
        const float4 v = row[col];
        acc[c].x += v.x; acc[c].y += v.y; acc[c].z += v.z; acc[c].w += v.w;
      }
    }
  }
  float4* out = reinterpret_cast<float4*>(pooled + (u64)b * t.dim);
#pragma unroll
  for (int c = 0; c < kMaxCols; ++c) {
    const u32 col = sub + c * LPR;
    if (col < dim4) out[col] = acc[c];
  }
}

}  // namespace hps
