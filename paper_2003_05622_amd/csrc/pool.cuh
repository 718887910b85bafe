// Row gather + per-bag sum pooling: pooled[b, :] = sum over the bag's occurrences
// of the row of that occurrence's key.  A group of LPR lanes owns one bag; each lane
// carries float4 columns (lane*4 + k*LPR*4).  Four occurrences are in flight at a
// time: their ranks, then their row numbers, then their rows.
#pragma once

#include "common.cuh"
#include "table.cuh"

namespace hps {

constexpr int kPoolThreads = 256;
constexpr int kPoolMaxBlocks = 2048;   // the groups loop over the bags
constexpr int kPoolCols = 4;   // float4 columns per lane: dim <= LPR * 16

template <int LPR>
__device__ __forceinline__ void add_row(float4* acc, const TableView& t, u32 r, u32 sub) {
  if (r == kNoRow) return;
  const float4* row = reinterpret_cast<const float4*>(t.w + (u64)r * t.dim);
  const u32 dim4 = t.dim >> 2;
#pragma unroll
  for (int c = 0; c < kPoolCols; ++c) {
    const u32 col = sub + c * LPR;
    if (col < dim4) {
      const float4 v = row[col];
      acc[c].x += v.x; acc[c].y += v.y; acc[c].z += v.z; acc[c].w += v.w;
    }
  }
}

template <int LPR>
__global__ void __launch_bounds__(kPoolThreads)
pool_bags(TableView t, const i32* __restrict__ offsets, u32 n_bags, u32 n,
          const i32* __restrict__ inverse, const u32* __restrict__ rows,
          float* __restrict__ pooled) {
  const u32 sub = threadIdx.x % LPR;
  if (load_error(t.st) != 0) return;
  const u32 dim4 = t.dim >> 2;
  const u32 n_groups = gridDim.x * (kPoolThreads / LPR);
  for (u32 b = (blockIdx.x * kPoolThreads + threadIdx.x) / LPR; b < n_bags; b += n_groups) {
  float4 acc[kPoolCols];
#pragma unroll
  for (int c = 0; c < kPoolCols; ++c) acc[c] = make_float4(0.f, 0.f, 0.f, 0.f);
  // clamped, so that no offsets array can make the kernel read outside inverse[0, n)
  const i32 lo = max(offsets[b], 0), hi = min(offsets[b + 1], (i32)n);
  i32 i = lo;
  for (; i + 3 < hi; i += 4) {
    const i32 u0 = inverse[i], u1 = inverse[i + 1], u2 = inverse[i + 2], u3 = inverse[i + 3];
    const u32 r0 = rows[u0], r1 = rows[u1], r2 = rows[u2], r3 = rows[u3];
    float4 a0[kPoolCols], a1[kPoolCols], a2[kPoolCols], a3[kPoolCols];
#pragma unroll
    for (int c = 0; c < kPoolCols; ++c) a0[c] = a1[c] = a2[c] = a3[c] = make_float4(0.f, 0.f, 0.f, 0.f);
    add_row<LPR>(a0, t, r0, sub);
    add_row<LPR>(a1, t, r1, sub);
    add_row<LPR>(a2, t, r2, sub);
    add_row<LPR>(a3, t, r3, sub);
    // same order of additions as one occurrence after the other
#pragma unroll
    for (int c = 0; c < kPoolCols; ++c) {
      acc[c].x = (((acc[c].x + a0[c].x) + a1[c].x) + a2[c].x) + a3[c].x;
      acc[c].y = (((acc[c].y + a0[c].y) + a1[c].y) + a2[c].y) + a3[c].y;
      acc[c].z = (((acc[c].z + a0[c].z) + a1[c].z) + a2[c].z) + a3[c].z;
      acc[c].w = (((acc[c].w + a0[c].w) + a1[c].w) + a2[c].w) + a3[c].w;
    }
  }
  if (i < hi) {
    const i32 u0 = inverse[i];
    const i32 u1 = i + 1 < hi ? inverse[i + 1] : u0;
    const i32 u2 = i + 2 < hi ? inverse[i + 2] : u0;
    const u32 r0 = rows[u0], r1 = rows[u1], r2 = rows[u2];
    add_row<LPR>(acc, t, r0, sub);
    if (i + 1 < hi) add_row<LPR>(acc, t, r1, sub);
    if (i + 2 < hi) add_row<LPR>(acc, t, r2, sub);
  }
  float4* out = reinterpret_cast<float4*>(pooled + (u64)b * t.dim);
#pragma unroll
  for (int c = 0; c < kPoolCols; ++c) {
    const u32 col = sub + c * LPR;
    if (col < dim4) out[col] = acc[c];
  }
  }
}

}  // namespace hps
