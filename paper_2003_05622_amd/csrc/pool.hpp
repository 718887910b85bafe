// Row gather + per-bag pooling: pooled[b, :] = sum over the bag's occurrences of the
// row of that occurrence's key (inv_len == null), or their mean (inv_len != null: it
// also receives 1 / (bag length) per bag, which the push needs to hand every occurrence
// its share of the bag's gradient).  A group of LPR lanes owns one bag at a time;
// each lane carries COLS float4 columns (lane*4 + k*LPR*4; COLS = 1 up to dim 256).
// Eight occurrences are in flight at a time: their ranks, then their row numbers,
// then their rows.  Block 0 also books the rows the preceding insert created.
#pragma once

#include "common.hpp"
#include "table.hpp"

namespace hps {

constexpr int kPoolThreads = 256;
constexpr int kPoolMaxBlocks = 1024;   // the groups loop over the bags (1536 to 3072 blocks measured no faster)
constexpr int kPoolInFlight = 8;

// The rows of the mini-batch's most frequent keys, held in LDS by every workgroup: a hash
// table from unique index to slot and the rows as float32.  Zipf-distributed keys send a large
// share of all occurrences to a few dozen keys; their rows then come from LDS instead of L2.
constexpr u32 kHotTable = 2048;          // hash slots (a power of two, at least 4 * kMaxHot)
constexpr u32 kHotEmpty = ~0u;
struct HotLds {
  u32 tag[kHotTable];                    // unique index, or kHotEmpty
  u32 slot[kHotTable];                   // which of the cached rows
  float4 rows[kHotBytes / 16];
};
__device__ __forceinline__ u32 hot_hash(u32 u) { return (u * 0x9E3779B1u) >> 21; }   // 11 bits

// All threads of the block; n_hot rows of dim floats fit kHotBytes.
__device__ __forceinline__ void load_hot_rows(HotLds& H, const TableView& t, const uint2* hot_list,
                                              u32 n_hot) {
  for (u32 i = threadIdx.x; i < kHotTable; i += kPoolThreads) H.tag[i] = kHotEmpty;
  __syncthreads();
  const u32 dim4 = t.dim >> 2;
  for (u32 i = threadIdx.x; i < n_hot; i += kPoolThreads) {
    const u32 u = hot_list[i].x;
    u32 h = hot_hash(u);
    while (atomicCAS(&H.tag[h], kHotEmpty, u) != kHotEmpty) h = (h + 1) & (kHotTable - 1);
    H.slot[h] = i;
  }
  for (u32 e = threadIdx.x; e < n_hot * dim4; e += kPoolThreads) {
    const u32 i = e / dim4, col = e % dim4;
    H.rows[e] = load_w4(t, hot_list[i].y, col);
  }
  __syncthreads();
}

// Slot of unique index u among the cached rows, or kHotEmpty.
__device__ __forceinline__ u32 hot_find(const HotLds& H, u32 u) {
  u32 h = hot_hash(u);
  while (true) {
    const u32 tag = H.tag[h];
    if (tag == u) return H.slot[h];
    if (tag == kHotEmpty) return kHotEmpty;
    h = (h + 1) & (kHotTable - 1);
  }
}

template <int LPR, int COLS, bool BF16, bool HOT>
__device__ __forceinline__ void pool_bags_as(const TableView& t, const i32* __restrict__ offsets,
                                             u32 n_bags, u32 n, const i32* __restrict__ inverse,
                                             const u32* __restrict__ rows, float* __restrict__ pooled,
                                             float* __restrict__ inv_len, const HotLds& H) {
  const u32 sub = threadIdx.x % LPR;
  const u32 dim4 = t.dim >> 2;
  const u32 n_groups = gridDim.x * (kPoolThreads / LPR);
  for (u32 b = (blockIdx.x * kPoolThreads + threadIdx.x) / LPR; b < n_bags; b += n_groups) {
    float4 acc[COLS];
#pragma unroll
    for (int c = 0; c < COLS; ++c) acc[c] = make_float4(0.f, 0.f, 0.f, 0.f);
    // clamped, so that no offsets array can make the kernel read outside inverse[0, n)
    const i32 lo = max(offsets[b], 0), hi = min(offsets[b + 1], (i32)n);
    for (i32 i0 = lo; i0 < hi; i0 += kPoolInFlight) {
      u32 r[kPoolInFlight];
      u32 hot[kPoolInFlight];      // slot among the rows in LDS, or kHotEmpty
#pragma unroll
      for (int k = 0; k < kPoolInFlight; ++k) r[k] = i0 + k < hi ? (u32)inverse[i0 + k] : 0u;
#pragma unroll
      for (int k = 0; k < kPoolInFlight; ++k) {
        hot[k] = (HOT && i0 + k < hi) ? hot_find(H, r[k]) : kHotEmpty;
        r[k] = (i0 + k < hi && hot[k] == kHotEmpty) ? rows[r[k]] : kNoRow;
      }
      // the rows as stored (all loads first: nothing between them that needs their data) ...
      StoredW4<BF16> raw[kPoolInFlight][COLS];
#pragma unroll
      for (int k = 0; k < kPoolInFlight; ++k) {
#pragma unroll
        for (int c = 0; c < COLS; ++c) {
          const u32 col = sub + c * LPR;
          raw[k][c] = (r[k] != kNoRow && col < dim4) ? load_stored_w4<BF16>(t, r[k], col) : StoredW4<BF16>();
        }
      }
      // ... then as float32 (all-zero bits are 0.0 in both formats); the cached rows from LDS
      float4 v[kPoolInFlight][COLS];
#pragma unroll
      for (int k = 0; k < kPoolInFlight; ++k)
#pragma unroll
        for (int c = 0; c < COLS; ++c) {
          const u32 col = sub + c * LPR;
          v[k][c] = (HOT && hot[k] != kHotEmpty && col < dim4) ? H.rows[hot[k] * dim4 + col] : raw[k][c].value();
        }
      // the (up to) eight rows as a balanced tree, then onto the running sum: a fixed shape,
      // and a smaller rounding error than adding one row after the other
#pragma unroll
      for (int c = 0; c < COLS; ++c) {
#pragma unroll
        for (int w = 1; w < kPoolInFlight; w <<= 1) {
#pragma unroll
          for (int k = 0; k + w < kPoolInFlight; k += 2 * w) {
            v[k][c].x += v[k + w][c].x; v[k][c].y += v[k + w][c].y;
            v[k][c].z += v[k + w][c].z; v[k][c].w += v[k + w][c].w;
          }
        }
        acc[c].x += v[0][c].x; acc[c].y += v[0][c].y; acc[c].z += v[0][c].z; acc[c].w += v[0][c].w;
      }
    }
    if (inv_len) {
      const float len = (float)max(hi - lo, 1);
      if (sub == 0) inv_len[b] = 1.0f / len;
#pragma unroll
      for (int c = 0; c < COLS; ++c) { acc[c].x /= len; acc[c].y /= len; acc[c].z /= len; acc[c].w /= len; }
    }
    float4* out = reinterpret_cast<float4*>(pooled + (u64)b * t.dim);
#pragma unroll
    for (int c = 0; c < COLS; ++c) {
      const u32 col = sub + c * LPR;
      if (col < dim4) out[col] = acc[c];
    }
  }
}

// hot_list / n_hot_ptr: the (unique index, row) pairs the lookup listed and their number
// (device); at most hot_cap of them are used (as many rows as fit kHotBytes).  HOT = false: no
// rows are kept in LDS.
template <int LPR, int COLS, bool HOT>
__global__ void __launch_bounds__(kPoolThreads)
pool_bags(TableView t, const i32* __restrict__ offsets, u32 n_bags, u32 n,
          const i32* __restrict__ inverse, const u32* __restrict__ rows,
          float* __restrict__ pooled, float* __restrict__ inv_len,
          const uint2* __restrict__ hot_list, const u32* __restrict__ n_hot_ptr, u32 hot_cap) {
  __shared__ HotLds H;
  if (load_error(t.st) != 0) return;
  if (blockIdx.x == 0 && threadIdx.x < kWave) commit_insert_wave(t.st);
  if (HOT) load_hot_rows(H, t, hot_list, min(*n_hot_ptr, hot_cap));
  if (t.bf16) pool_bags_as<LPR, COLS, true, HOT>(t, offsets, n_bags, n, inverse, rows, pooled, inv_len, H);
  else pool_bags_as<LPR, COLS, false, HOT>(t, offsets, n_bags, n, inverse, rows, pooled, inv_len, H);
}

// Measurement aid, not part of the path: reads random rows of LPR * 16 bytes of an array the
// way the pooling kernel reads table rows (LPR lanes x 16 bytes per row, eight rows in flight
// per lane group, same block size and grid) and nothing else, so that a benchmark can time
// the rate at which this GPU returns such rows.  Every lane group takes per_group rows
// (a multiple of 8) at pseudo-random places; the sums go to sink[group * LPR + lane] only
// to keep the loads alive.
template <int LPR>
__global__ void __launch_bounds__(kPoolThreads)
random_row_probe(const float4* __restrict__ rows, u64 n_rows, u32 per_group, float* __restrict__ sink) {
  const u32 group = (blockIdx.x * kPoolThreads + threadIdx.x) / LPR, sub = threadIdx.x % LPR;
  u64 state = mix64((u64)group + 1);
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  for (u32 i = 0; i < per_group; i += kPoolInFlight) {
    float4 v[kPoolInFlight];
#pragma unroll
    for (int k = 0; k < kPoolInFlight; ++k) {
      state = state * 6364136223846793005ull + 1442695040888963407ull;
      v[k] = rows[__umul64hi(state, n_rows) * LPR + sub];
    }
#pragma unroll
    for (int k = 0; k < kPoolInFlight; ++k) { acc.x += v[k].x; acc.y += v[k].y; acc.z += v[k].z; acc.w += v[k].w; }
  }
  sink[(u64)group * LPR + sub] = acc.x + acc.y + acc.z + acc.w;
}

}  // namespace hps
