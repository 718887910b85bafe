// Key dedup, part 1: stable least-significant-digit radix sort of
// (32-bit sort word, 32-bit occurrence index) pairs packed in one 64-bit word
// (sort word in the high half).  A 64-bit key order is obtained from two such
// sorts: by the low key half first, then -- after re-reading each element's key
// through its index -- by the high half.
//
// One pass = three kernels over tiles of kSortTile elements:
//   radix_hist     per-tile digit histogram            -> hist[digit][tile]
//   radix_scan     exclusive scan of hist in that order (one block)
//   radix_scatter  stable in-tile ranking with wave ballots, LDS staging,
//                  then digit runs are written out contiguously
#pragma once

#include "common.cuh"

namespace hps {

constexpr int kRadixBits = 8;
constexpr int kRadix = 1 << kRadixBits;
constexpr int kSortThreads = 256;
constexpr int kSortWaves = kSortThreads / kWave;
constexpr int kSortItems = 16;                         // per thread
constexpr int kSortTile = kSortThreads * kSortItems;   // 4096 elements
constexpr int kSortWaveSpan = kWave * kSortItems;      // 1024 consecutive elements per wave

__device__ __forceinline__ u32 pair_digit(u64 e, int shift) {
  return (u32)(e >> (32 + shift)) & (kRadix - 1);
}

// pairs[i] = (low or high 32 bits of keys[i], i)
__global__ void __launch_bounds__(256) pairs_from_keys(const u64* __restrict__ keys, u32 n,
                                                       int key_shift, u64* __restrict__ pairs) {
  const u32 i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const u64 k = keys[i];
  pairs[i] = ((u64)(u32)(k >> key_shift) << 32) | i;
}

// pairs[j] = (32 bits of keys[idx_j], idx_j) keeping the current order
__global__ void __launch_bounds__(256) pairs_regather(const u64* __restrict__ keys, u32 n,
                                                      int key_shift, u64* __restrict__ pairs) {
  const u32 j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= n) return;
  const u32 idx = (u32)pairs[j];
  const u64 k = keys[idx];
  pairs[j] = ((u64)(u32)(k >> key_shift) << 32) | idx;
}

__global__ void __launch_bounds__(kSortThreads) radix_hist(const u64* __restrict__ in, u32 n,
                                                           int shift, u32* __restrict__ hist,
                                                           u32 n_tiles) {
  __shared__ u32 h[kRadix];
  const u32 tile = blockIdx.x;
  for (int d = threadIdx.x; d < kRadix; d += kSortThreads) h[d] = 0;
  __syncthreads();
  const u32 base = tile * kSortTile;
#pragma unroll
  for (int k = 0; k < kSortItems; ++k) {
    const u32 i = base + k * kSortThreads + threadIdx.x;
    if (i < n) atomicAdd(&h[pair_digit(in[i], shift)], 1u);
  }
  __syncthreads();
  for (int d = threadIdx.x; d < kRadix; d += kSortThreads) hist[(u32)d * n_tiles + tile] = h[d];
}

// In-place exclusive scan of `len` counters by a single block of 1024 threads.
__global__ void __launch_bounds__(1024) scan_counters(u32* __restrict__ data, u32 len) {
  __shared__ u32 scratch[1024 / kWave + 1];
  const u32 per = (len + 1023) / 1024;
  const u32 lo = min(threadIdx.x * per, len), hi = min(lo + per, len);
  u32 s = 0;
  for (u32 i = lo; i < hi; ++i) s += data[i];
  u32 total;
  u32 run = block_excl_sum<1024>(s, scratch, &total);
  for (u32 i = lo; i < hi; ++i) {
    const u32 c = data[i];
    data[i] = run;
    run += c;
  }
}

__global__ void __launch_bounds__(kSortThreads)
radix_scatter(const u64* __restrict__ in, u64* __restrict__ out, u32 n, int shift,
              const u32* __restrict__ hist_scanned, u32 n_tiles) {
  __shared__ u32 wave_cnt[kSortWaves][kRadix];   // per-wave digit counts, then wave offsets
  __shared__ u32 local_start[kRadix];            // first staged position of each digit
  __shared__ u32 out_base[kRadix];               // global position of the digit's run - local_start
  __shared__ u32 scratch[kSortThreads / kWave + 1];
  __shared__ u64 stage[kSortTile];

  const u32 tile = blockIdx.x, tid = threadIdx.x;
  const u32 wave = tid / kWave, lane = tid & (kWave - 1);
  volatile u32* cnt = &wave_cnt[wave][0];
  for (int d = tid; d < kSortWaves * kRadix; d += kSortThreads) (&wave_cnt[0][0])[d] = 0;
  __syncthreads();

  const u32 tile_base = tile * kSortTile;
  const u32 tile_n = min((u32)kSortTile, n - tile_base);
  const u32 wave_base = tile_base + wave * kSortWaveSpan;
  const u64 lt = lanemask_lt();

  u64 e[kSortItems];
  u32 rank[kSortItems];
#pragma unroll
  for (int r = 0; r < kSortItems; ++r) {
    const u32 i = wave_base + r * kWave + lane;
    e[r] = (i < n) ? in[i] : ~0ull;
  }
  // Round by round, rank each element among the wave's earlier elements with the
  // same digit (element order inside a wave is round-major, then lane).
#pragma unroll
  for (int r = 0; r < kSortItems; ++r) {
    const u32 i = wave_base + r * kWave + lane;
    const bool valid = i < n;
    const u32 d = pair_digit(e[r], shift);
    u64 same = __ballot(valid);
#pragma unroll
    for (int b = 0; b < kRadixBits; ++b) {
      const bool bit = (d >> b) & 1;
      const u64 bb = __ballot(bit);
      same &= bit ? bb : ~bb;
    }
    const u32 before = __popcll(same & lt);
    u32 old = 0;
    if (valid) old = cnt[d];
    __builtin_amdgcn_wave_barrier();
    if (valid && before == 0) cnt[d] = old + __popcll(same);
    __builtin_amdgcn_wave_barrier();
    rank[r] = old + before;
  }
  __syncthreads();

  // Per digit: offsets of each wave inside the digit's run, and the tile's digit count.
  u32 digit_total = 0;
  if (tid < kRadix) {
#pragma unroll
    for (int w = 0; w < kSortWaves; ++w) {
      const u32 c = wave_cnt[w][tid];
      wave_cnt[w][tid] = digit_total;
      digit_total += c;
    }
  }
  u32 tile_total;
  const u32 start = block_excl_sum<kSortThreads>(tid < kRadix ? digit_total : 0, scratch,
                                                 &tile_total);
  if (tid < kRadix) {
    local_start[tid] = start;
    out_base[tid] = hist_scanned[tid * n_tiles + tile] - start;
  }
  __syncthreads();

#pragma unroll
  for (int r = 0; r < kSortItems; ++r) {
    const u32 i = wave_base + r * kWave + lane;
    if (i < n) {
      const u32 d = pair_digit(e[r], shift);
      stage[local_start[d] + wave_cnt[wave][d] + rank[r]] = e[r];
    }
  }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < kSortItems; ++k) {
    const u32 p = k * kSortThreads + tid;
    if (p < tile_n) {
      const u64 el = stage[p];
      out[out_base[pair_digit(el, shift)] + p] = el;
    }
  }
}

}  // namespace hps
