// Key dedup, part 1: ordering the key occurrences.
//
// Each occurrence i becomes one 64-bit element: the key's high bits with the
// occurrence index in the low `idx_bits` bits (idx_bits = bits needed for N).
// Elements are sorted by their top `8 * n_pass` bits with a stable
// least-significant-digit radix sort, 8 bits per pass, ONE kernel per pass:
//
//   sort_prepare    digit histograms of all passes in one read of the keys
//   onesweep_pass   a tile takes a ticket, ranks its elements with wave ballots,
//                   obtains the number of same-digit elements in earlier tiles by
//                   decoupled look-back over per-tile status words, stages the tile
//                   in LDS and writes each digit's run contiguously.
//
// Mini-batch keys are hashed feature ids, so the top 8*n_pass bits separate
// almost all distinct keys; the rare runs that still mix different keys are
// found and put right afterwards (dedup.cuh), so the result is exact for any input.
//
// Look-back status word (64-bit): epoch << 34 | flag << 32 | count.  The epoch is
// the pull's serial number, so words of earlier pulls read as "not ready" and
// nothing has to be cleared between pulls.
#pragma once

#include "common.cuh"

namespace hps {

constexpr int kRadixBits = 8;
constexpr int kRadix = 1 << kRadixBits;
constexpr int kMaxPasses = 8;
constexpr int kSortThreads = 256;
constexpr int kSortWaves = kSortThreads / kWave;
constexpr int kSortItems = 16;                         // per thread
constexpr int kSortTile = kSortThreads * kSortItems;   // 4096 elements
constexpr int kSortWaveSpan = kWave * kSortItems;      // 1024 consecutive elements per wave

constexpr u64 kFlagAggregate = 1;   // count of this tile only
constexpr u64 kFlagInclusive = 2;   // count of this tile and all earlier tiles
constexpr u32 kSpinLimit = 1u << 26;

struct SortPlan {
  int n_pass;       // digits sorted
  int idx_bits;     // low bits of an element that hold the occurrence index
  int low_shift;    // 64 - 8 * n_pass: position of the least significant sorted digit
};

__device__ __forceinline__ u64 make_elem(u64 key, u32 i, int idx_bits) {
  return ((key >> idx_bits) << idx_bits) | (u64)i;
}
__device__ __forceinline__ u32 elem_idx(u64 e, int idx_bits) {
  return (u32)(e & ((1ull << idx_bits) - 1));
}
__device__ __forceinline__ u32 elem_digit(u64 e, int shift) {
  return (u32)(e >> shift) & (kRadix - 1);
}

__device__ __forceinline__ u64 state_word(u32 epoch, u64 flag, u32 count) {
  return ((u64)epoch << 34) | (flag << 32) | count;
}

// Number of lanes of the wave (among `valid` ones) whose digit equals this lane's,
// and how many of them have a lower lane id.
__device__ __forceinline__ void match_digit(u32 d, bool valid, u64 lt, u32* before, u32* count) {
  u64 same = __ballot(valid);
#pragma unroll
  for (int b = 0; b < kRadixBits; ++b) {
    const bool bit = (d >> b) & 1;
    const u64 bb = __ballot(bit);
    same &= bit ? bb : ~bb;
  }
  *before = __popcll(same & lt);
  *count = __popcll(same);
}

// Histograms of every pass's digit over all keys; also resets what the passes need.
//   ghist      [kMaxPasses][kRadix] of this pull (zero on entry), ghist_next the
//              buffer the next pull will use (cleared here)
//   tickets    [kMaxPasses + 1] tile tickets of the passes and of the unique scan
__global__ void __launch_bounds__(kSortThreads)
sort_prepare(const u64* __restrict__ keys, u32 n, SortPlan plan, u32* __restrict__ ghist,
             u32* __restrict__ ghist_next, u32* __restrict__ tickets, PullCtx* __restrict__ ctx) {
  __shared__ u32 h[kMaxPasses][kRadix];
  for (int i = threadIdx.x; i < kMaxPasses * kRadix; i += kSortThreads) (&h[0][0])[i] = 0;
  if (blockIdx.x == 0) {
    for (int i = threadIdx.x; i < kMaxPasses * kRadix; i += kSortThreads) ghist_next[i] = 0;
    if (threadIdx.x <= kMaxPasses) tickets[threadIdx.x] = 0;
    if (threadIdx.x == 0) {
      ctx->n_unique = 0;
      ctx->n_long = 0;
      ctx->n_chunk_items = 0;
      ctx->n_evidence = 0;
      ctx->sort_error = 0;
    }
  }
  __syncthreads();
  const u32 n_tiles = (n + kSortTile - 1) / kSortTile;
  for (u32 tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
    const u32 base = tile * kSortTile;
#pragma unroll 4
    for (int k = 0; k < kSortItems; ++k) {
      const u32 i = base + k * kSortThreads + threadIdx.x;
      if (i < n) {
        const u64 key = keys[i];
        for (int p = 0; p < plan.n_pass; ++p)
          atomicAdd(&h[p][(u32)(key >> (plan.low_shift + p * kRadixBits)) & (kRadix - 1)], 1u);
      }
    }
  }
  __syncthreads();
  for (int i = threadIdx.x; i < plan.n_pass * kRadix; i += kSortThreads) {
    const u32 c = (&h[0][0])[i];
    if (c) atomicAdd(&ghist[i], c);
  }
}

// One stable radix pass.  FIRST: elements are built from the keys; otherwise read
// from `in`.  `ghist` is this pass's global digit histogram, `state` this pass's
// [n_tiles][kRadix] status words.
template <bool FIRST>
__global__ void __launch_bounds__(kSortThreads)
onesweep_pass(const u64* __restrict__ keys, const u64* __restrict__ in, u64* __restrict__ out,
              u32 n, int shift, int idx_bits, const u32* __restrict__ ghist,
              u64* __restrict__ state, u32* __restrict__ ticket, u32 epoch,
              PullCtx* __restrict__ ctx) {
  __shared__ u32 wave_cnt[kSortWaves][kRadix];   // per-wave digit counts, then wave offsets
  __shared__ u32 local_start[kRadix];            // first staged position of each digit
  __shared__ u32 out_base[kRadix];               // global position of the digit's run - local_start
  __shared__ u32 scratch[kSortThreads / kWave + 1];
  __shared__ u32 s_tile;
  __shared__ u64 stage[kSortTile];

  const u32 tid = threadIdx.x;
  if (tid == 0) s_tile = atomicAdd(ticket, 1u);
  for (int d = tid; d < kSortWaves * kRadix; d += kSortThreads) (&wave_cnt[0][0])[d] = 0;
  __syncthreads();
  const u32 tile = s_tile;
  const u32 wave = tid / kWave, lane = tid & (kWave - 1);
  volatile u32* cnt = &wave_cnt[wave][0];

  const u32 tile_base = tile * kSortTile;
  const u32 tile_n = min((u32)kSortTile, n - tile_base);
  const u32 wave_base = tile_base + wave * kSortWaveSpan;
  const u64 lt = lanemask_lt();

  u64 e[kSortItems];
  u32 rank[kSortItems];
#pragma unroll
  for (int r = 0; r < kSortItems; ++r) {
    const u32 i = wave_base + r * kWave + lane;
    if (FIRST)
      e[r] = (i < n) ? make_elem(keys[i], i, idx_bits) : ~0ull;
    else
      e[r] = (i < n) ? in[i] : ~0ull;
  }
  // Rank each element among the wave's earlier elements with the same digit
  // (element order inside a wave: round by round, then by lane).
#pragma unroll
  for (int r = 0; r < kSortItems; ++r) {
    const u32 i = wave_base + r * kWave + lane;
    const bool valid = i < n;
    const u32 d = elem_digit(e[r], shift);
    u32 before, same;
    match_digit(d, valid, lt, &before, &same);
    u32 old = 0;
    if (valid) old = cnt[d];
    __builtin_amdgcn_wave_barrier();
    if (valid && before == 0) cnt[d] = old + same;
    __builtin_amdgcn_wave_barrier();
    rank[r] = old + before;
  }
  __syncthreads();

  // Thread d owns digit d: the tile's count, the waves' offsets inside the run.
  u32 digit_total = 0;
#pragma unroll
  for (int w = 0; w < kSortWaves; ++w) {
    const u32 c = wave_cnt[w][tid];
    wave_cnt[w][tid] = digit_total;
    digit_total += c;
  }
  // Publish, then look back over earlier tiles for the same digit.
  u64* my_state = state + (u64)tile * kRadix + tid;
  u32 earlier = 0;
  if (tile == 0) {
    __hip_atomic_store(my_state, state_word(epoch, kFlagInclusive, digit_total), __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
  } else {
    __hip_atomic_store(my_state, state_word(epoch, kFlagAggregate, digit_total), __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
    u32 prev = tile - 1;
    u32 spins = 0;
    while (true) {
      const u64 w = __hip_atomic_load(state + (u64)prev * kRadix + tid, __ATOMIC_RELAXED,
                                      __HIP_MEMORY_SCOPE_AGENT);
      const u64 flag = (w >> 32) & 3;
      if ((u32)(w >> 34) != epoch || flag == 0) {
        if (++spins > kSpinLimit) { ctx->sort_error = 1; break; }   // never expected
        __builtin_amdgcn_s_sleep(1);
        continue;
      }
      earlier += (u32)w;
      if (flag == kFlagInclusive || prev == 0) break;
      --prev;
    }
    __hip_atomic_store(my_state, state_word(epoch, kFlagInclusive, earlier + digit_total),
                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  u32 total;
  const u32 gbase = block_excl_sum<kSortThreads>(ghist[tid], scratch, &total);
  const u32 start = block_excl_sum<kSortThreads>(digit_total, scratch, &total);
  local_start[tid] = start;
  out_base[tid] = gbase + earlier - start;
  __syncthreads();

#pragma unroll
  for (int r = 0; r < kSortItems; ++r) {
    const u32 i = wave_base + r * kWave + lane;
    if (i < n) {
      const u32 d = elem_digit(e[r], shift);
      stage[local_start[d] + wave_cnt[wave][d] + rank[r]] = e[r];
    }
  }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < kSortItems; ++k) {
    const u32 p = k * kSortThreads + tid;
    if (p < tile_n) {
      const u64 el = stage[p];
      out[out_base[elem_digit(el, shift)] + p] = el;
    }
  }
}

}  // namespace hps
