// Key dedup, part 2, plain form (a table's first dedups and very large ones; the usual
// form is in bucket.hpp): from the occurrences sorted by the top bits of their keys
// (skeys[j], spay[j]; payload = occurrence index | bag << 32) to
//   uniq[U]      ascending unique keys
//   inverse[N]   rank of each occurrence's key among them
//   bagperm[N]   bag of each occurrence, occurrences grouped by key (ascending key)
//   seg_off[U+1] start of each key's group in bagperm
//
//   unique_emit     group heads, their running count across tiles by decoupled
//                   look-back, and all outputs.  It also records "evidence": positions
//                   where two neighbours agree in the sorted bits but are different
//                   keys, i.e. where the order below the sorted bits may be wrong.
//   fix_mixed_runs  one workgroup; does nothing without evidence (the normal case
//                   for hashed keys); otherwise orders every mixed run by full key --
//                   runs of up to 64 elements inside one wave, longer ones (or, with
//                   too much evidence, the whole array) by a workgroup-local radix
//                   sort through global memory;
//   unique_emit     runs a second time, and only does anything then, if there was
//                   evidence (REDO instance).
#pragma once

#include "common.hpp"
#include "sort.hpp"

namespace hps {

constexpr int kHeadThreads = 256;
constexpr int kHeadItems = 8;
constexpr int kHeadTile = kHeadThreads * kHeadItems;
constexpr int kFixThreads = 1024;
constexpr int kFixWaves = kFixThreads / kWave;

// ---- workgroup-local (one block of kFixThreads) stable radix sort of the pairs in
// ---- [a, b) by the full 64-bit key, through global memory.  Slow; rare inputs only.

struct FixLds {
  u32 hist[kRadix];
  u32 bin[kRadix];
  u32 wave_cnt[kFixWaves][kRadix];
  u32 scratch[kFixThreads / kWave + 1];
};

__device__ void wg_radix_pass(const u64* ksrc, const u64* isrc, u64* kdst, u64* idst, u32 a, u32 b,
                              int shift, FixLds& L) {
  const u32 tid = threadIdx.x, wave = tid / kWave;
  const u64 lt = lanemask_lt();
  if (tid < kRadix) L.hist[tid] = 0;
  __syncthreads();
  for (u32 j = a + tid; j < b; j += kFixThreads) atomicAdd(&L.hist[key_digit(ksrc[j], shift)], 1u);
  __syncthreads();
  u32 total;
  const u32 ex = block_excl_sum<kFixThreads>(tid < kRadix ? L.hist[tid] : 0, L.scratch, &total);
  if (tid < kRadix) L.bin[tid] = a + ex;
  __syncthreads();
  for (u32 base = a; base < b; base += kFixThreads) {
    const u32 j = base + tid;
    const bool valid = j < b;
    const u64 key = valid ? ksrc[j] : 0;
    const u64 idx = valid ? isrc[j] : 0;
    const u32 d = key_digit(key, shift);
    u32 before, same;
    match_digit(d, valid, lt, &before, &same);
    const bool leader = valid && before == 0;
    if (leader) L.wave_cnt[wave][d] = same;
    __syncthreads();
    u32 dest = 0;
    if (valid) {
      dest = L.bin[d] + before;
      for (u32 w = 0; w < wave; ++w) dest += L.wave_cnt[w][d];
    }
    __syncthreads();
    if (leader) {
      atomicAdd(&L.bin[d], same);
      L.wave_cnt[wave][d] = 0;
    }
    if (valid) { kdst[dest] = key; idst[dest] = idx; }
    __syncthreads();
  }
}

// Orders the pairs in [a, b) by full key; equal keys keep their order.  Eight passes
// (an even number), so the result ends up in (skeys, sidx) again.
__device__ void wg_sort_range_full(u64* skeys, u64* sidx, u64* kalt, u64* ialt, u32 a, u32 b,
                                   FixLds& L) {
  for (int w = threadIdx.x; w < kFixWaves * kRadix; w += kFixThreads) (&L.wave_cnt[0][0])[w] = 0;
  __syncthreads();
  for (int shift = 0; shift < 64; shift += 2 * kRadixBits) {
    wg_radix_pass(skeys, sidx, kalt, ialt, a, b, shift, L);
    wg_radix_pass(kalt, ialt, skeys, sidx, a, b, shift + kRadixBits, L);
  }
}

__global__ void __launch_bounds__(kFixThreads)
fix_mixed_runs(u64* __restrict__ skeys, u64* __restrict__ sidx, u64* __restrict__ kalt,
               u64* __restrict__ ialt, u32 n, const PullCtx* __restrict__ ctx,
               const u32* __restrict__ evidence) {
  const u32 E = ctx->n_evidence;
  if (E == 0) return;
  __shared__ FixLds L;
  __shared__ u32 ev[kMaxEvidence];
  __shared__ u32 run_lo[kMaxEvidence];
  __shared__ u32 run_hi[kMaxEvidence];
  const u32 tid = threadIdx.x;
  if (E > kMaxEvidence) {
    wg_sort_range_full(skeys, sidx, kalt, ialt, 0, n, L);
    return;
  }
  // sort the evidence positions (bitonic, one per thread)
  ev[tid] = tid < E ? evidence[tid] : ~0u;
  for (u32 k = 2; k <= kMaxEvidence; k <<= 1) {
    for (u32 j = k >> 1; j > 0; j >>= 1) {
      __syncthreads();
      const u32 partner = tid ^ j;
      if (partner > tid) {
        const u32 x = ev[tid], y = ev[partner];
        const bool up = (tid & k) == 0;
        if ((x > y) == up) { ev[tid] = y; ev[partner] = x; }
      }
    }
  }
  __syncthreads();
  // the run of equal sorted bits around each evidence position; later evidence of the
  // same run is dropped (run_lo = run_hi)
  if (tid < E) {
    const u32 j = ev[tid];
    const KeyRange range = ctx->range;
    const u64 v = sorted_prefix(skeys[j], range);
    u32 lo = 0, hi = j;                       // first position with top bits >= v
    while (lo < hi) {
      const u32 mid = lo + (hi - lo) / 2;
      if (sorted_prefix(skeys[mid], range) < v) lo = mid + 1; else hi = mid;
    }
    const u32 a = lo;
    lo = j; hi = n;                           // first position with top bits > v
    while (lo < hi) {
      const u32 mid = lo + (hi - lo) / 2;
      if (sorted_prefix(skeys[mid], range) <= v) lo = mid + 1; else hi = mid;
    }
    const bool first = tid == 0 || ev[tid - 1] < a;
    run_lo[tid] = a;
    run_hi[tid] = first ? lo : a;
  }
  __syncthreads();
  // short runs: one wave each, rank by comparing against every other element
  const u32 wave = tid / kWave, lane = tid & (kWave - 1);
  for (u32 r = wave; r < E; r += kFixWaves) {
    const u32 a = run_lo[r], len = run_hi[r] - a;
    if (len == 0 || len > (u32)kWave) continue;
    u64 key = 0, idx = 0;       // idx: the payload; its low half (the index) breaks ties
    if (lane < len) { key = skeys[a + lane]; idx = sidx[a + lane]; }
    u32 rank = 0;
    for (u32 m = 0; m < len; ++m) {
      const u64 okey = __shfl(key, (int)m, kWave);
      const u64 oidx = __shfl(idx, (int)m, kWave);
      rank += (okey < key || (okey == key && (u32)oidx < (u32)idx)) ? 1u : 0u;
    }
    if (lane < len) { skeys[a + rank] = key; sidx[a + rank] = idx; }
  }
  __syncthreads();
  // long runs: the whole workgroup, one run after the other
  for (u32 r = 0; r < E; ++r) {
    const u32 a = run_lo[r], b = run_hi[r];
    if (b - a > (u32)kWave) wg_sort_range_full(skeys, sidx, kalt, ialt, a, b, L);
  }
}

// Heads of the key groups, their ranks, and every output of the dedup.
//   head_rows [n_tiles] and head_groups [n_groups]: status words of the tiles' and
//   tile groups' head counts (see sort.hpp), ticket: tile tickets
//   bagperm[j] = bag of the occurrence at sorted position j, bit 31 set on group heads
// REDO = false: the first instance; counts evidence.  REDO = true: the instance after
// fix_mixed_runs; returns at once unless there was evidence.
template <bool REDO>
__global__ void __launch_bounds__(kHeadThreads)
unique_emit(const u64* __restrict__ skeys, const u64* __restrict__ spay, u32 n,
            u32* __restrict__ head_rows, u32* __restrict__ head_groups, u32 group,
            u32* __restrict__ ticket, u32 epoch,
            u32 n_bags, u64* __restrict__ uniq,
            i32* __restrict__ inverse, u32* __restrict__ bagperm, u32* __restrict__ seg_off,
            PullCtx* __restrict__ ctx, u32* __restrict__ evidence, TableState* __restrict__ st) {
  __shared__ u32 scratch[kHeadThreads / kWave + 1];
  __shared__ u32 s_tile, s_earlier;
  __shared__ u64 lds_key[kHeadTile];     // the tile, read coalesced, handed out in runs of 8
  __shared__ u64 lds_pay[kHeadTile];
  __shared__ u32 lds_out[kHeadTile];     // the bagperm words going out
  if (REDO && ctx->n_evidence == 0) return;
  const KeyRange range = ctx->range;
  if (threadIdx.x == 0) s_tile = atomicAdd(ticket, 1u);
  __syncthreads();
  const u32 tile = s_tile;
  const u32 tile_base = tile * kHeadTile;
#pragma unroll
  for (int k = 0; k < kHeadItems; ++k) {
    const u32 p = k * kHeadThreads + threadIdx.x;
    const u32 j = tile_base + p;
    lds_key[p] = (j < n) ? skeys[j] : 0;
    lds_pay[p] = (j < n) ? spay[j] : 0;
  }
  __syncthreads();
  const u32 first = tile_base + threadIdx.x * kHeadItems;
  u64 key[kHeadItems];
  u32 idx[kHeadItems], bag[kHeadItems];
  bool head[kHeadItems];
  u64 prev = 0;
  if (first > 0 && first < n) prev = threadIdx.x ? lds_key[threadIdx.x * kHeadItems - 1] : skeys[first - 1];
  u32 heads = 0;
#pragma unroll
  for (int k = 0; k < kHeadItems; ++k) {
    key[k] = lds_key[threadIdx.x * kHeadItems + k];
    const u64 pay = lds_pay[threadIdx.x * kHeadItems + k];
    idx[k] = (u32)pay;
    // clamped: whatever the offsets said, the push must stay inside the gradient buffer
    bag[k] = min((u32)(pay >> 32), n_bags ? n_bags - 1 : 0u);
  }
#pragma unroll
  for (int k = 0; k < kHeadItems; ++k) {
    const u32 j = first + k;
    head[k] = (j < n) && (j == 0 || key[k] != prev);
    heads += head[k] ? 1u : 0u;
    if (!REDO && head[k] && j > 0 && sorted_prefix(key[k], range) == sorted_prefix(prev, range)) {
      const u32 slot = atomicAdd(&ctx->n_evidence, 1u);
      if (slot < kMaxEvidence) evidence[slot] = j;
    }
    prev = key[k];
  }
  u32 tile_heads;
  const u32 before = block_excl_sum<kHeadThreads>(heads, scratch, &tile_heads);
  if (threadIdx.x < kWave) {
    // Wave 0 publishes the tile's head count, then adds up the counts of the earlier
    // tiles of its group and of all earlier groups.
    const u32 lane = threadIdx.x;
    bool ok = true;
    if (lane == 0)
      __hip_atomic_store(head_rows + tile, status_word(epoch, tile_heads), __ATOMIC_RELAXED,
                         __HIP_MEMORY_SCOPE_AGENT);
    const u32 g = tile / group;
    u32 earlier = wave_sum_words(head_rows, g * group, tile, lane, epoch, &ok);
    if (tile % group == group - 1 && lane == 0)
      __hip_atomic_store(head_groups + g, status_word(epoch, earlier + tile_heads), __ATOMIC_RELAXED,
                         __HIP_MEMORY_SCOPE_AGENT);
    earlier += wave_sum_words(head_groups, 0, g, lane, epoch, &ok);
    if (!ok) ctx->sort_error = 1;
    if (lane == 0) {
      s_earlier = earlier;
      if ((u64)(tile + 1) * kHeadTile >= n) {     // the last tile knows U
        ctx->n_unique = earlier + tile_heads;
        seg_off[earlier + tile_heads] = n;
      }
    }
  }
  __syncthreads();
  u32 rank = s_earlier + before;   // heads before this thread's first position
#pragma unroll
  for (int k = 0; k < kHeadItems; ++k) {
    const u32 j = first + k;
    if (j < n) {
      if (head[k]) {
        uniq[rank] = key[k];
        seg_off[rank] = j;
        if (key[k] == kEmptyKey) raise_error(st, kErrReserved);
        ++rank;
      }
      lds_out[threadIdx.x * kHeadItems + k] = bag[k] | (head[k] ? 0x80000000u : 0u);
      inverse[idx[k]] = (i32)(rank - 1);
    }
  }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < kHeadItems; ++k) {
    const u32 p = k * kHeadThreads + threadIdx.x;
    if (tile_base + p < n) bagperm[tile_base + p] = lds_out[p];
  }
}

}  // namespace hps
