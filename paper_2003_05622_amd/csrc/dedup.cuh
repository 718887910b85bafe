// Key dedup, part 2: from the elements sorted by their top bits to
//   uniq[U]      ascending unique keys
//   inverse[N]   rank of each occurrence's key among them
//   perm[N]      occurrence indices grouped by key (ascending key)
//   seg_off[U+1] start of each key's group in perm
//
//   detect_mixed_runs  reads every sorted occurrence's full key (skeys) and records
//                      the positions where two neighbours agree in the sorted bits
//                      but are different keys ("evidence" of a mixed run);
//   fix_mixed_runs     one workgroup; does nothing when there is no evidence (the
//                      normal case for hashed keys); otherwise orders every mixed run
//                      by full key -- runs of up to 64 elements inside one wave,
//                      longer ones (or, with too much evidence, the whole array) by
//                      a workgroup-local radix sort through global memory;
//   unique_emit        group heads, their running count across tiles by decoupled
//                      look-back, and all outputs.
#pragma once

#include "common.cuh"
#include "sort.cuh"

namespace hps {

constexpr int kHeadThreads = 256;
constexpr int kHeadItems = 8;
constexpr int kHeadTile = kHeadThreads * kHeadItems;
constexpr u32 kMaxEvidence = 1024;
constexpr int kFixThreads = 1024;
constexpr int kFixWaves = kFixThreads / kWave;

__global__ void __launch_bounds__(kHeadThreads)
detect_mixed_runs(const u64* __restrict__ elems, const u64* __restrict__ keys, u32 n,
                  SortPlan plan, u64* __restrict__ skeys, PullCtx* __restrict__ ctx,
                  u32* __restrict__ evidence) {
  const u32 first = blockIdx.x * kHeadTile + threadIdx.x * kHeadItems;
  if (first >= n) return;
  u64 prev_e = 0, prev_key = 0;
  if (first > 0) {
    prev_e = elems[first - 1];
    prev_key = keys[elem_idx(prev_e, plan.idx_bits)];
  }
  u64 e[kHeadItems], key[kHeadItems];
#pragma unroll
  for (int k = 0; k < kHeadItems; ++k) {
    const u32 j = first + k;
    e[k] = (j < n) ? elems[j] : 0;
  }
#pragma unroll
  for (int k = 0; k < kHeadItems; ++k) {
    const u32 j = first + k;
    key[k] = (j < n) ? keys[elem_idx(e[k], plan.idx_bits)] : 0;
  }
#pragma unroll
  for (int k = 0; k < kHeadItems; ++k) {
    const u32 j = first + k;
    if (j < n) {
      skeys[j] = key[k];
      if (j > 0 && key[k] != prev_key && (e[k] >> plan.low_shift) == (prev_e >> plan.low_shift)) {
        const u32 slot = atomicAdd(&ctx->n_evidence, 1u);
        if (slot < kMaxEvidence) evidence[slot] = j;
      }
      prev_e = e[k];
      prev_key = key[k];
    }
  }
}

// ---- workgroup-local (one block of kFixThreads) stable radix sort of elems[a, b) by
// ---- the full 64-bit key, through global memory.  Slow; for rare inputs only.

struct FixLds {
  u32 hist[kRadix];
  u32 bin[kRadix];
  u32 wave_cnt[kFixWaves][kRadix];
  u32 scratch[kFixThreads / kWave + 1];
};

// One pass over words (sort word << 32 | idx) in src[a, b) -> dst[a, b).
__device__ void wg_radix_pass(const u64* src, u64* dst, u32 a, u32 b, int shift, FixLds& L) {
  const u32 tid = threadIdx.x, wave = tid / kWave;
  const u64 lt = lanemask_lt();
  if (tid < kRadix) L.hist[tid] = 0;
  __syncthreads();
  for (u32 j = a + tid; j < b; j += kFixThreads) atomicAdd(&L.hist[(u32)(src[j] >> (32 + shift)) & 255u], 1u);
  __syncthreads();
  u32 total;
  const u32 ex = block_excl_sum<kFixThreads>(tid < kRadix ? L.hist[tid] : 0, L.scratch, &total);
  if (tid < kRadix) L.bin[tid] = a + ex;
  __syncthreads();
  for (u32 base = a; base < b; base += kFixThreads) {
    const u32 j = base + tid;
    const bool valid = j < b;
    const u64 e = valid ? src[j] : 0;
    const u32 d = (u32)(e >> (32 + shift)) & 255u;
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
    if (valid) dst[dest] = e;
    __syncthreads();
  }
}

// Orders elems[a, b) (and skeys) by full key; equal keys keep their order.
__device__ void wg_sort_range_full(u64* elems, u64* alt, u64* skeys, const u64* keys, u32 a, u32 b,
                                   int idx_bits, FixLds& L) {
  const u32 tid = threadIdx.x;
  for (int w = tid; w < kFixWaves * kRadix; w += kFixThreads) (&L.wave_cnt[0][0])[w] = 0;
  // Two stable 32-bit sorts: by the key's low half, then by its high half.  Elements
  // with equal keys keep their current relative order.
  for (int half = 0; half < 2; ++half) {
    __syncthreads();
    for (u32 j = a + tid; j < b; j += kFixThreads) {
      const u32 idx = half == 0 ? elem_idx(elems[j], idx_bits) : (u32)elems[j];
      const u64 key = keys[idx];
      elems[j] = ((u64)(half == 0 ? (u32)key : (u32)(key >> 32)) << 32) | idx;
    }
    __syncthreads();
    for (int shift = 0; shift < 32; shift += kRadixBits) {
      wg_radix_pass(elems, alt, a, b, shift, L);
      u64* t = elems; elems = alt; alt = t;
    }
  }
  __syncthreads();
  for (u32 j = a + tid; j < b; j += kFixThreads) {
    const u32 idx = (u32)elems[j];
    const u64 key = keys[idx];
    elems[j] = make_elem(key, idx, idx_bits);
    skeys[j] = key;
  }
  __syncthreads();
}

__global__ void __launch_bounds__(kFixThreads)
fix_mixed_runs(u64* __restrict__ elems, u64* __restrict__ alt, u64* __restrict__ skeys,
               const u64* __restrict__ keys, u32 n, SortPlan plan, PullCtx* __restrict__ ctx,
               const u32* __restrict__ evidence) {
  const u32 E = ctx->n_evidence;
  if (E == 0) return;
  __shared__ FixLds L;
  __shared__ u32 ev[kMaxEvidence];
  __shared__ u32 run_lo[kMaxEvidence];
  __shared__ u32 run_hi[kMaxEvidence];
  const u32 tid = threadIdx.x;
  if (E > kMaxEvidence) {
    wg_sort_range_full(elems, alt, skeys, keys, 0, n, plan.idx_bits, L);
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
    const u64 v = elems[j] >> plan.low_shift;
    u32 lo = 0, hi = j;                       // first position with top bits >= v
    while (lo < hi) {
      const u32 mid = lo + (hi - lo) / 2;
      if ((elems[mid] >> plan.low_shift) < v) lo = mid + 1; else hi = mid;
    }
    const u32 a = lo;
    lo = j; hi = n;                           // first position with top bits > v
    while (lo < hi) {
      const u32 mid = lo + (hi - lo) / 2;
      if ((elems[mid] >> plan.low_shift) <= v) lo = mid + 1; else hi = mid;
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
    u64 e = 0, key = 0;
    u32 idx = 0;
    if (lane < len) {
      e = elems[a + lane];
      idx = elem_idx(e, plan.idx_bits);
      key = keys[idx];
    }
    u32 rank = 0;
    for (u32 m = 0; m < len; ++m) {
      const u64 okey = __shfl(key, (int)m, kWave);
      const u32 oidx = __shfl(idx, (int)m, kWave);
      rank += (okey < key || (okey == key && oidx < idx)) ? 1u : 0u;
    }
    if (lane < len) {
      elems[a + rank] = e;
      skeys[a + rank] = key;
    }
  }
  __syncthreads();
  // long runs: the whole workgroup, one run after the other
  for (u32 r = 0; r < E; ++r) {
    const u32 a = run_lo[r], b = run_hi[r];
    if (b - a > (u32)kWave) wg_sort_range_full(elems, alt, skeys, keys, a, b, plan.idx_bits, L);
  }
}

// Heads of the key groups, their ranks, and every output of the dedup.
//   head_state [n_tiles] look-back status words (see sort.cuh), ticket: tile tickets
__global__ void __launch_bounds__(kHeadThreads)
unique_emit(const u64* __restrict__ elems, const u64* __restrict__ skeys, u32 n, int idx_bits,
            u64* __restrict__ head_state, u32* __restrict__ ticket, u32 epoch,
            u64* __restrict__ uniq, i32* __restrict__ inverse, u32* __restrict__ perm,
            u32* __restrict__ seg_off, PullCtx* __restrict__ ctx, TableState* __restrict__ st) {
  __shared__ u32 scratch[kHeadThreads / kWave + 1];
  __shared__ u32 s_tile, s_earlier;
  if (threadIdx.x == 0) s_tile = atomicAdd(ticket, 1u);
  __syncthreads();
  const u32 tile = s_tile;
  const u32 first = tile * kHeadTile + threadIdx.x * kHeadItems;
  u64 key[kHeadItems];
  bool head[kHeadItems];
  u64 prev = 0;
  if (first > 0 && first < n) prev = skeys[first - 1];
  u32 heads = 0;
#pragma unroll
  for (int k = 0; k < kHeadItems; ++k) {
    const u32 j = first + k;
    key[k] = (j < n) ? skeys[j] : 0;
    head[k] = (j < n) && (j == 0 || key[k] != prev);
    heads += head[k] ? 1u : 0u;
    prev = key[k];
  }
  u32 tile_heads;
  const u32 before = block_excl_sum<kHeadThreads>(heads, scratch, &tile_heads);
  if (threadIdx.x == 0) {
    u32 earlier = 0;
    if (tile == 0) {
      __hip_atomic_store(head_state, state_word(epoch, kFlagInclusive, tile_heads),
                         __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    } else {
      __hip_atomic_store(head_state + tile, state_word(epoch, kFlagAggregate, tile_heads),
                         __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      u32 p = tile - 1, spins = 0;
      while (true) {
        const u64 w = __hip_atomic_load(head_state + p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const u64 flag = (w >> 32) & 3;
        if ((u32)(w >> 34) != epoch || flag == 0) {
          if (++spins > kSpinLimit) { ctx->sort_error = 1; break; }   // never expected
          __builtin_amdgcn_s_sleep(1);
          continue;
        }
        earlier += (u32)w;
        if (flag == kFlagInclusive || p == 0) break;
        --p;
      }
      __hip_atomic_store(head_state + tile, state_word(epoch, kFlagInclusive, earlier + tile_heads),
                         __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    s_earlier = earlier;
    if ((u64)(tile + 1) * kHeadTile >= n) {     // the last tile knows U
      ctx->n_unique = earlier + tile_heads;
      seg_off[earlier + tile_heads] = n;
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
      const u32 idx = elem_idx(elems[j], idx_bits);
      perm[j] = idx;
      inverse[idx] = (i32)(rank - 1);
    }
  }
}

}  // namespace hps
