// Key dedup, the short way: two radix passes by bucket id, then every chunk of the
// array is finished inside one workgroup.
//
// After the passes (sort.cuh, by_id mode) the occurrences are ordered by bucket id:
// buckets of keys that share their leading bits (a few hundred occurrences each, in
// occurrence order) and, between them, one bucket per heavy key.  chunk_sort_emit
// cuts the array into regions at bucket borders (about kChunkSpan positions each; a
// heavy key's bucket may be cut anywhere, it holds one key), orders each region by
// full key in LDS -- stable, so equal keys keep their occurrence order -- and writes
// the dedup's outputs directly:
//   uniq[U]      ascending unique keys
//   inverse[N]   rank of each occurrence's key among them
//   bagperm[N]   bag of each occurrence, occurrences grouped by key, bit 31 on group heads
//   seg_off[U+1] start of each key's group in bagperm
// The number of unique keys in earlier regions comes from the grouped look-back over
// status words (sort.cuh).
//
// Which keys are heavy is a hint, taken from an earlier mini-batch (the lookup lists
// the keys that occurred often, the kernel after it puts them in order; common.cuh).  Hot keys of click
// logs persist from batch to batch, so the hint is nearly always right; when it is
// not (first batch, a new hot key) some region exceeds the LDS capacity and its
// workgroup orders it through global memory instead: slower, same result.
#pragma once

#include "common.cuh"
#include "sort.cuh"

namespace hps {

constexpr int kChunkThreads = 512;
constexpr int kChunkWaves = kChunkThreads / kWave;
constexpr int kChunkItems = 8;                                // per thread: regions of up to 4096 elements in LDS
constexpr u32 kChunkSpan = 2048;                              // positions between nominal cuts
constexpr u32 kNaturalBucket = 512;                           // mean size of a leading-bits bucket, at most
constexpr u32 kHeavyShare = 16384;                            // heavy: more than n / kHeavyShare occurrences
constexpr u32 kHeavyMin = 64;
constexpr int kSortBits = 32;
constexpr u32 kIndexMask = 0xFFFFFFu;   // payload: occurrence index in bits 0..23, bag in 32..63      // key bits a region is ordered by at first (all of them if that fails)

// ---- stable LSD radix sort of 64-bit words inside LDS --------------------------------
// Sorts words[0, cnt) by bits [first_bit, first_bit + 8 * n_pass).  cnt <= THREADS *
// ITEMS; the words up to the next multiple of THREADS are overwritten with all-ones.
// hist: two sets (used by alternate passes) of 256 * 8 16-bit counters, digit-major: the
// eight waves' counters of a digit are 16 consecutive bytes.  Three barriers per pass.
constexpr int kLdsSortHist = 2 * kRadix * 8;      // 16-bit words

template <int THREADS, int ITEMS>
__device__ __forceinline__ void lds_radix_sort(u64* words, u32 cnt, int first_bit, int n_pass,
                                               uint16_t* hist) {
  constexpr int WAVES = THREADS / kWave;
  static_assert(WAVES == 8, "a digit's counters are read as one 16-byte vector");
  const u32 tid = threadIdx.x, wave = tid / kWave, lane = tid & (kWave - 1);
  const u32 items = (cnt + THREADS - 1) / THREADS;     // rounds of the whole block
  const u32 padded = items * THREADS;
  for (u32 q = cnt + tid; q < padded; q += THREADS) words[q] = ~0ull;
  const u64 lt = lanemask_lt();
  const u32 wave_first = wave * kWave * items;          // a wave owns `items` runs of 64 words
  if (n_pass > 0 && tid < (u32)kRadix) reinterpret_cast<uint4*>(hist)[tid] = make_uint4(0, 0, 0, 0);
  __syncthreads();
  for (int pass = 0; pass < n_pass; ++pass) {
    const int bit = first_bit + 8 * pass;
    uint16_t* h = hist + (pass & 1) * (kRadix * WAVES);
    uint4* h4 = reinterpret_cast<uint4*>(h);             // [digit]: waves 0..7, 16 bits each
    u64 wd[ITEMS];
    u32 rank[ITEMS];
    // This wave's counter of digit d is the 16-bit word h[8 * d + wave]; the atomic works
    // on the 32-bit word it shares with the neighbouring wave's (counts stay below 2^16,
    // so nothing carries over).
    u32* pairs = reinterpret_cast<u32*>(h) + (wave >> 1);
    const int half = (wave & 1) * 16;
#pragma unroll
    for (int r = 0; r < ITEMS; ++r) {
      if ((u32)r < items) {
        wd[r] = words[wave_first + r * kWave + lane];
        const u32 d = (u32)(wd[r] >> bit) & (kRadix - 1);
        const u64 same = match_mask(d, true);
        const u32 before = __popcll(same & lt);
        u32 old = 0;
        if (before == 0) old = atomicAdd(pairs + (WAVES / 2) * d, (u32)__popcll(same) << half);
        old = __shfl(old, __ffsll((unsigned long long)same) - 1, kWave);
        rank[r] = ((old >> half) & 0xFFFFu) + before;
      }
    }
    __syncthreads();
    if (wave == 0) {
      // Lane l owns digits 4l .. 4l+3: per digit the waves' offsets inside the digit's run,
      // then (wave scan) the run's start, added to both 16-bit halves of a word at once
      // (all sums stay below 2^16, so nothing carries from one half into the other).
      uint4 c[4];
      u32 tot[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        c[q] = h4[4 * lane + q];
        u32 run = 0, v;
        v = c[q].x & 0xFFFFu; const u32 o0 = run; run += v;
        v = c[q].x >> 16;     const u32 o1 = run; run += v;
        v = c[q].y & 0xFFFFu; const u32 o2 = run; run += v;
        v = c[q].y >> 16;     const u32 o3 = run; run += v;
        v = c[q].z & 0xFFFFu; const u32 o4 = run; run += v;
        v = c[q].z >> 16;     const u32 o5 = run; run += v;
        v = c[q].w & 0xFFFFu; const u32 o6 = run; run += v;
        v = c[q].w >> 16;     const u32 o7 = run; run += v;
        c[q] = make_uint4(o0 | (o1 << 16), o2 | (o3 << 16), o4 | (o5 << 16), o6 | (o7 << 16));
        tot[q] = run;
      }
      const u32 mine = tot[0] + tot[1] + tot[2] + tot[3];
      u32 start = wave_incl_sum(mine) - mine;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const u32 both = start | (start << 16);
        h4[4 * lane + q] = make_uint4(c[q].x + both, c[q].y + both, c[q].z + both, c[q].w + both);
        start += tot[q];
      }
    } else if (wave == 1 || wave == 2 || wave == 3 || wave == 4) {
      // meanwhile: clear the other set of counters for the next pass
      uint4* other = reinterpret_cast<uint4*>(hist + ((pass + 1) & 1) * (kRadix * WAVES));
      other[tid - kWave] = make_uint4(0, 0, 0, 0);
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < ITEMS; ++r) {
      if ((u32)r < items) {
        const u32 d = (u32)(wd[r] >> bit) & (kRadix - 1);
        words[h[WAVES * d + wave] + rank[r]] = wd[r];
      }
    }
    __syncthreads();
  }
}

// ---- the slow way: a region too large for LDS ----------------------------------------
struct SlowLds {
  u32 hist[kRadix];
  u32 bin[kRadix];
  u32 wave_cnt[kChunkWaves][kRadix];
  u32 scratch[kChunkWaves + 1];
  u32 flag;
};

// One stable pass of the pairs in [a, b) from (ksrc, psrc) to (kdst, pdst) by the
// digit at `shift`.  Returns false, having moved nothing, if all digits are equal.
__device__ bool slow_radix_pass(const u64* ksrc, const u64* psrc, u64* kdst, u64* pdst, u32 a,
                                u32 b, int shift, SlowLds& L) {
  const u32 tid = threadIdx.x, wave = tid / kWave;
  const u64 lt = lanemask_lt();
  if (tid < (u32)kRadix) L.hist[tid] = 0;
  for (int w = tid; w < kChunkWaves * kRadix; w += kChunkThreads) (&L.wave_cnt[0][0])[w] = 0;
  if (tid == 0) L.flag = 0;
  __syncthreads();
  for (u32 j = a + tid; j < b; j += kChunkThreads) atomicAdd(&L.hist[key_digit(ksrc[j], shift)], 1u);
  __syncthreads();
  if (tid < (u32)kRadix && L.hist[tid] == b - a) L.flag = 1;
  u32 total;
  const u32 ex = block_excl_sum<kChunkThreads>(tid < (u32)kRadix ? L.hist[tid] : 0, L.scratch, &total);
  if (L.flag) return false;        // written before the scan's barriers
  if (tid < (u32)kRadix) L.bin[tid] = a + ex;
  __syncthreads();
  for (u32 base = a; base < b; base += kChunkThreads) {
    const u32 j = base + tid;
    const bool valid = j < b;
    const u64 key = valid ? ksrc[j] : 0;
    const u64 pay = valid ? psrc[j] : 0;
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
    if (valid) { kdst[dest] = key; pdst[dest] = pay; }
    __syncthreads();
  }
  return true;
}

// Orders the pairs in [a, b) of (skeys, spay) by full key, equal keys keeping their
// order, WITHOUT writing to (skeys, spay): other workgroups read them meanwhile.  The
// passes alternate between two scratch arrays of the same shape; *kres / *pres tell
// where the result is (the source itself if all keys were equal).
__device__ void slow_sort_region(const u64* skeys, const u64* spay, u64* ka, u64* pa, u64* kb,
                                 u64* pb, u32 a, u32 b, SlowLds& L, const u64** kres,
                                 const u64** pres) {
  const u64 *kc = skeys, *pc = spay;
  u64 *kd = ka, *pd = pa;
  for (int shift = 0; shift < 64; shift += kRadixBits) {
    if (slow_radix_pass(kc, pc, kd, pd, a, b, shift, L)) {
      kc = kd; pc = pd;
      kd = kd == ka ? kb : ka;
      pd = pd == pa ? pb : pa;
    }
    __syncthreads();
  }
  *kres = kc;
  *pres = pc;
}

// ---- regions ---------------------------------------------------------------------------
// A region may start where the bucket id changes, or anywhere inside a heavy key's
// bucket.  border(p0) = the first such position >= p0, n if there is none; region c is
// [border(c * kChunkSpan), border((c + 1) * kChunkSpan)), border(0) = 0.  Both borders
// are looked for at once, half the block each, kBorderWindow positions per round.
constexpr u32 kBorderWindow = kChunkThreads;     // positions per border per round

__device__ __forceinline__ bool is_border(const u64* __restrict__ skeys, u32 p, u32 p0,
                                          const HeavyLds& hv) {
  bool heavy, heavy_prev;
  const u32 id = bucket_id(skeys[p], hv, &heavy);
  const u32 id_prev = bucket_id(skeys[p - 1], hv, &heavy_prev);
  return id != id_prev || (p == p0 && heavy);
}

// s_border[0] / [1] (LDS) must hold ~0u for a border still to be found, else its value.
__device__ void find_borders(const u64* __restrict__ skeys, u32 n, u32 p0_lo, u32 p0_hi,
                             const HeavyLds& hv, u32* s_border) {
  const u32 half = threadIdx.x / (kChunkThreads / 2);          // which border this thread serves
  const u32 t = threadIdx.x % (kChunkThreads / 2);
  const u32 p0 = half ? p0_hi : p0_lo;
  for (u32 round = 0;; ++round) {
    const bool open = s_border[half] == ~0u;
    __syncthreads();
    if (open) {
#pragma unroll
      for (int k = 0; k < 2; ++k) {
        const u32 p = p0 + round * kBorderWindow + k * (kChunkThreads / 2) + t;
        if (p < n && is_border(skeys, p, p0, hv)) atomicMin(&s_border[half], p);
      }
    }
    __syncthreads();
    bool done = true;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const u32 q0 = h ? p0_hi : p0_lo;
      if (s_border[h] == ~0u) {
        if ((u64)q0 + (u64)(round + 1) * kBorderWindow >= n) {
          __syncthreads();                 // every thread has read the ~0u
          if (threadIdx.x == 0) s_border[h] = n;
          __syncthreads();
        } else {
          done = false;
        }
      }
    }
    if (done) break;
  }
  __syncthreads();
}

template <int ITEMS>
struct ChunkLds {
  union {
    u64 words[kChunkThreads * ITEMS];
    u32 out[kChunkThreads * ITEMS];
    SlowLds slow;
  };
  uint16_t hist[kLdsSortHist];
  HeavyLds hv;
  u32 scratch[kChunkWaves + 1];
  u32 s_chunk, s_earlier, s_flag;
  u32 s_border[2];
  unsigned long long s_or;
};

// Cross-region head counts (grouped status words, sort.cuh).  A region publishes its
// number of group heads as soon as it knows it; the last region of a group then also
// publishes the group's total.  Wave 0 only; the other waves go on.
__device__ __forceinline__ void publish_heads(u32 chunk, u32 heads, u32 group, u32 epoch,
                                              u32* head_rows, u32* head_groups, PullCtx* ctx) {
  if (threadIdx.x >= kWave) return;
  const u32 lane = threadIdx.x;
  if (lane == 0)
    __hip_atomic_store(head_rows + chunk, status_word(epoch, heads), __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
  if (chunk % group == group - 1) {
    bool ok = true;
    const u32 g = chunk / group;
    const u32 earlier = wave_sum_words(head_rows, g * group, chunk, lane, epoch, &ok);
    if (lane == 0)
      __hip_atomic_store(head_groups + g, status_word(epoch, earlier + heads), __ATOMIC_RELAXED,
                         __HIP_MEMORY_SCOPE_AGENT);
    if (!ok) ctx->sort_error = 1;
  }
}

// The number of heads in earlier regions, to all threads (contains a barrier).
__device__ __forceinline__ u32 heads_before(u32* s_earlier, u32 chunk, u32 group, u32 epoch,
                                            const u32* head_rows, const u32* head_groups,
                                            PullCtx* ctx) {
  if (threadIdx.x < kWave) {
    const u32 lane = threadIdx.x;
    bool ok = true;
    const u32 g = chunk / group;
    u32 earlier = wave_sum_words(head_rows, g * group, chunk, lane, epoch, &ok);
    earlier += wave_sum_words(head_groups, 0, g, lane, epoch, &ok);
    if (!ok) ctx->sort_error = 1;
    if (lane == 0) *s_earlier = earlier;
  }
  __syncthreads();
  return *s_earlier;
}

// Number of distinct keys among the thread block's keys (key[r] valid for r < items and
// r * THREADS + tid < cnt), counted with a hash set of `slots` 64-bit words in LDS.
// Contains barriers; `table` is free again afterwards.
template <int ITEMS>
__device__ __forceinline__ u32 count_distinct(const u64* key, u32 items, u32 cnt, u64* table,
                                              u32* scratch) {
  constexpr int kChunkItems = ITEMS;
  constexpr u32 kCountSlots = kChunkThreads * ITEMS;
  const u32 tid = threadIdx.x;
#pragma unroll
  for (int r = 0; r < kChunkItems; ++r) table[r * kChunkThreads + tid] = ~0ull;
  __syncthreads();
  u32 fresh = 0;
#pragma unroll
  for (int r = 0; r < kChunkItems; ++r) {
    const u32 p = r * kChunkThreads + tid;
    if ((u32)r < items && p < cnt && key[r] != ~0ull) {
      const u64 k = key[r];
      // the keys of a region share their leading bits: hash the low half
      u32 slot = (u32)(((u64)((u32)k * 0x9E3779B1u) * kCountSlots) >> 32);
      for (u32 step = 0; step < kCountSlots; ++step) {
        unsigned long long* cell = reinterpret_cast<unsigned long long*>(table + slot);
        u64 seen = *reinterpret_cast<volatile u64*>(cell);
        if (seen == ~0ull) seen = atomicCAS(cell, ~0ull, (unsigned long long)k);
        if (seen == ~0ull) { ++fresh; break; }
        if (seen == k) break;
        slot = slot + 1 == kCountSlots ? 0 : slot + 1;
      }
    }
  }
  u32 total;
  (void)block_excl_sum<kChunkThreads>(fresh, scratch, &total);
  __syncthreads();
  return total;
}

// A whole region the slow way: ordered in global memory, then walked.  Kept out of line
// so that its registers do not weigh on the usual path.
__device__ __forceinline__ void slow_region(const u64* skeys, const u64* spay, u64* ka, u64* pa, u64* kb,
                                         u64* pb, u32 n, u32 start, u32 end, u32 chunk, bool last,
                                         SlowLds& slow, u32* scratch, u32* s_earlier, u32* head_rows,
                                         u32* head_groups, u32 group, u32 epoch, u32 n_bags, u64* uniq,
                                         i32* inverse, u32* bagperm, u32* seg_off, PullCtx* ctx,
                                         TableState* st) {
  const u32 tid = threadIdx.x;
  const u64 *sk, *sp;
  slow_sort_region(skeys, spay, ka, pa, kb, pb, start, end, slow, &sk, &sp);
  if (tid == 0) {
    // For the host's choice of the next dedups' form: how much went this way, and how much
    // of that because ONE key fills the region (then the sorted region's middle element is
    // that key: count it) -- a key that turned frequent without warning, which the next
    // hint will list, and not keys that do not suit the buckets.
    const u64 mid_key = sk[start + (end - start) / 2];
    u32 lo = start, hi = end;
    while (lo < hi) { const u32 m = lo + (hi - lo) / 2; if (sk[m] < mid_key) lo = m + 1; else hi = m; }
    const u32 first = lo;
    hi = end;
    while (lo < hi) { const u32 m = lo + (hi - lo) / 2; if (sk[m] <= mid_key) lo = m + 1; else hi = m; }
    atomicAdd(&ctx->n_slow, end - start);
    if ((lo - first) * 2 >= end - start) atomicAdd(&ctx->n_slow_one_key, end - start);
  }
  // the element before the region is read from the untouched source
  const bool first_is_head = start == 0 || sk[start] != skeys[start - 1];
  u32 heads = 0;
  for (u32 j = start + tid; j < end; j += kChunkThreads)
    heads += (j == start ? first_is_head : sk[j] != sk[j - 1]) ? 1u : 0u;
  u32 total;
  (void)block_excl_sum<kChunkThreads>(heads, scratch, &total);
  publish_heads(chunk, total, group, epoch, head_rows, head_groups, ctx);
  u32 rank = heads_before(s_earlier, chunk, group, epoch, head_rows, head_groups, ctx);
  if (last && tid == 0) { ctx->n_unique = rank + total; seg_off[rank + total] = n; }
  for (u32 base = start; base < end; base += kChunkThreads) {
    const u32 j = base + tid;
    const bool valid = j < end;
    const u64 key = valid ? sk[j] : 0;
    const bool head = valid && (j == start ? first_is_head : key != sk[j - 1]);
    u32 tile_heads;
    const u32 before = block_excl_sum<kChunkThreads>(head ? 1u : 0u, scratch, &tile_heads);
    if (valid) {
      const u32 r = rank + before + (head ? 1u : 0u) - 1;   // rank of this occurrence's key
      const u64 pay = sp[j];
      if (head) {
        uniq[r] = key;
        seg_off[r] = j;
        if (key == kEmptyKey) raise_error(st, kErrReserved);
      }
      inverse[(u32)pay & kIndexMask] = (i32)r;
      bagperm[j] = min((u32)(pay >> 32), n_bags - 1) | (head ? 0x80000000u : 0u);
    }
    rank += tile_heads;
  }
}

// Two keys of the region agreed in the bits [lo, hb) it was ordered by without being
// equal: order by the bits below lo first, then (stable) by the bits above, so that all
// 64 bits count.  Rare; out of line.
template <int ITEMS>
__device__ __forceinline__ void resort_all_bits(u64* words, uint16_t* hist, const u64* skeys, u32 start,
                                             u32 cnt, int lo, u64 bit_mask, int top_pass) {
  const u32 tid = threadIdx.x;
  const u32 items = (cnt + kChunkThreads - 1) / kChunkThreads;
#pragma unroll
  for (int r = 0; r < ITEMS; ++r) {
    const u32 p = r * kChunkThreads + tid;
    if ((u32)r < items && p < cnt) words[p] = ((skeys[start + p] & ((1ull << lo) - 1)) << 16) | p;
  }
  __syncthreads();
  lds_radix_sort<kChunkThreads, ITEMS>(words, cnt, 16, (lo + 7) / 8, hist);
#pragma unroll
  for (int r = 0; r < ITEMS; ++r) {
    const u32 q = r * kChunkThreads + tid;
    if ((u32)r < items && q < cnt) {
      const u32 p = (u32)words[q] & 0xFFFFu;
      words[q] = (((skeys[start + p] >> lo) & bit_mask) << 16) | p;
    }
  }
  __syncthreads();
  lds_radix_sort<kChunkThreads, ITEMS>(words, cnt, 16, top_pass, hist);
}

// skeys/spay: the pairs ordered by bucket id (payload = occurrence index | bag << 32),
// read only; ka/pa and kb/pb: scratch of the same shape (only touched the slow way).
template <int ITEMS>
__global__ void __launch_bounds__(kChunkThreads, 4)
chunk_sort_emit(const u64* __restrict__ skeys, const u64* __restrict__ spay, u64* __restrict__ ka,
                u64* __restrict__ pa, u64* __restrict__ kb, u64* __restrict__ pb, u32 n,
                u32 max_heavy,
                const HeavySet* __restrict__ heavy_set, u32* __restrict__ head_rows,
                u32* __restrict__ head_groups, u32 group, u32* __restrict__ ticket, u32 epoch,
                u32 n_bags, u64* __restrict__ uniq, i32* __restrict__ inverse,
                u32* __restrict__ bagperm, u32* __restrict__ seg_off, PullCtx* __restrict__ ctx,
                TableState* __restrict__ st) {
  constexpr int kChunkItems = ITEMS;
  constexpr u32 kChunkCap = kChunkThreads * ITEMS;
  constexpr u32 kCountMax = kChunkCap * 3 / 4;      // beyond this the table of the distinct count is too full
  __shared__ ChunkLds<ITEMS> L;
  const u32 tid = threadIdx.x;
  if (tid == 0) L.s_chunk = atomicAdd(ticket, 1u);
  load_heavy(L.hv, heavy_set, max_heavy);
  if (tid == 0) L.hv.range = ctx->range;
  __syncthreads();
  const u32 chunk = L.s_chunk;
  const u32 n_chunks = (n + kChunkSpan - 1) / kChunkSpan;
  const bool last = chunk + 1 == n_chunks;
  if (tid == 0) {
    L.s_border[0] = chunk == 0 ? 0u : ~0u;
    L.s_border[1] = last ? n : ~0u;
    L.s_or = 0;
  }
  __syncthreads();
  find_borders(skeys, n, chunk * kChunkSpan, (chunk + 1) * kChunkSpan, L.hv, L.s_border);
  const u32 start = L.s_border[0], end = L.s_border[1];
  const u32 cnt = end - start;       // start <= end: both borders come from the same rule

  if (cnt > kChunkCap) {
    slow_region(skeys, spay, ka, pa, kb, pb, n, start, end, chunk, last, L.slow, L.scratch, &L.s_earlier,
                head_rows, head_groups, group, epoch, n_bags, uniq, inverse, bagperm, seg_off, ctx, st);
    return;
  }

  // ---- the usual way: order the region in LDS ----
  const u32 items = (cnt + kChunkThreads - 1) / kChunkThreads;
  const u64 key0 = cnt ? skeys[start] : 0;
  u64 key[kChunkItems], pay[kChunkItems];
  {
    // which key bits vary inside the region
    u64 diff = 0;
#pragma unroll
    for (int r = 0; r < kChunkItems; ++r) {
      const u32 p = r * kChunkThreads + tid;
      key[r] = ((u32)r < items && p < cnt) ? skeys[start + p] : key0;
      diff |= key[r] ^ key0;
    }
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) diff |= __shfl_xor(diff, d, kWave);
    if ((tid & (kWave - 1)) == 0 && diff) atomicOr(&L.s_or, (unsigned long long)diff);
  }
  __syncthreads();
  const u64 vary = L.s_or;
  const int hb = vary ? 64 - __clzll((long long)vary) : 0;    // bits [hb, 64) are the same in all keys
  const int lo = hb > kSortBits ? hb - kSortBits : 0;         // the sort takes bits [lo, hb)
  const int n_bits = hb - lo;
  const u64 bit_mask = (1ull << n_bits) - 1;                  // bits above hb are dropped: all equal
  const int top_pass = (n_bits + 7) / 8;
  // The number of group heads is published before the sort, so that no later region has
  // to wait for this one's sort: it is the number of distinct keys, less one if the
  // region starts inside a heavy key's bucket whose earlier part belongs to the region before.
  const bool first_continues = cnt && start > 0 && skeys[start - 1] == key0;
  if (hb == 0) {
    // One key only (part of a heavy key's bucket, typically), or nothing: the region is
    // in order as it stands, its pairs are read in place.
    const u32 n_heads = cnt && !first_continues ? 1u : 0u;
    publish_heads(chunk, n_heads, group, epoch, head_rows, head_groups, ctx);
    const u32 earlier = heads_before(&L.s_earlier, chunk, group, epoch, head_rows, head_groups, ctx);
    if (last && tid == 0) { ctx->n_unique = earlier + n_heads; seg_off[earlier + n_heads] = n; }
    const u32 rank = earlier + n_heads - 1;      // of the key (cnt > 0: earlier + n_heads >= 1)
    if (n_heads && tid == 0) {
      uniq[rank] = key0;
      seg_off[rank] = start;
      if (key0 == kEmptyKey) raise_error(st, kErrReserved);
    }
#pragma unroll
    for (int r = 0; r < kChunkItems; ++r) {
      const u32 p = r * kChunkThreads + tid;
      if ((u32)r < items && p < cnt) {
        const u64 pay = spay[start + p];
        bagperm[start + p] = min((u32)(pay >> 32), n_bags - 1) | (p == 0 && n_heads ? 0x80000000u : 0u);
        inverse[(u32)pay & kIndexMask] = (i32)rank;
      }
    }
    return;
  }
  const bool early = cnt <= kCountMax;
  u32 n_heads = 0;
  if (early) {
    const u32 distinct = count_distinct<ITEMS>(key, items, cnt, L.words, L.scratch);
    n_heads = distinct - (first_continues ? 1u : 0u);
    publish_heads(chunk, n_heads, group, epoch, head_rows, head_groups, ctx);
  }

  u64 prev_key = 0;
  const u32 j0 = tid * items;          // this thread's run of sorted positions
  bool mixed = false;
  for (int attempt = 0; attempt < 2; ++attempt) {
    if (attempt == 0) {
#pragma unroll
      for (int r = 0; r < kChunkItems; ++r) {
        const u32 p = r * kChunkThreads + tid;
        key[r] = (((key[r] >> lo) & bit_mask) << 16) | p;     // from here on: the word
      }
      __syncthreads();       // the words replace the table of the distinct count
#pragma unroll
      for (int r = 0; r < kChunkItems; ++r) {
        const u32 p = r * kChunkThreads + tid;
        if ((u32)r < items && p < cnt) L.words[p] = key[r];
      }
      __syncthreads();
      lds_radix_sort<kChunkThreads, kChunkItems>(L.words, cnt, 16, top_pass, L.hist);
    } else {
      resort_all_bits<ITEMS>(L.words, L.hist, skeys, start, cnt, lo, bit_mask, top_pass);
    }
    // sorted position j0 + k -> its pair
    u64 prev_word = ~0ull;
    if (j0 > 0 && j0 < cnt) {
      prev_word = L.words[j0 - 1];
      prev_key = skeys[start + ((u32)prev_word & 0xFFFFu)];
    } else if (j0 == 0 && start > 0 && cnt) {
      prev_key = skeys[start - 1];
    }
    bool bad = false;
#pragma unroll
    for (int k = 0; k < kChunkItems; ++k) {
      const u32 j = j0 + k;
      if ((u32)k < items && j < cnt) {
        const u64 w = L.words[j];
        const u32 p = (u32)w & 0xFFFFu;
        key[k] = skeys[start + p];
        pay[k] = spay[start + p];
        const u64 pk = k ? key[k - 1] : prev_key;
        const u64 pw = k ? L.words[j - 1] : prev_word;
        if (j > 0 && (pw >> 16) == (w >> 16) && pk != key[k]) bad = true;
      }
    }
    mixed = __syncthreads_or(bad && lo > 0 && attempt == 0);
    if (!mixed) break;
  }

  bool head[kChunkItems];
  u32 heads = 0;
#pragma unroll
  for (int k = 0; k < kChunkItems; ++k) {
    const u32 j = j0 + k;
    head[k] = false;
    if ((u32)k < items && j < cnt) {
      const u64 pk = k ? key[k - 1] : prev_key;
      head[k] = (start + j == 0) || key[k] != pk;
      heads += head[k] ? 1u : 0u;
    }
  }
  // the bags, back in sorted order (does not need the ranks: before the wait below)
  __syncthreads();        // every thread has read its words: L.out may overwrite them
#pragma unroll
  for (int k = 0; k < kChunkItems; ++k) {
    const u32 j = j0 + k;
    // clamped: whatever the offsets said, the push must stay inside the gradient buffer
    if ((u32)k < items && j < cnt)
      L.out[j] = min((u32)(pay[k] >> 32), n_bags - 1) | (head[k] ? 0x80000000u : 0u);
  }
  __syncthreads();
#pragma unroll
  for (int r = 0; r < kChunkItems; ++r) {
    const u32 p = r * kChunkThreads + tid;
    if ((u32)r < items && p < cnt) bagperm[start + p] = L.out[p];
  }
  u32 total;
  const u32 before = block_excl_sum<kChunkThreads>(heads, L.scratch, &total);
  if (early && total != n_heads && tid == 0) ctx->sort_error = 1;     // never expected
  if (!early) publish_heads(chunk, total, group, epoch, head_rows, head_groups, ctx);
  const u32 earlier = heads_before(&L.s_earlier, chunk, group, epoch, head_rows, head_groups, ctx);
  if (last && tid == 0) { ctx->n_unique = earlier + total; seg_off[earlier + total] = n; }
  u32 rank = earlier + before;         // heads before this thread's first position
#pragma unroll
  for (int k = 0; k < kChunkItems; ++k) {
    const u32 j = j0 + k;
    if ((u32)k < items && j < cnt) {
      if (head[k]) {
        uniq[rank] = key[k];
        seg_off[rank] = start + j;
        if (key[k] == kEmptyKey) raise_error(st, kErrReserved);
        ++rank;
      }
      inverse[(u32)pay[k] & kIndexMask] = (i32)(rank - 1);
    }
  }
}

}  // namespace hps
