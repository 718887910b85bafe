// Key dedup, bucket form, part 2: every region of the array is finished inside one workgroup.
//
// After the partition (partition.hpp) the occurrences are ordered by bucket id: buckets of
// keys that share their place in the key range (a few hundred occurrences each, in
// occurrence order) and, between them, one bucket per heavy key.  region_borders has cut the
// array into regions at bucket borders (about kChunkSpan positions each; a heavy key's bucket
// may be cut anywhere, it holds one key).  Two launches, neither waits for another workgroup:
//   region_sort   orders each region by full key in LDS -- stable, so equal keys keep their
//                 occurrence order -- and leaves, per region, the order (one word per
//                 position), how many group heads (distinct keys) it holds, and how it was
//                 ordered; per group of 64 regions, the heads of the group;
//   region_emit   adds up the heads of earlier groups and regions and writes the dedup's
//                 outputs:
//   uniq[U]      ascending unique keys
//   inverse[N]   rank of each occurrence's key among them
//   bagperm[N]   bag of each occurrence, occurrences grouped by key, bit 31 on group heads
//   seg_off[U+1] start of each key's group in bagperm
//
// Which keys are heavy is a hint, taken from an earlier mini-batch (the lookup lists
// the keys that occurred often, the kernel after it puts them in order; common.hpp).  Hot keys of click
// logs persist from batch to batch, so the hint is nearly always right; when it is
// not (first batch, a new hot key) some region exceeds the LDS capacity and its
// workgroup orders it through global memory instead: slower, same result.
#pragma once

#include "common.hpp"
#include "sort.hpp"
#include "partition.hpp"

namespace hps {

constexpr int kChunkThreads = 512;
constexpr int kChunkWaves = kChunkThreads / kWave;
constexpr int kChunkItems = 8;                                // per thread: regions of up to 4096 elements in LDS
constexpr u32 kChunkSpan = kRegionSpan;                       // positions between nominal cuts
constexpr u32 kNaturalBucket = 512;                           // mean size of a leading-bits bucket, at most
constexpr u32 kHeavyShare = 16384;                            // heavy: more than n / kHeavyShare occurrences
constexpr u32 kHeavyMin = 64;
constexpr int kSortBits = 32;           // key bits a region is ordered by at first (all of them if that fails)

// ---- stable LSD radix sort of 64-bit words inside LDS --------------------------------
// Sorts words[0, cnt) by bits [first_bit, first_bit + 8 * n_pass) (all below bit 48: a word's
// upper 16 bits must be zero and come back zero).  cnt <= THREADS *
// ITEMS, and `words` has room for THREADS * ITEMS words: the words from cnt up to the next
// multiple of THREADS are overwritten with all-ones, and whatever lies behind them may be
// overwritten with anything.
// hist: two sets (used by alternate passes) of 256 * 8 16-bit counters, digit-major: the
// eight waves' counters of a digit are 16 consecutive bytes.  Three barriers per pass.
//
// Every thread goes through ITEMS rounds without a branch (ITEMS >= the rounds cnt needs;
// lds_radix_sort_any picks the instance), so that the LDS operations of a pass are issued
// back to back instead of each waiting for the one before: a round behind the last one reads
// whatever is there, adds zero to a counter and writes into the unused tail of `words`
// (which therefore has to hold THREADS * (ITEMS + 1) words, or THREADS * ITEMS if cnt needs
// all ITEMS rounds).
constexpr int kLdsSortHist = 2 * kRadix * 8;      // 16-bit words

template <int THREADS, int ITEMS, bool ORDERED>
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
  // (only used by rounds behind the last: items < ITEMS then)
  const u32 spare = padded + tid;
  if (n_pass > 0 && tid < (u32)kRadix) reinterpret_cast<uint4*>(hist)[tid] = make_uint4(0, 0, 0, 0);
  __syncthreads();
  for (int pass = 0; pass < n_pass; ++pass) {
    const int bit = first_bit + 8 * pass;
    uint16_t* h = hist + (pass & 1) * (kRadix * WAVES);
    uint4* h4 = reinterpret_cast<uint4*>(h);             // [digit]: waves 0..7, 16 bits each
    // A word uses its low 48 bits; the element's rank inside (digit, wave) travels in the
    // upper 16 until the word is stored again.
    u64 wd[ITEMS];
    // This wave's counter of digit d is the 16-bit word h[8 * d + wave]; the atomic works
    // on the 32-bit word it shares with the neighbouring wave's (counts stay below 2^16,
    // so nothing carries over).
    u32* pairs = reinterpret_cast<u32*>(h) + (wave >> 1);
    const int half = (wave & 1) * 16;
#pragma unroll
    for (int r = 0; r < ITEMS; ++r) wd[r] = words[wave_first + r * kWave + lane];
#pragma unroll
    for (int r = 0; r < ITEMS; ++r) {
      const bool on = (u32)r < items;
      const u32 d = (u32)(wd[r] >> bit) & (kRadix - 1);
      u32 rank;
      if (ORDERED) {      // (sort.hpp: digit_rank)
        rank = (atomicAdd(pairs + (WAVES / 2) * d, on ? 1u << half : 0u) >> half) & 0xFFFFu;
      } else {
        const u64 same = match_mask(d, on);
        const u32 before = __popcll(same & lt);
        u32 old = 0;
        if (before == 0) old = atomicAdd(pairs + (WAVES / 2) * d, (u32)__popcll(same) << half);
        old = __shfl(old, same ? __ffsll((unsigned long long)same) - 1 : 0, kWave);
        rank = ((old >> half) & 0xFFFFu) + before;
      }
      wd[r] = (wd[r] & 0xFFFFFFFFFFFFull) | ((u64)rank << 48);
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
      const u32 base = h[WAVES * ((u32)(wd[r] >> bit) & (kRadix - 1)) + wave];
      words[(u32)r < items ? base + (u32)(wd[r] >> 48) : spare] = wd[r] & 0xFFFFFFFFFFFFull;
    }
    __syncthreads();
  }
}

// The same for any cnt <= THREADS * MAX_ITEMS, with as few rounds as cnt needs (`words` holds
// THREADS * MAX_ITEMS words).
template <int THREADS, int MAX_ITEMS, bool ORDERED>
__device__ __forceinline__ void lds_radix_sort_any(u64* words, u32 cnt, int first_bit, int n_pass,
                                                   uint16_t* hist) {
  static_assert(MAX_ITEMS == 8, "one case per number of rounds");
  switch ((cnt + THREADS - 1) / THREADS) {
    case 0: case 1: case 2: lds_radix_sort<THREADS, 2, ORDERED>(words, cnt, first_bit, n_pass, hist); break;
    case 3: case 4: lds_radix_sort<THREADS, 4, ORDERED>(words, cnt, first_bit, n_pass, hist); break;
    case 5: lds_radix_sort<THREADS, 5, ORDERED>(words, cnt, first_bit, n_pass, hist); break;
    case 6: lds_radix_sort<THREADS, 6, ORDERED>(words, cnt, first_bit, n_pass, hist); break;
    default: lds_radix_sort<THREADS, 8, ORDERED>(words, cnt, first_bit, n_pass, hist); break;
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

template <int ITEMS>
struct ChunkLds {
  union {
    u64 words[kChunkThreads * ITEMS];
    SlowLds slow;
  };
  uint16_t hist[kLdsSortHist];
  u32 scratch[kChunkWaves + 1];
  unsigned long long s_or;
};

// ---- what region_sort leaves for region_emit --------------------------------------------
// kind[c]   how region c was ordered:
constexpr u32 kRegionSorted = 0;     // in LDS: order[] describes its sorted positions
constexpr u32 kRegionOneKey = 1;     // it holds one key (or nothing): in order as it stands
constexpr u32 kRegionSlowSrc = 2;    // the slow way; the ordered pairs are in the source arrays
constexpr u32 kRegionSlowA = 3;      //   ... in the first scratch pair (ka, pa)
constexpr u32 kRegionSlowB = 4;      //   ... in the second scratch pair (kb, pb)
// heads[c]  number of group heads (first occurrences of a key in sorted order) in region c;
//           group_heads[c / kRegionGroup] their sum over a group of regions
// order[start + j] (kRegionSorted) for sorted position j of the region:
//           place inside the region of the pair that belongs there (bits 0..11), number of
//           heads at or before j (bits 12..24; 0: j continues the last key of the region
//           before), bit 31: j is a head
constexpr u32 kRegionGroup = 64;
constexpr u32 kOrderPlaceMask = 0xFFFu;
constexpr int kOrderHeadsShift = 12;
constexpr u32 kOrderHeadsMask = 0x1FFFu;
constexpr u32 kOrderHeadBit = 0x80000000u;
static_assert(kChunkThreads * kChunkItems <= (int)kOrderPlaceMask + 1, "a place fits 12 bits");

static_assert(kRegionGroup == (u32)kWave, "region_emit adds up a group's regions one per lane");

// Called by ONE thread of the region's workgroup.
__device__ __forceinline__ void publish_region(u32 chunk, u32 kind, u32 heads, u32* region_kind,
                                               u32* region_heads, u32* group_heads) {
  region_kind[chunk] = kind;
  region_heads[chunk] = heads;
  if (heads) atomicAdd(group_heads + chunk / kRegionGroup, heads);
}

// skeys/spay: the pairs ordered by bucket id (payload = occurrence index | bag << 32),
// read only; ka/pa and kb/pb: scratch of the same shape (only touched the slow way);
// borders[0 .. n_regions]: the regions (region_borders).  One region per workgroup; no
// workgroup waits for another.  group_heads must be zero on entry.
//
// After the LDS sort a thread owns the sorted positions tid, tid + 512, ... of its region
// (conflict-free LDS reads, coalesced writes); the number of heads up to a position comes
// from wave ballots per round of 512 positions and one 64-entry scan over (round, wave).
template <int ITEMS, bool ORDERED>
__global__ void __launch_bounds__(kChunkThreads, 4)
region_sort(const u64* __restrict__ skeys, const u64* __restrict__ spay, u64* __restrict__ ka,
            u64* __restrict__ pa, u64* __restrict__ kb, u64* __restrict__ pb, u32 n,
            const u32* __restrict__ borders, u32* __restrict__ region_kind,
            u32* __restrict__ region_heads, u32* __restrict__ group_heads,
            u32* __restrict__ order, PullCtx* __restrict__ ctx) {
  static_assert(ITEMS == kChunkWaves, "the (round, wave) head counts are scanned by one wave");
  constexpr u32 kChunkCap = kChunkThreads * ITEMS;
  __shared__ ChunkLds<ITEMS> L;
  const u32 tid = threadIdx.x, wave = tid / kWave, lane = tid & (kWave - 1);
  const u64 lt = lanemask_lt();
  const u32 chunk = blockIdx.x;
  if (tid == 0) L.s_or = 0;
  const u32 start = borders[chunk], end = borders[chunk + 1];
  const u32 cnt = end - start;       // start <= end: both borders come from the same rule
  __syncthreads();

  if (cnt > kChunkCap) {
    // ---- the slow way: ordered through global memory, described by where the result is ----
    const u64 *sk, *sp;
    slow_sort_region(skeys, spay, ka, pa, kb, pb, start, end, L.slow, &sk, &sp);
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
    (void)block_excl_sum<kChunkThreads>(heads, L.scratch, &total);
    if (tid == 0)
      publish_region(chunk, sk == skeys ? kRegionSlowSrc : sk == ka ? kRegionSlowA : kRegionSlowB, total,
                     region_kind, region_heads, group_heads);
    return;
  }

  // ---- the usual way: order the region in LDS ----
  const u32 items = (cnt + kChunkThreads - 1) / kChunkThreads;
  // loads behind the region's end repeat its last key (an empty region reads a key it does not use)
  const u32 last_p = cnt ? start + cnt - 1 : min(start, n - 1);
  const u64 key0 = skeys[min(start, last_p)];
  u64 key[ITEMS];
  {
    // which key bits vary inside the region
    u64 diff = 0;
#pragma unroll
    for (int r = 0; r < ITEMS; ++r) {
      const u32 p = r * kChunkThreads + tid;
      key[r] = skeys[min(start + p, last_p)];
      diff |= key[r] ^ key0;
    }
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) diff |= __shfl_xor(diff, d, kWave);
    if (lane == 0 && diff) atomicOr(&L.s_or, (unsigned long long)diff);
  }
  __syncthreads();
  const u64 vary = L.s_or;
  const int hb = vary ? 64 - __clzll((long long)vary) : 0;    // bits [hb, 64) are the same in all keys
  const int lo = hb > kSortBits ? hb - kSortBits : 0;         // the sort takes bits [lo, hb)
  const int n_bits = hb - lo;
  const u64 bit_mask = (1ull << n_bits) - 1;                  // bits above hb are dropped: all equal
  const int top_pass = (n_bits + 7) / 8;
  // the key before the region: a region that starts inside a heavy key's bucket continues
  // that key's group
  const u64 key_before = start > 0 ? skeys[start - 1] : 0;
  if (hb == 0) {
    // One key only (part of a heavy key's bucket, typically), or nothing: the region is
    // in order as it stands.
    if (tid == 0)
      publish_region(chunk, kRegionOneKey, cnt && !(start > 0 && key_before == key0) ? 1u : 0u, region_kind,
                     region_heads, group_heads);
    return;
  }

  // The sorted words stay in LDS to the end: sorted position j holds the place (inside the
  // region) of its pair in the low 16 bits.  The region is ordered by the bits [lo, hb) first;
  // if two different keys then agree in all of those bits (rare with 32 of them), it is
  // ordered again, stably, piece by piece from the lowest bits up, so that all 64 bits count.
  // One sort loop serves all pieces.  Afterwards the rounds are taken four at a time, so that
  // few gathered keys are in registers at once.
#pragma unroll
  for (int r = 0; r < ITEMS; ++r) {
    const u32 q = r * kChunkThreads + tid;
    if (q < cnt) L.words[q] = (((key[r] >> lo) & bit_mask) << 16) | q;
  }
  __syncthreads();
  u32 head_bits = 0;       // bit k: the key at sorted position k * 512 + tid differs from the key before it
  const u32 last_j = cnt - 1;          // (cnt > 0 here) loads behind the region's end repeat its last pair
  // piece of the key the coming sort orders by: bits [piece_lo, piece_lo + piece_bits).  First
  // [lo, hb); if that leaves different keys side by side (redo), the bits below lo from the
  // bottom up, at most 32 at a time (a word has room for 32), and then [lo, hb) again.
  int piece_lo = lo, piece_bits = n_bits;
  bool redo = false;
  while (true) {
    lds_radix_sort_any<kChunkThreads, ITEMS, ORDERED>(L.words, cnt, 16, (piece_bits + 7) / 8, L.hist);
    if (redo && piece_lo != lo) {
      // a piece below lo is in order: the next piece, taken in the order reached so far
      piece_lo += piece_bits;
      piece_bits = piece_lo == lo ? n_bits : min(32, lo - piece_lo);
      const u64 piece_mask = piece_bits == 64 ? ~0ull : (1ull << piece_bits) - 1;
#pragma unroll 1
      for (int r = 0; r < ITEMS; ++r) {
        const u32 q = r * kChunkThreads + tid;
        if (q < cnt) {
          const u32 place = (u32)L.words[q] & 0xFFFFu;
          L.words[q] = (((skeys[start + place] >> piece_lo) & piece_mask) << 16) | place;
        }
      }
      __syncthreads();
      continue;
    }
    bool bad = false;
    head_bits = 0;
#pragma unroll
    for (int k0 = 0; k0 < ITEMS; k0 += 4) {
      if ((u32)k0 >= items) break;       // block-uniform
      u64 word[4], skey[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) word[q] = L.words[min((k0 + q) * kChunkThreads + tid, last_j)];
#pragma unroll
      for (int q = 0; q < 4; ++q) skey[q] = skeys[start + ((u32)word[q] & 0xFFFFu)];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const u32 j = (k0 + q) * kChunkThreads + tid;
        // the pair at the sorted position before: the neighbouring lane's, or (lane 0) looked up
        u64 prev_key = __shfl_up(skey[q], 1, kWave);
        u64 prev_word = __shfl_up(word[q], 1, kWave);
        if (lane == 0) {
          if (j == 0) {
            prev_word = ~0ull;
            prev_key = key_before;
          } else if (j < cnt) {
            prev_word = L.words[j - 1];
            prev_key = skeys[start + ((u32)prev_word & 0xFFFFu)];
          }
        }
        if (j < cnt) {
          const bool differs = skey[q] != prev_key;
          if (start + j == 0 || differs) head_bits |= 1u << (k0 + q);
          if (j > 0 && differs && (prev_word >> 16) == (word[q] >> 16)) bad = true;
        }
      }
    }
    if (redo || !__syncthreads_or(bad && lo > 0)) break;
    // two different keys agreed in all of the bits [lo, hb): start over from the lowest bits,
    // in the order the pairs arrived in
    redo = true;
    piece_lo = 0;
    piece_bits = min(32, lo);
#pragma unroll 1
    for (int r = 0; r < ITEMS; ++r) {
      const u32 q = r * kChunkThreads + tid;
      if (q < cnt) L.words[q] = ((skeys[start + q] & ((1ull << piece_bits) - 1)) << 16) | q;
    }
    __syncthreads();
  }

  // heads up to each of this thread's positions: per round a wave ballot, and one scan over
  // the (round, wave) counts in the order of the positions
  u32 my_count = 0;       // lane k of wave w: heads in round k of wave w
#pragma unroll
  for (int k = 0; k < ITEMS; ++k) {
    const u64 m = __ballot((head_bits >> k) & 1u);
    if (lane == (u32)k) my_count = (u32)__popcll(m);
  }
  u32* counts = reinterpret_cast<u32*>(L.hist);      // [round][wave], then their exclusive prefix
  if (lane < (u32)ITEMS) counts[lane * kChunkWaves + wave] = my_count;
  __syncthreads();
  if (wave == 0) {
    const u32 c = counts[lane];
    const u32 incl = wave_incl_sum(c);
    counts[lane] = incl - c;
    if (lane == kWave - 1) publish_region(chunk, kRegionSorted, incl, region_kind, region_heads, group_heads);
  }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < ITEMS; ++k) {
    const u32 j = k * kChunkThreads + tid;
    const bool head = (head_bits >> k) & 1u;
    const u64 m = __ballot(head);
    if (j < cnt) {
      const u32 upto = counts[k * kChunkWaves + wave] + (u32)__popcll(m & lt) + (head ? 1u : 0u);
      order[start + j] = ((u32)L.words[j] & kOrderPlaceMask) | (upto << kOrderHeadsShift) | (head ? kOrderHeadBit : 0u);
    }
  }
}

// The dedup's outputs for region blockIdx.x from what region_sort left.  The number of heads
// in earlier regions -- the rank of the region's first new key -- is the sum of the earlier
// groups' totals and of the earlier regions of the own group.
__global__ void __launch_bounds__(kChunkThreads)
region_emit(const u64* __restrict__ skeys, const u64* __restrict__ spay, const u64* __restrict__ ka,
            const u64* __restrict__ pa, const u64* __restrict__ kb, const u64* __restrict__ pb, u32 n,
            const u32* __restrict__ borders, const u32* __restrict__ region_kind,
            const u32* __restrict__ region_heads, const u32* __restrict__ group_heads,
            const u32* __restrict__ order, u32 n_bags, u64* __restrict__ uniq,
            i32* __restrict__ inverse, u32* __restrict__ bagperm, u32* __restrict__ seg_off,
            PullCtx* __restrict__ ctx, TableState* __restrict__ st) {
  __shared__ u32 scratch[kChunkWaves + 1];
  __shared__ u32 s_earlier;
  const u32 tid = threadIdx.x;
  const u32 chunk = blockIdx.x, n_chunks = gridDim.x;
  const u32 start = borders[chunk], end = borders[chunk + 1];
  const u32 cnt = end - start;
  const u32 kind = region_kind[chunk];
  const u32 bag_max = n_bags ? n_bags - 1 : 0;
  if (tid < kWave) {
    const u32 g = chunk / kRegionGroup;
    u32 c = 0;
    for (u32 i = tid; i < g; i += kWave) c += group_heads[i];
    const u32 r = g * kRegionGroup + tid;          // kRegionGroup == kWave: one region per lane
    if (r < chunk) c += region_heads[r];
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) c += __shfl_xor(c, d, kWave);
    if (tid == 0) s_earlier = c;
  }
  __syncthreads();
  const u32 earlier = s_earlier;
  if (chunk + 1 == n_chunks && tid == 0) {
    const u32 total = earlier + region_heads[chunk];
    ctx->n_unique = total;
    seg_off[total] = n;
  }
  if (cnt == 0) return;

  if (kind == kRegionSorted) {
    for (u32 j = tid; j < cnt; j += kChunkThreads) {
      const u32 o = order[start + j];
      const u32 at = start + (o & kOrderPlaceMask);
      const u64 pay = spay[at];
      const bool head = (o & kOrderHeadBit) != 0;
      // rank of this pair's key: heads at or before its position, less one
      const u32 rank = earlier + ((o >> kOrderHeadsShift) & kOrderHeadsMask) - 1u;
      // clamped: whatever the offsets said, the push must stay inside the gradient buffer
      bagperm[start + j] = min((u32)(pay >> 32), bag_max) | (head ? kOrderHeadBit : 0u);
      inverse[(u32)pay] = (i32)rank;
      if (head) {
        const u64 key = skeys[at];
        uniq[rank] = key;
        seg_off[rank] = start + j;
        if (key == kEmptyKey) raise_error(st, kErrReserved);
      }
    }
    return;
  }
  if (kind == kRegionOneKey) {
    const u64 key0 = skeys[start];
    const bool is_head = !(start > 0 && skeys[start - 1] == key0);
    const u32 rank = earlier + (is_head ? 1u : 0u) - 1u;      // (earlier >= 1 if it is not a head)
    if (is_head && tid == 0) {
      uniq[rank] = key0;
      seg_off[rank] = start;
      if (key0 == kEmptyKey) raise_error(st, kErrReserved);
    }
    for (u32 j = tid; j < cnt; j += kChunkThreads) {
      const u64 pay = spay[start + j];
      bagperm[start + j] = min((u32)(pay >> 32), bag_max) | (j == 0 && is_head ? kOrderHeadBit : 0u);
      inverse[(u32)pay] = (i32)rank;
    }
    return;
  }
  // ordered the slow way: walk the ordered pairs, a block-wide count of heads per round
  const u64* sk = kind == kRegionSlowSrc ? skeys : kind == kRegionSlowA ? ka : kb;
  const u64* sp = kind == kRegionSlowSrc ? spay : kind == kRegionSlowA ? pa : pb;
  const bool first_is_head = start == 0 || sk[start] != skeys[start - 1];
  u32 rank = earlier;
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
      inverse[(u32)pay] = (i32)r;
      bagperm[j] = min((u32)(pay >> 32), bag_max) | (head ? kOrderHeadBit : 0u);
    }
    rank += tile_heads;
  }
}

}  // namespace hps
