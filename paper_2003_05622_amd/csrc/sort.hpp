// Key dedup, part 1: ordering the key occurrences.
//
// The occurrences (key, payload) -- payload = occurrence index and bag number in one
// 64-bit word -- are ordered with a stable least-significant-digit radix sort, 8 bits per
// pass, ONE kernel per pass:
//
//   sort_prepare    digit histograms of all passes in one read of the keys (also
//                   writes bag_of[i], the bag of occurrence i);
//   onesweep_pass   a tile takes a ticket and counts its digits; an extra wave then
//                   publishes the counts and obtains, by decoupled look-back over the
//                   per-tile status words, how many same-digit elements earlier tiles
//                   hold, while the three worker waves rank the tile's elements with
//                   wave ballots; the tile is staged in LDS and each digit's run is
//                   written contiguously.
//
// These passes are the plain form of the dedup: they sort by the top 8 * n_pass bits of the
// key's place in the range the mini-batch's keys span (for hashed keys: of the key).
// Mini-batch keys are hashed feature ids, so these bits separate almost all distinct keys;
// the rare runs that still mix different keys are found and put right afterwards
// (dedup.hpp).  With eight passes every bit is sorted and nothing is left to put right.
// The usual form, by bucket ids (bucket_id below), has passes of its own without any waits
// between workgroups (partition.hpp) and finishes per region (bucket.hpp); it shares this
// file's key range, bucket ids and ranking helpers.
// Either way the dedup's result is exact for any input.
//
// Cross-tile counts without a serial chain: tiles are grouped, `group` consecutive
// tiles (by ticket) per group.  Every tile publishes its digit counts (a row of 256
// status words); the last tile of a group also publishes the group's counts.  A tile
// then needs the rows of the earlier tiles of its own group and the rows of all
// earlier groups: two dependent waits however many tiles there are.  A tile only ever
// waits for tiles with smaller tickets, which are running, so the waits end.
//
// Status word (32-bit): epoch << 20 | count.  The epoch (1..4095) is the pull's serial
// number modulo 4095, so words of earlier pulls read as "not ready"; the host clears
// the words each time the epoch wraps.
#pragma once

#include "common.hpp"

namespace hps {

constexpr int kRadixBits = 8;
constexpr int kRadix = 1 << kRadixBits;
constexpr int kMaxPasses = 8;
constexpr int kSortThreads = 256;                      // three worker waves + the look-back wave
constexpr int kSortWorkers = kSortThreads - kWave;     // threads that hold elements
constexpr int kSortWaves = kSortWorkers / kWave;
constexpr int kSortItems = 16;                         // per worker thread
constexpr int kSortTile = kSortWorkers * kSortItems;   // 3072 elements
constexpr int kSortWaveSpan = kWave * kSortItems;      // 1024 consecutive elements per wave
constexpr int kPrepThreads = 256;
// The global digit histograms are kept in kHistShards copies (block b adds to copy b %
// kHistShards; readers add the copies up): hundreds of blocks adding to ONE set of
// counters queue up behind each other, same-address device atomics being slow.
constexpr int kHistShards = 16;
constexpr int kHistWords = kHistShards * kMaxPasses * kRadix;   // one pull's histograms

// A wait for another workgroup's status word gives up after this long (100 MHz ticks: five
// seconds).  Nothing legitimate comes near: only the plain form's passes wait, a tile for
// the counts of tiles with smaller tickets, which are running and need microseconds each
// (the bucket form has no waits between workgroups at all).
constexpr u64 kWaitTicks = 500000000ull;
constexpr u32 kRangeSamples = 2048;    // keys sampled for the key range (sort_prepare)
constexpr u32 kEpochMod = 4095;        // epochs run 1..4095
constexpr u32 kMaxTileGroup = 64;      // tiles per group at most (count fits 19 bits)
constexpr int kLookChunk = 8;          // status rows read per round trip

static_assert(kRadix == kSortThreads, "thread d owns digit d");
static_assert(kRadix == 4 * kWave, "each look-back lane owns four digits");

struct SortPlan {
  int n_pass;       // digits sorted
  int low_shift;    // plain mode: 64 - 8 * n_pass: so many low bits stay unsorted if keys fill 64 bits
  u32 group;        // tiles per group
  int by_id;        // 1: the passes sort by the bucket id of the key (see bucket_id) instead
  int nat_shift;    // by_id: 64 - log2 of the number of natural buckets
  u32 max_heavy;    // by_id: heavy keys that get buckets of their own, at most
};

__device__ __forceinline__ u32 key_digit(u64 k, int shift) {
  return (u32)(k >> shift) & (kRadix - 1);
}

// ---- key range ------------------------------------------------------------------------
// A key's place in the range its mini-batch's keys span: monotone in the key, and the
// same for keys outside the (sampled, slightly widened) range as for the range's ends.
__device__ __forceinline__ u64 range_rel(u64 key, const KeyRange& r) {
  const u64 rel = key > r.lo ? key - r.lo : 0;
  return min(rel, r.span);
}
// Plain form: the bits of a key the passes sort by (and which unique_emit compares).
__device__ __forceinline__ u64 sorted_prefix(u64 key, const KeyRange& r) {
  return range_rel(key, r) >> r.base;
}
// Bucket form: the range cut into 2^nat_bits equal parts.
__device__ __forceinline__ u32 natural_bucket(u64 key, const KeyRange& r) {
  const u64 rel = range_rel(key, r);
  return r.direct ? (u32)rel : (u32)(((rel >> r.pre) * r.mult) >> 32);
}
// From the smallest and largest sampled key.  The range is widened by 1/256 of its length
// at both ends: with kRangeSamples samples of evenly spread keys, the share of keys
// beyond the widened ends (they all land in the first / last part) is then far below one
// part's share.
__device__ __forceinline__ KeyRange make_range(u64 lo, u64 hi, const SortPlan& plan) {
  const u64 widen = (hi - lo) >> 8;
  lo = lo > widen ? lo - widen : 0;
  hi = hi + widen >= hi ? hi + widen : ~0ull;
  KeyRange r;
  r.lo = lo;
  r.span = hi - lo;
  const u32 bits = r.span ? 64 - __clzll((long long)r.span) : 0;
  r.pre = bits > 32 ? bits - 32 : 0;
  const u32 nat_bits = plan.by_id ? 64 - plan.nat_shift : 0;
  r.direct = (r.span >> nat_bits) == 0;
  // span >= 2^nat_bits here, so the quotient is below 2^32 and parts are numbered below 2^nat_bits
  r.mult = r.direct ? 0u : (u32)((1ull << (32 + nat_bits)) / ((r.span >> r.pre) + 1));
  if (plan.by_id) {
    r.base = 0;
    return r;
  }
  // Plain form: the passes order sorted_bits bits of rel from bit `base` up, so every key with
  // rel < 2^(base + sorted_bits) is placed exactly, not only those inside the sampled range:
  // the range that is covered reaches that far, with the sampled range in its middle (a
  // long-tailed set of raw ids has many keys beyond its largest sample; clamped to one
  // place they would all have to be put in order afterwards).
  const u32 sorted_bits = 64 - plan.low_shift;
  r.base = bits > sorted_bits ? bits - sorted_bits : 0;
  const u64 cover = r.base + sorted_bits >= 64 ? ~0ull : (1ull << (r.base + sorted_bits)) - 1;
  const u64 spare = (cover - r.span) / 2;
  r.lo = lo > spare ? lo - spare : 0;
  r.span = cover;
  return r;
}

// ---- bucket ids ---------------------------------------------------------------------
// Keys that make up a large share of a mini-batch ("heavy" keys; found from a sample,
// bucket.hpp) get buckets of their own, so that every other bucket stays small enough
// to be sorted inside one workgroup.  With the heavy keys h_0 < h_1 < ... the id of a
// key is
//     natural(key) + 2 * #{i : h_i < key} + (key is heavy ? 1 : 0),
// natural(key) = which of 2^(64 - nat_shift) equal parts of the mini-batch's key range the
// key lies in (natural_bucket; for hashed keys: the key's leading bits),
// which is monotone in the key; keys share an id only if they share the part and no
// heavy key lies between them, and a heavy key shares its id with nothing.

// The heavy keys in LDS, with their spans per value of the top bits, so that a lookup
// costs one LDS read unless heavy keys share the key's top bits.  A list of more than
// kSmallHeavy keys (rare) stays in global memory: `keys` points to it instead of `lds_keys`.
struct HeavyLds {
  u64 lds_keys[kSmallHeavy + 1];
  const u64* keys;
  u32 span[1 << kHeavyTopBits];
  KeyRange range;
  u32 max_heavy;     // only the max_heavy smallest heavy keys get buckets of their own
};

// All threads of the block; the caller's next barrier makes the copy visible.  H.range is
// the caller's to fill.
__device__ __forceinline__ void load_heavy(HeavyLds& H, const HeavySet* set, u32 max_heavy) {
  // (only the listed keys are ever looked at: the spans index nothing behind them)
  const u32 count = min(set->count, (u32)kMaxHeavy);
  const bool small = count <= (u32)kSmallHeavy;
  if (small)
    for (u32 i = threadIdx.x; i < count; i += blockDim.x) H.lds_keys[i] = set->keys[i];
  for (u32 i = threadIdx.x; i < (1u << kHeavyTopBits); i += blockDim.x) H.span[i] = set->span[i];
  if (threadIdx.x == 0) {
    H.max_heavy = max_heavy;
    H.keys = small ? H.lds_keys : set->keys;
  }
}

// *heavy tells whether the key is one of the heavy keys (that count: see max_heavy;
// limiting them keeps the ids of a small dedup below 256, one pass, and the id monotone).
__device__ __forceinline__ u32 bucket_id(u64 key, const HeavyLds& H, bool* heavy) {
  const u32 sp = H.span[(u32)(key >> (64 - kHeavyTopBits))];
  u32 m = sp & 0xFFFFu;
  const u32 end = m + (sp >> 16);
  bool is_heavy = false;
  if (m < end) {                       // (most keys: no heavy key shares their top bits)
    const u64* hk = H.keys;
    while (m < end && hk[m] < key) ++m;
    is_heavy = m < end && m < H.max_heavy && hk[m] == key;
  }
  *heavy = is_heavy;
  m = min(m, H.max_heavy);
  return natural_bucket(key, H.range) + 2 * m + (is_heavy ? 1u : 0u);
}

// ---- status words -------------------------------------------------------------------
__device__ __forceinline__ u32 status_word(u32 epoch, u32 count) { return (epoch << 20) | count; }
__device__ __forceinline__ bool status_ready(u32 w, u32 epoch) { return (w >> 20) == epoch; }
__device__ __forceinline__ u32 status_count(u32 w) { return w & 0xFFFFFu; }

// A lane's four consecutive status words (16 bytes) as two 64-bit device-scope
// accesses.  Every 32-bit word is valid on its own, so nothing orders them.
__device__ __forceinline__ void store_row4(u32* row, u32 lane, u32 epoch, const u32* count) {
  u64* p = reinterpret_cast<u64*>(row + 4 * lane);
  __hip_atomic_store(p, (u64)status_word(epoch, count[0]) | ((u64)status_word(epoch, count[1]) << 32),
                     __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  __hip_atomic_store(p + 1, (u64)status_word(epoch, count[2]) | ((u64)status_word(epoch, count[3]) << 32),
                     __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void load_row4(const u32* row, u32 lane, u32* w) {
  const u64* p = reinterpret_cast<const u64*>(row + 4 * lane);
  const u64 a = __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  const u64 b = __hip_atomic_load(p + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  w[0] = (u32)a; w[1] = (u32)(a >> 32); w[2] = (u32)b; w[3] = (u32)(b >> 32);
}

// One more round of a wait for another workgroup: sleeps (longer and longer: hundreds of
// waves polling in a tight loop take memory bandwidth from the workgroup they wait for)
// and tells whether to go on.  `spins` and `since` are the wait's state, spins = 0 at first.
__device__ __forceinline__ bool keep_waiting(u32* spins, u64* since) {
  const u32 s = (*spins)++;
  if (s == 0) *since = wall_clock64();
  if (s < 64) {
    __builtin_amdgcn_s_sleep(8);
    return true;
  }
  const u32 naps = min((s - 64) / 64 + 1, 32u);      // 127 * 64 cycles each
  for (u32 k = 0; k < naps; ++k) __builtin_amdgcn_s_sleep(127);
  return wall_clock64() - *since < kWaitTicks;
}

// Adds to sum[0..3] this lane's digits of rows [first, last) of `rows` (kRadix words
// per row), waiting for each row to be published.  Returns false if a wait gave up.
__device__ __forceinline__ bool sum_rows(const u32* rows, u32 first, u32 last, u32 lane, u32 epoch,
                                         u32* sum) {
  for (u32 r0 = first; r0 < last; r0 += kLookChunk) {
    u32 spins = 0;
    u64 since = 0;
    while (true) {
      u32 w[kLookChunk][4];
#pragma unroll
      for (int k = 0; k < kLookChunk; ++k) {
        if (r0 + k < last) {
          load_row4(rows + (u64)(r0 + k) * kRadix, lane, w[k]);
        } else {
#pragma unroll
          for (int q = 0; q < 4; ++q) w[k][q] = status_word(epoch, 0);
        }
      }
      bool ready = true;
#pragma unroll
      for (int k = 0; k < kLookChunk; ++k)
#pragma unroll
        for (int q = 0; q < 4; ++q) ready = ready && status_ready(w[k][q], epoch);
      if (ready) {
#pragma unroll
        for (int k = 0; k < kLookChunk; ++k)
#pragma unroll
          for (int q = 0; q < 4; ++q) sum[q] += status_count(w[k][q]);
        break;
      }
      if (!keep_waiting(&spins, &since)) return false;   // never expected
    }
  }
  return true;
}

// Wave-wide sum of the counts in words[first, last) (one status word each), waiting
// for every word to be published.  All lanes get the sum; *ok is cleared if a wait
// gave up.
__device__ __forceinline__ u32 wave_sum_words(const u32* words, u32 first, u32 last, u32 lane,
                                              u32 epoch, bool* ok) {
  u32 c = 0;
  for (u32 r = first + lane; r < last; r += kWave) {
    u32 spins = 0;
    u64 since = 0;
    while (true) {
      const u32 w = __hip_atomic_load(words + r, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (status_ready(w, epoch)) { c += status_count(w); break; }
      if (!keep_waiting(&spins, &since)) { *ok = false; break; }   // never expected
    }
  }
#pragma unroll
  for (int d = 1; d < kWave; d <<= 1) c += __shfl_xor(c, d, kWave);
  return c;
}

// The lanes of the wave (among `valid` ones) whose digit equals this lane's.
__device__ __forceinline__ u64 match_mask(u32 d, bool valid) {
  u64 same = __ballot(valid);
#pragma unroll
  for (int b = 0; b < kRadixBits; ++b) {
    const bool bit = (d >> b) & 1;
    const u64 bb = __ballot(bit);
    same &= bit ? bb : ~bb;
  }
  return same;
}

// Rank of this lane's element among the wave's elements with the same digit, counted
// over all calls so far: `counter` (LDS) holds the digit's running count for this wave.
//
// ORDERED = false: the lanes with the same digit are found with wave ballots; the first of
// them adds the group's size with ONE returning atomic and hands the old value to the
// others by a shuffle, so consecutive calls do not wait for each other (LDS executes a
// wave's operations in order; nothing has to come back before the next call's atomic is
// issued).  About fifty vector instructions per call.
// ORDERED = true: every lane adds one with its own returning atomic and takes the old value
// as its rank.  That is only the rank in lane order if the LDS serves the lanes of one
// instruction that hit the same address in ascending lane order -- which the instruction
// set manual does not promise, so the library measures it (probe_lane_order below, once per
// GPU when the first table is created there) and uses this form only where it holds.
template <bool ORDERED>
__device__ __forceinline__ u32 digit_rank(u32* counter, u32 d, bool valid, u64 lt) {
  if (ORDERED) return valid ? atomicAdd(counter, 1u) : 0u;
  const u64 same = match_mask(d, valid);
  const u32 before = __popcll(same & lt);
  u32 old = 0;
  if (valid && before == 0) old = atomicAdd(counter, (u32)__popcll(same));
  old = __shfl(old, same ? __ffsll((unsigned long long)same) - 1 : 0, kWave);
  return old + before;
}

// Counts, over `rounds` rounds of pseudo-random digits per wave (uniform digits, few distinct
// digits, one digit only, one frequent digit, all distinct; all lanes or a random part of
// them active), the lanes whose ORDERED rank differs from the ballot rank; adds the count to
// *n_bad.  Two atomics per round, the second on top of the first's counts.
__global__ void __launch_bounds__(kSortThreads)
probe_lane_order(u32 rounds, u32* __restrict__ n_bad) {
  __shared__ u32 cnt[kSortThreads / kWave][kRadix];
  const u32 wave = threadIdx.x / kWave, lane = lane_id();
  const u64 lt = lanemask_lt();
  u32 bad = 0;
  for (u32 r = 0; r < rounds; ++r) {
    for (u32 d = lane; d < (u32)kRadix; d += kWave) cnt[wave][d] = 0;
    const u64 h = mix64(((u64)blockIdx.x << 40) ^ ((u64)wave << 32) ^ ((u64)r << 8) ^ lane);
    const u64 hw = mix64(((u64)blockIdx.x << 40) ^ ((u64)wave << 32) ^ r ^ 0xABCDEFull);   // the same in all lanes
    const u32 mode = (u32)(hw % 6);
    u32 d;
    if (mode == 0) d = (u32)h & 255u;
    else if (mode == 1) d = (u32)h & 3u;
    else if (mode == 2) d = 7u;
    else if (mode == 3) d = ((u32)h & 255u) < 200u ? 42u : (u32)(h >> 8) & 255u;
    else if (mode == 4) d = lane;
    else d = lane / 2;
    const bool active = mode == 0 ? ((h >> 20) & 3) != 0 : true;
    const u64 same = match_mask(d, active);
    const u32 expect = __popcll(same & lt);
    const u32 first = digit_rank<true>(&cnt[wave][d], d, active, lt);
    const u32 second = digit_rank<true>(&cnt[wave][d], d, active, lt);
    if (active && (first != expect || second != expect + (u32)__popcll(same))) ++bad;
  }
  if (bad) atomicAdd(n_bad, bad);
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

// Resets of the pull context, shared by the first kernel of either dedup form.
__device__ __forceinline__ void reset_ctx(PullCtx* ctx, u32 n, u32 by_id) {
  if (threadIdx.x == 0) {
    ctx->n_unique = 0;
    ctx->n_long = 0;
    ctx->n_chunk_items = 0;
    ctx->n_evidence = 0;
    ctx->sort_error = 0;
    ctx->n_slow = 0;
    ctx->n_slow_one_key = 0;
    ctx->n_hot = 0;
    ctx->n_total = n;
    ctx->by_id = by_id;
  }
  if (threadIdx.x < kCountShards) ctx->med_count[threadIdx.x] = 0;
}

// bag_of[i] = bag of occurrence i, by the blocks of a launch that are given this role:
// `block` of `n_blocks`, kPrepThreads threads each.  A wave takes 64 bags at a time; bags of
// more than 8 occurrences are filled by the whole wave.  offsets == nullptr: bag_of[i] = i.
__device__ __forceinline__ void expand_bags(const i32* __restrict__ offsets, u32 n_bags, u32 n,
                                            i32* __restrict__ bag_of, u32 block, u32 n_blocks) {
  if (offsets == nullptr) {
    for (u32 i = block * kPrepThreads + threadIdx.x; i < n; i += n_blocks * kPrepThreads)
      bag_of[i] = (i32)i;
    return;
  }
  const u32 wave_global = (block * kPrepThreads + threadIdx.x) / kWave;
  const u32 n_waves = n_blocks * (kPrepThreads / kWave);
  for (u32 b0 = wave_global * kWave; b0 < n_bags; b0 += n_waves * kWave) {
    const u32 b = b0 + lane_id();
    i32 lo = 0, hi = 0;
    if (b < n_bags) { lo = offsets[b]; hi = offsets[b + 1]; }
    lo = max(lo, 0);
    hi = min(hi, (i32)n);          // never write outside bag_of, whatever the offsets say
    const bool big = hi - lo > 8;
    if (!big) for (i32 i = lo; i < hi; ++i) bag_of[i] = (i32)b;
    u64 todo = __ballot(big);
    while (todo) {
      const int src = __ffsll((unsigned long long)todo) - 1;
      todo &= todo - 1;
      const i32 blo = __shfl(lo, src, kWave), bhi = __shfl(hi, src, kWave);
      for (i32 i = blo + (i32)lane_id(); i < bhi; i += kWave) bag_of[i] = (i32)(b0 + src);
    }
  }
}

// Smallest and largest of kRangeSamples sampled keys, to every thread of the block (kPrepThreads
// threads; contains barriers; s_lo / s_hi: kPrepThreads / kWave words of LDS each).  The samples
// are kRangeSamples / 8 evenly spaced runs of 8 consecutive keys (a 64-byte line each, the first
// and the last included), so that a wave's request is 8 lines and not 64: every block asks for
// the same lines, and the caches serve requests, not bytes.
__device__ __forceinline__ void sample_key_range(const u64* __restrict__ keys, u32 n, u64* s_lo,
                                                 u64* s_hi) {
  u64 lo = ~0ull, hi = 0;
  const u32 n_samples = min(n, kRangeSamples);
  const u32 n_lines = n >> 3;
  for (u32 j = threadIdx.x; j < n_samples; j += kPrepThreads) {
    const u32 at = n > kRangeSamples
                       ? (u32)(((u64)(j >> 3) * (n_lines - 1)) / (kRangeSamples / 8 - 1)) * 8 + (j & 7)
                       : j;
    const u64 key = keys[at];
    lo = min(lo, key);
    hi = max(hi, key);
  }
#pragma unroll
  for (int d = 1; d < kWave; d <<= 1) {
    lo = min(lo, (u64)__shfl_xor((unsigned long long)lo, d, kWave));
    hi = max(hi, (u64)__shfl_xor((unsigned long long)hi, d, kWave));
  }
  if (lane_id() == 0) { s_lo[threadIdx.x / kWave] = lo; s_hi[threadIdx.x / kWave] = hi; }
}

// First kernel of a plain-form dedup: histograms of every pass's digit over all keys (the
// first hist_blocks blocks, which also reset what the passes need) and bag_of[i] (the other
// blocks, at least one).
//   ghist      [kHistShards][kMaxPasses][kRadix] of this pull (zero on entry), ghist_next the
//              buffer the next pull will use (cleared here)
//   tickets    [kMaxPasses + 2] tile tickets of the passes and of the two unique scans
// Every histogram block first works out the range of the keys from the same kRangeSamples
// sampled keys (so all agree); block 0 leaves it in ctx->range for the later kernels.
__global__ void __launch_bounds__(kPrepThreads)
sort_prepare(const u64* __restrict__ keys, u32 n, SortPlan plan, u32* __restrict__ ghist,
             u32* __restrict__ ghist_next, u32* __restrict__ tickets, PullCtx* __restrict__ ctx,
             const i32* __restrict__ offsets, u32 n_bags, i32* __restrict__ bag_of, u32 hist_blocks) {
  if (blockIdx.x >= hist_blocks) {
    expand_bags(offsets, n_bags, n, bag_of, blockIdx.x - hist_blocks, gridDim.x - hist_blocks);
    return;
  }
  __shared__ u32 h[kMaxPasses][kRadix];
  __shared__ KeyRange s_range;
  __shared__ u64 s_lo[kPrepThreads / kWave], s_hi[kPrepThreads / kWave];
  // The block's first tile is requested before anything waits for the samples, so that the
  // two round trips to memory overlap (hist_blocks <= number of tiles: every block has one).
  constexpr int kPrepItems = kSortTile / kPrepThreads;
  u64 first_keys[kPrepItems];
#pragma unroll
  for (int k = 0; k < kPrepItems; ++k) {
    const u32 i = blockIdx.x * kSortTile + k * kPrepThreads + threadIdx.x;
    first_keys[k] = i < n ? keys[i] : 0;
  }
  sample_key_range(keys, n, s_lo, s_hi);
  for (u32 sh = blockIdx.x; sh < (u32)kHistShards; sh += hist_blocks)     // the next pull's counters
    for (int i = threadIdx.x; i < kMaxPasses * kRadix; i += kPrepThreads)
      ghist_next[sh * kMaxPasses * kRadix + i] = 0;
  for (int i = threadIdx.x; i < kMaxPasses * kRadix; i += kPrepThreads) (&h[0][0])[i] = 0;
  if (blockIdx.x == 0) {
    if (threadIdx.x < kMaxPasses + 2) tickets[threadIdx.x] = 0;
    reset_ctx(ctx, n, 0u);
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    u64 lo = s_lo[0], hi = s_hi[0];
    for (int w = 1; w < kPrepThreads / kWave; ++w) { lo = min(lo, s_lo[w]); hi = max(hi, s_hi[w]); }
    if (lo > hi) lo = hi = 0;            // n == 0
    s_range = make_range(lo, hi, plan);
    if (blockIdx.x == 0) ctx->range = s_range;
  }
  __syncthreads();
  const KeyRange range = s_range;
  const u32 n_tiles = (n + kSortTile - 1) / kSortTile;
  auto count_key = [&](u64 key) {
    const u64 prefix = sorted_prefix(key, range);
    for (int p = 0; p < plan.n_pass; ++p)
      atomicAdd(&h[p][key_digit(prefix, p * kRadixBits)], 1u);
  };
#pragma unroll
  for (int k = 0; k < kPrepItems; ++k) {
    const u32 i = blockIdx.x * kSortTile + k * kPrepThreads + threadIdx.x;
    if (i < n) count_key(first_keys[k]);
  }
  for (u32 tile = blockIdx.x + hist_blocks; tile < n_tiles; tile += hist_blocks) {
    const u32 base = tile * kSortTile;
#pragma unroll 4
    for (int k = 0; k < kPrepItems; ++k) {
      const u32 i = base + k * kPrepThreads + threadIdx.x;
      if (i < n) count_key(keys[i]);
    }
  }
  __syncthreads();
  for (int i = threadIdx.x; i < plan.n_pass * kRadix; i += kPrepThreads) {
    const u32 c = (&h[0][0])[i];
    if (c) atomicAdd(&ghist[(blockIdx.x % kHistShards) * kMaxPasses * kRadix + i], c);
  }
}

// One stable radix pass over (key, payload) pairs; payload = index | bag << 32.
// FIRST: the payload is built from the position and bag_of (read in order).
// The digit is bits shift .. shift + 7 of the key's sorted prefix (sorted_prefix).  `ghist`
// is this pass's global digit histogram; tile_rows [n_tiles][kRadix] and group_rows
// [n_groups][kRadix] are this pass's status words.
template <bool FIRST>
__global__ void __launch_bounds__(kSortThreads)
onesweep_pass(const u64* __restrict__ keys_in, const u64* __restrict__ pay_in,
              const i32* __restrict__ bag_of, u64* __restrict__ keys_out,
              u64* __restrict__ pay_out, u32 n, int shift,
              const u32* __restrict__ ghist, u32* __restrict__ tile_rows,
              u32* __restrict__ group_rows, u32 group, u32* __restrict__ ticket, u32 epoch,
              PullCtx* __restrict__ ctx) {
  __shared__ u32 tile_hist[kRadix];              // digit counts of the tile
  __shared__ u32 earlier[kRadix];                // same-digit elements in earlier tiles
  __shared__ u32 wave_cnt[kSortWaves][kRadix];   // per-wave digit counts, then wave offsets
  __shared__ u32 local_start[kRadix];            // first staged position of each digit
  __shared__ u32 out_base[kRadix];               // global position of the digit's run - local_start
  __shared__ u32 scratch[kSortThreads / kWave + 1];
  __shared__ u32 s_tile;
  __shared__ u64 stage[kSortTile];               // keys first, then the payloads
  __shared__ uint8_t stage_digit[kSortTile];     // digit of each staged key

  const u32 tid = threadIdx.x;
  const bool worker = tid < kSortWorkers;
  if (tid == 0) s_tile = atomicAdd(ticket, 1u);
  for (int d = tid; d < kSortWaves * kRadix; d += kSortThreads) (&wave_cnt[0][0])[d] = 0;
  tile_hist[tid] = 0;
  __syncthreads();
  const u32 tile = s_tile;
  const u32 wave = tid / kWave, lane = tid & (kWave - 1);
  const u32 tile_base = tile * kSortTile;
  const u32 tile_n = min((u32)kSortTile, n - tile_base);
  const u32 wave_base = tile_base + wave * kSortWaveSpan;
  const KeyRange range = ctx->range;

  u64 key[kSortItems];
  u64 pay[kSortItems];
  u32 rank[kSortItems];
  u32 digit[kSortItems];
  if (worker) {
#pragma unroll
    for (int r = 0; r < kSortItems; ++r) {
      const u32 i = wave_base + r * kWave + lane;
      key[r] = (i < n) ? keys_in[i] : ~0ull;
      if (FIRST)
        pay[r] = (i < n) ? ((u64)i | ((u64)(u32)bag_of[i] << 32)) : 0ull;
      else
        pay[r] = (i < n) ? pay_in[i] : 0ull;
      digit[r] = key_digit(sorted_prefix(key[r], range), shift);
    }
#pragma unroll
    for (int r = 0; r < kSortItems; ++r) {
      const u32 i = wave_base + r * kWave + lane;
      if (i < n) atomicAdd(&tile_hist[digit[r]], 1u);
    }
  }
  __syncthreads();

  if (!worker) {
    // Look-back wave: lane l owns digits 4l .. 4l+3.
    u32 mine[4], sum[4] = {0, 0, 0, 0};
#pragma unroll
    for (int q = 0; q < 4; ++q) mine[q] = tile_hist[4 * lane + q];
    store_row4(tile_rows + (u64)tile * kRadix, lane, epoch, mine);
    const u32 g = tile / group;
    bool ok = sum_rows(tile_rows, g * group, tile, lane, epoch, sum);   // earlier tiles of my group
    if (tile % group == group - 1) {                                    // last of the group
      u32 total[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) total[q] = sum[q] + mine[q];
      store_row4(group_rows + (u64)g * kRadix, lane, epoch, total);
    }
    ok = sum_rows(group_rows, 0, g, lane, epoch, sum) && ok;            // all earlier groups
    if (!ok) ctx->sort_error = 1;
#pragma unroll
    for (int q = 0; q < 4; ++q) earlier[4 * lane + q] = sum[q];
  } else {
    // Workers: rank each element among the wave's earlier elements with the same
    // digit (element order inside a wave: round by round, then by lane).
    const u64 lt = lanemask_lt();
#pragma unroll
    for (int r = 0; r < kSortItems; ++r) {
      const u32 i = wave_base + r * kWave + lane;
      rank[r] = digit_rank<false>(&wave_cnt[wave][digit[r]], digit[r], i < n, lt);
    }
  }
  __syncthreads();

  // Thread d owns digit d: the waves' offsets inside the run, the run's place.
  u32 digit_total = 0;
#pragma unroll
  for (int w = 0; w < kSortWaves; ++w) {
    const u32 c = wave_cnt[w][tid];
    wave_cnt[w][tid] = digit_total;
    digit_total += c;
  }
  u32 total;
  u32 digit_count = 0;
#pragma unroll
  for (int sh = 0; sh < kHistShards; ++sh) digit_count += ghist[sh * kMaxPasses * kRadix + tid];
  const u32 gbase = block_excl_sum<kSortThreads>(digit_count, scratch, &total);
  const u32 start = block_excl_sum<kSortThreads>(digit_total, scratch, &total);
  local_start[tid] = start;
  out_base[tid] = gbase + earlier[tid] - start;
  __syncthreads();

  u32 pos[kSortItems];
  if (worker) {
#pragma unroll
    for (int r = 0; r < kSortItems; ++r) {
      const u32 i = wave_base + r * kWave + lane;
      pos[r] = 0;
      if (i < n) {
        const u32 d = digit[r];
        pos[r] = local_start[d] + wave_cnt[wave][d] + rank[r];
        stage[pos[r]] = key[r];
        stage_digit[pos[r]] = (uint8_t)d;
      }
    }
  }
  __syncthreads();
  u32 dest[kSortItems];
  if (worker) {
#pragma unroll
    for (int k = 0; k < kSortItems; ++k) {
      const u32 p = k * kSortWorkers + tid;
      dest[k] = 0;
      if (p < tile_n) {
        dest[k] = out_base[stage_digit[p]] + p;
        keys_out[dest[k]] = stage[p];
      }
    }
  }
  __syncthreads();
  if (worker) {
#pragma unroll
    for (int r = 0; r < kSortItems; ++r) {
      const u32 i = wave_base + r * kWave + lane;
      if (i < n) stage[pos[r]] = pay[r];
    }
  }
  __syncthreads();
  if (worker) {
#pragma unroll
    for (int k = 0; k < kSortItems; ++k) {
      const u32 p = k * kSortWorkers + tid;
      if (p < tile_n) pay_out[dest[k]] = stage[p];
    }
  }
}

}  // namespace hps
