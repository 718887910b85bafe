// Shared device-side definitions of the HBM-PS pull/push kernels (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hps {

typedef uint32_t u32;
typedef uint64_t u64;
typedef int32_t i32;

constexpr u64 kEmptyKey = ~u64(0);   // marks a free slot; never a legal key
constexpr u32 kNoRow = ~u32(0);      // "this key has no row" (lookup miss / table full)
constexpr int kWave = 64;
constexpr int kSlotsPerLine = 8;     // 8 keys of 8 bytes = one 64-byte line, probed by 8 lanes

// Device-side status values mirror hps_status.
constexpr int kErrFull = -2;
constexpr int kErrReserved = -3;
constexpr int kErrInternal = -5;   // HPS_EDEVICE: a dedup's cross-workgroup wait gave up (never expected)

// Plain form of the dedup: places where different keys agree in all sorted bits that
// fix_mixed_runs can note; beyond that one workgroup puts the whole array in order.
constexpr u32 kMaxEvidence = 1024;

// Rows of the mini-batch's most frequent keys that every workgroup of the pooling kernel keeps
// in LDS: at most kHotBytes of them (as float32) and at most kMaxHot keys.
constexpr u32 kHotBytes = 16384;
constexpr u32 kMaxHot = 512;

constexpr int kCountShards = 64;   // counters that many blocks add to are spread over this many words

// Lives in the table's storage for the table's whole life.
struct TableState {
  unsigned long long size;      // keys stored
  unsigned long long inserted;  // keys created by the last pull / insert call
  int error;                    // sticky: 0 or a negative status
  int absent;                   // distinct keys the last accumulate did not find
  unsigned long long dump_count;  // rows seen by the running dump
  // Keys the running lookup found missing / rows the running insert created, spread
  // over shards so that blocks do not all hit one address.
  u32 miss_shard[kCountShards];
  u32 made_shard[kCountShards];
  u32 miss_overflow;            // the list of missing keys did not fit: scan instead
  u32 probe_bad;                // result word of probe_lane_order (written once, at creation)
  // hps_probe_lengths: lines looked at to find each stored key, summed / the most for one key
  unsigned long long probe_sum;
  unsigned long long probe_max;
};

// Where a mini-batch's keys lie, estimated from a sample of them (sort_prepare).  The
// dedup orders keys by rel = clamp(key - lo, 0, span) instead of by the key itself, which
// is the same order, but raw ids that all share their leading bits spread over the
// buckets / digits like hashed keys do (sort.hpp: range_rel, natural_bucket).
struct KeyRange {
  u64 lo;
  u64 span;      // largest rel
  u32 mult;      // bucket form: natural bucket = ((rel >> pre) * mult) >> 32
  u32 pre;       //   (rel >> pre fits 32 bits)
  u32 direct;    // bucket form: span is below the number of natural buckets, natural bucket = rel
  u32 base;      // plain form: the sorted digits start at this bit of rel
};

// Lives in the workspace; describes the outstanding pull.
struct PullCtx {
  u32 n_unique;        // U
  u32 n_long;          // keys the push handles chunk by chunk
  u32 n_slow;          // bucket form: occurrences in regions that did not fit LDS
  u32 n_chunk_items;   // (key, chunk) work items of the push
  u32 n_evidence;      // sorted positions where a run of equal sorted bits mixes keys
  u32 sort_error;      // set if a look-back wait gave up (never expected)
  u32 n_total;         // occurrences of this dedup
  u32 by_id;           // 1: this dedup took the bucket form
  u32 med_count[kCountShards];   // keys the push handles with one wave each, per list shard
  KeyRange range;                // written by the dedup's first kernel for the later ones
  u32 n_slow_one_key;            // ... of n_slow, in regions that one key fills at least half of
  u32 n_hot;                     // keys listed for the pooling kernel's LDS-resident rows (pool.hpp)
};

// Keys that make up a large share of a mini-batch (bucket.hpp).  HeavySet: ascending,
// padded with all-ones.  HeavyRaw: the keys the last lookup saw often, in arrival
// order; only a hint, readers cope with any content.
constexpr int kMaxHeavy = 4095;
constexpr int kSmallHeavy = 1023;    // lists up to this long are copied to LDS by the kernels that look keys up in them
constexpr int kHeavyTopBits = 10;
struct HeavySet {
  u32 count;
  u32 pad;
  u64 keys[kMaxHeavy + 1];
  // per value of a key's top kHeavyTopBits bits: index of the first heavy key with these
  // top bits (low half) and how many there are (high half)
  u32 span[1 << kHeavyTopBits];
};
struct HeavyRaw {
  u32 count;
  u32 pad;
  u64 keys[kMaxHeavy + 1];
};
// Lookup s (s = 1, 2, ...) fills raw[s % 3]; the push of the same pull (an extra block of
// its kernel; for an accumulate the kernel after the lookup) puts that list in order as
// set[s % 3] and empties raw[(s + 1) % 3] for the next lookup.  A dedup issued when s
// lookups have been issued reads set[(s - 1) % 3]: the push of pull s - 1 is certainly
// complete (the dedup waits for the push that released its context, which is that push or a
// later one) and nobody writes the slot again before push s + 2, which comes after this
// dedup's pull.  So every kernel of a dedup sees the same, unchanging list, whatever
// streams the calls were issued on.
constexpr u32 kHeavyRing = 3;
struct HeavyRing {
  HeavyRaw raw[kHeavyRing];
  HeavySet set[kHeavyRing];
};

// SplitMix64 output function for state x (Steele, Lea, Flood 2014).  The row
// initialiser is defined on top of it.
__device__ __forceinline__ u64 mix64(u64 x) {
  u64 z = x + 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

// Slot hash: the 64-bit finaliser of MurmurHash3 (Appleby), so that the table
// does not rely on keys arriving well mixed.
__device__ __forceinline__ u64 slot_hash(u64 k) {
  k ^= k >> 33;
  k *= 0xFF51AFD7ED558CCDull;
  k ^= k >> 33;
  k *= 0xC4CEB9FE1A85EC53ull;
  k ^= k >> 33;
  return k;
}

// Element j of key's initial row: uniform on [-a, a) from 24 random bits, as a
// rounded product followed by a rounded difference.  The two must never be fused
// into one multiply-add (that would round once and change the bits), so
// contraction is switched off for this function.
__device__ __forceinline__ float init_weight(u64 base, u32 j, float a) {
#pragma clang fp contract(off)
  const u64 r = mix64(base + j);
  const float u = (float)(u32)(r >> 40) * 0x1.0p-24f;   // exact
  const float scaled = u * (a * 2.0f);
  return scaled - a;
}

__device__ __forceinline__ u32 lane_id() { return threadIdx.x & (kWave - 1); }

__device__ __forceinline__ u64 lanemask_lt() {
  const u32 l = lane_id();
  return l == 0 ? 0ull : (~0ull >> (64 - l));
}

// Inclusive sum over the 64 lanes of a wave.
__device__ __forceinline__ u32 wave_incl_sum(u32 v) {
#pragma unroll
  for (int d = 1; d < kWave; d <<= 1) {
    const u32 o = __shfl_up(v, d, kWave);
    if ((int)lane_id() >= d) v += o;
  }
  return v;
}

// Exclusive sum over a block of THREADS threads (multiple of 64, at most 1024).
// `scratch` needs THREADS/64 + 1 words of LDS.  Returns the exclusive prefix of v
// and the block total in *total.  Contains __syncthreads().
template <int THREADS>
__device__ __forceinline__ u32 block_excl_sum(u32 v, u32* scratch, u32* total) {
  constexpr int NW = THREADS / kWave;
  const u32 incl = wave_incl_sum(v);
  const u32 w = threadIdx.x / kWave;
  __syncthreads();   // scratch may still be in use by a previous call
  if (lane_id() == kWave - 1) scratch[w] = incl;
  __syncthreads();
  if (threadIdx.x == 0) {
    u32 run = 0;
    for (int i = 0; i < NW; ++i) {
      const u32 c = scratch[i];
      scratch[i] = run;
      run += c;
    }
    scratch[NW] = run;
  }
  __syncthreads();
  *total = scratch[NW];
  return scratch[w] + incl - v;
}

__device__ __forceinline__ int load_error(const TableState* st) {
  return __hip_atomic_load(&st->error, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ void raise_error(TableState* st, int code) {
  atomicCAS(&st->error, 0, code);
}

}  // namespace hps
