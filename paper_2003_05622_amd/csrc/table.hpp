// The HBM hash table: open addressing over 64-byte lines of 8 slots, linear
// probing line by line, one 8-lane group per key (each lane looks at one slot of
// the line), lock-free insertion by 64-bit compare-and-swap on the slot's key.
//
// Layout (structure of arrays, row index = slot index):
//   keys[n_slots]            u64, kEmptyKey when free
//   w[n_slots][dim]          f32
//   acc[n_slots][acc_len]    f32
//
// Looking keys up and creating the missing ones are two kernels, so that the room
// check against the capacity is one consistent decision and no block has to hit a
// single counter: lookup_keys counts the missing keys into sharded counters,
// insert_missing (every block reads the same total) claims slots only if all of
// them fit and counts the rows it creates, commit_insert adds that count to the
// table size.
#pragma once

#include "common.hpp"

namespace hps {

struct TableView {
  u64* keys;
  // Row r's weights start w_pitch * r bytes after w, its accumulator(s) acc_pitch * r bytes
  // after acc.  Two layouts: weights and accumulators in arrays of their own, or (float32
  // rows with one accumulator per element, where a row's 8 * dim bytes divide the 128-byte
  // memory line or are a multiple of it) side by side, acc = w + 4 * dim and both pitches
  // 8 * dim: the push then finds a row's accumulators in the line(s) it fetched for the
  // weights, and the pooling fetches a full line per 64-byte row either way.
  char* w;
  char* acc;
  u32 w_pitch;
  u32 acc_pitch;
  TableState* st;
  u64 n_lines;      // n_slots / 8
  u64 capacity;
  u32 dim;
  u32 acc_len;
  float init_acc;
  float init_range;
  u64 init_seed;
  u32 bf16;         // 1: w holds bfloat16 values (2 bytes each) instead of float32
};

// ---- weights as stored --------------------------------------------------------------
// Rows hold float32 or bfloat16 values (the upper half of a float32; stored with
// round-to-nearest, ties to even); all arithmetic is float32 either way.
__device__ __forceinline__ float bf16_value(u32 h) { return __uint_as_float(h << 16); }
__device__ __forceinline__ u32 bf16_nearest(float f) {
  const u32 u = __float_as_uint(f);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u >> 16) | 0x40u;     // NaN stays NaN
  return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}
__device__ __forceinline__ char* w_row(const TableView& t, u64 row) { return t.w + row * t.w_pitch; }
// The accumulator(s) of row `row`.
__device__ __forceinline__ float* acc_row(const TableView& t, u64 row) {
  return reinterpret_cast<float*>(t.acc + row * t.acc_pitch);
}
// Element j of row `row`.
__device__ __forceinline__ float load_w(const TableView& t, u64 row, u32 j) {
  if (t.bf16) return bf16_value(reinterpret_cast<const unsigned short*>(w_row(t, row))[j]);
  return reinterpret_cast<const float*>(w_row(t, row))[j];
}
__device__ __forceinline__ void store_w(const TableView& t, u64 row, u32 j, float v) {
  if (t.bf16) reinterpret_cast<unsigned short*>(w_row(t, row))[j] = (unsigned short)bf16_nearest(v);
  else reinterpret_cast<float*>(w_row(t, row))[j] = v;
}
// Elements 4*col4 .. 4*col4+3 of row `row` (dim is a multiple of 4: one 16- or 8-byte access).
// Loops that keep several loads in flight take the format as a template argument and
// separate the load from the conversion (a test of t.bf16, or a conversion, between the
// loads makes the compiler wait for each load before it issues the next).
template <bool BF16> struct StoredW4;
template <> struct StoredW4<false> {
  float4 raw = make_float4(0.f, 0.f, 0.f, 0.f);
  __device__ __forceinline__ float4 value() const { return raw; }
};
template <> struct StoredW4<true> {
  uint2 raw = make_uint2(0u, 0u);
  __device__ __forceinline__ float4 value() const {
    return make_float4(bf16_value(raw.x & 0xFFFFu), bf16_value(raw.x >> 16), bf16_value(raw.y & 0xFFFFu),
                       bf16_value(raw.y >> 16));
  }
};
template <bool BF16>
__device__ __forceinline__ StoredW4<BF16> load_stored_w4(const TableView& t, u64 row, u32 col4) {
  StoredW4<BF16> s;
  s.raw = reinterpret_cast<const decltype(s.raw)*>(w_row(t, row))[col4];
  return s;
}
template <bool BF16>
__device__ __forceinline__ float4 load_w4_as(const TableView& t, u64 row, u32 col4) {
  return load_stored_w4<BF16>(t, row, col4).value();
}
__device__ __forceinline__ float4 load_w4(const TableView& t, u64 row, u32 col4) {
  return t.bf16 ? load_w4_as<true>(t, row, col4) : load_w4_as<false>(t, row, col4);
}
__device__ __forceinline__ void store_w4(const TableView& t, u64 row, u32 col4, float4 v) {
  if (t.bf16)
    reinterpret_cast<uint2*>(w_row(t, row))[col4] = make_uint2(bf16_nearest(v.x) | (bf16_nearest(v.y) << 16),
                                                   bf16_nearest(v.z) | (bf16_nearest(v.w) << 16));
  else
    reinterpret_cast<float4*>(w_row(t, row))[col4] = v;
}

constexpr int kProbeThreads = 256;
constexpr int kProbeGroups = kProbeThreads / kSlotsPerLine;   // insert: 8-lane groups per block
constexpr int kProbeInFlight = 8;                             // keys a group probes at a time
// Lookups take four lanes per key, each reading two of the line's eight slots with one
// 16-byte load: a wave's load instruction then asks for sixteen lines instead of eight, and
// the rate at which lines come back follows the lines asked for per instruction.
constexpr int kLookupLanes = 4;
// Keys a group of the pull's lookup has in flight, a multiple of the lanes of a group (two, four
// and eight were measured: two and four run alike, eight needs too many registers: 158, three
// waves per SIMD, a third slower; forcing five or six waves per SIMD by spilling gains nothing).
constexpr int kPullInFlight = 4;
static_assert(kPullInFlight % kLookupLanes == 0, "every lane of a group owns the same number of keys");
constexpr int kLookupGroups = kProbeThreads / kLookupLanes;
constexpr int kProbeMaxBlocks = 1024;
constexpr u32 kNoSlot = ~0u;
constexpr u32 kMissLdsCap = 2048;        // missing keys a block can list per lookup
constexpr u32 kNewLdsCap = 1024;         // created keys a block lists for its common initialisation
constexpr u32 kLongLdsCap = 64;          // very frequent keys whose chunk items a block writes together
constexpr u32 kMedLdsCap = 512;          // medium keys a block buffers before it appends
constexpr u32 kShortSeg = 16;            // occurrences handled serially by one lane group
constexpr u32 kMedSeg = 512;             // occurrences handled by one wave
constexpr u32 kChunk = 1024;             // occurrences per queued chunk of a longer key

// What the pull leaves for the push about keys that occur often (push.hpp): keys with
// kShortSeg < occurrences <= kMedSeg go to a sharded list (shard b % 64 for block b,
// med_cap entries per shard), keys with more are cut into chunks of kChunk positions.
struct OftenLists {
  const u32* seg_off;
  PullCtx* ctx;
  u32* med_list;
  u32 med_cap;
  uint2* long_list;     // (unique index, first chunk item)
  uint2* chunk_items;   // (unique index, chunk number)
  HeavyRaw* heavy_raw;  // keys with at least heavy_min occurrences are listed for the next dedup
  u32 heavy_min;
  uint2* hot_list;      // (unique index, row) of keys with at least hot_min occurrences, for the pooling kernel
  u32 hot_min;
  u32 hot_cap;
  // Host memory (or null) that receives serial | flags << 32 about the dedup before this
  // lookup: kReportBucket = it took the bucket form, kReportSlow = and more than 1/8 of
  // the occurrences lay in regions that had to be ordered through global memory,
  // kReportOneKey = most of them in regions that one key fills at least half of (keys
  // that turned frequent without warning, which the next hint will list; otherwise the
  // keys do not suit the buckets); kReportMixed = it took the plain form and more places
  // than fix_mixed_runs can note had different keys agreeing in all sorted bits (keys in
  // clusters far apart), so that one workgroup had to put the whole array in order.  The host looks at it when it chooses the form of a later dedup, without
  // waiting for it.
  unsigned long long* report;
  u32 serial;
};
constexpr u32 kReportBucket = 1, kReportSlow = 2, kReportOneKey = 4, kReportMixed = 8;

// "Updated since the last dirty dump" is kept in the sign bit of a row's first
// accumulator element: accumulators are sums of squares, never negative, so the bit
// is free, and the push rewrites that element anyway -- marking costs no traffic.
// Every reader takes the absolute value.
__device__ __forceinline__ float acc_value(float stored) { return fabsf(stored); }
__device__ __forceinline__ float acc_marked(float value) {
  return __uint_as_float(__float_as_uint(value) | 0x80000000u);
}
__device__ __forceinline__ bool acc_is_marked(float stored) {
  return (__float_as_uint(stored) & 0x80000000u) != 0;
}

// One step of a bitonic sorting network over words[0, size), size a power of two; all threads
// of a block of 256, a barrier before every step.  GLOBAL: the words live in global memory
// and are read and written with device-scope accesses, so that what one wave wrote before the
// barrier is what another reads after it.
template <bool GLOBAL>
__device__ __forceinline__ void bitonic_sort_256(u64* words, u32 size) {
  const u32 tid = threadIdx.x;
  for (u32 k = 2; k <= size; k <<= 1) {
    for (u32 j = k >> 1; j > 0; j >>= 1) {
      if (GLOBAL) __threadfence();
      __syncthreads();
      for (u32 i = tid; i < size; i += 256) {
        const u32 partner = i ^ j;
        if (partner > i) {
          u64 x, y;
          if (GLOBAL) {
            x = __hip_atomic_load(words + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            y = __hip_atomic_load(words + partner, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          } else {
            x = words[i];
            y = words[partner];
          }
          const bool up = (i & k) == 0;
          if ((x > y) == up) {
            if (GLOBAL) {
              __hip_atomic_store(words + i, y, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
              __hip_atomic_store(words + partner, x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            } else {
              words[i] = y;
              words[partner] = x;
            }
          }
        }
      }
    }
  }
  if (GLOBAL) __threadfence();
  __syncthreads();
}

// Called by all threads of one block (exactly 256) once lookup `slot`'s list of frequent
// keys is complete: orders it into the ring's set and empties the next list.  A list of fewer
// than kHalfHeavy keys (nearly always) is put in order in LDS in one go; a longer one as two halves,
// each ordered in LDS and parked in the raw list's own storage (which nobody reads again before
// it is refilled), then merged: every element finds its place by a binary search in the other
// half.
constexpr u32 kHalfHeavy = (kMaxHeavy + 1) / 2;
__device__ __forceinline__ void finalize_heavy(HeavyRing* ring, u32 slot) {
  constexpr u32 kSize = kMaxHeavy + 1;             // a power of two
  __shared__ u64 sorted[kHalfHeavy];
  const u32 tid = threadIdx.x;
  HeavyRaw& raw = ring->raw[slot];
  HeavySet& set = ring->set[slot];
  const u32 count = min(raw.count, (u32)kMaxHeavy);
  const bool small = count < kHalfHeavy;
  if (small) {
    // the smallest power of two that holds the listed keys (the order of equal keys does not
    // matter; everything behind is all-ones already)
    u32 size = 2;
    while (size < count) size <<= 1;
    for (u32 i = tid; i < kHalfHeavy; i += 256) sorted[i] = i < count ? raw.keys[i] : ~0ull;
    bitonic_sort_256<false>(sorted, size);
    for (u32 i = tid; i < kSize; i += 256) set.keys[i] = i < kHalfHeavy ? sorted[i] : ~0ull;
  } else {
    for (u32 half = 0; half < 2; ++half) {
      u64* part = raw.keys + half * kHalfHeavy;
      for (u32 i = tid; i < kHalfHeavy; i += 256) sorted[i] = half * kHalfHeavy + i < count ? part[i] : ~0ull;
      bitonic_sort_256<false>(sorted, kHalfHeavy);
      for (u32 i = tid; i < kHalfHeavy; i += 256) part[i] = sorted[i];
      __syncthreads();
    }
    __threadfence();
    __syncthreads();
    // merge: an element's place = its index in its own half + the number of elements of the
    // other half before it (equal elements: those of the first half first)
    for (u32 e = tid; e < kSize; e += 256) {
      const bool second = e >= kHalfHeavy;
      const u32 i = second ? e - kHalfHeavy : e;
      const u64* mine = raw.keys + (second ? kHalfHeavy : 0);
      const u64* other = raw.keys + (second ? 0 : kHalfHeavy);
      const u64 x = __hip_atomic_load(mine + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      u32 m = 0;
#pragma unroll
      for (u32 step = kHalfHeavy / 2; step >= 1; step >>= 1) {
        const u64 y = __hip_atomic_load(other + m + step - 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (second ? y <= x : y < x) m += step;
      }
      // (m counts the elements other[0 .. m) that go before x; at most kHalfHeavy - 1 can be
      // found this way, the last one is looked at separately)
      const u64 last = __hip_atomic_load(other + kHalfHeavy - 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (m == kHalfHeavy - 1 && (second ? last <= x : last < x)) m = kHalfHeavy;
      set.keys[i + m] = x;
    }
    __threadfence();
    __syncthreads();
  }
  // spans: thread t takes top-bit values 4t .. 4t+3
  u32 first[5];
#pragma unroll
  for (int e = 0; e < 5; ++e) {
    const u32 v = 4 * tid + e;
    u32 m = count;
    if (v < (1u << kHeavyTopBits)) {
      const u64 bound = (u64)v << (64 - kHeavyTopBits);
      m = 0;
      if (small) {
#pragma unroll
        for (u32 step = kHalfHeavy / 2; step >= 1; step >>= 1)     // the all-ones padding is never below
          if (sorted[m + step - 1] < bound) m += step;
      } else {
#pragma unroll
        for (u32 step = kSize / 2; step >= 1; step >>= 1)
          if (__hip_atomic_load(set.keys + m + step - 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < bound) m += step;
      }
    }
    first[e] = m;
  }
#pragma unroll
  for (int e = 0; e < 4; ++e) set.span[4 * tid + e] = first[e] | ((first[e + 1] - first[e]) << 16);
  if (tid == 0) {
    set.count = count;
    ring->raw[(slot + 1) % kHeavyRing].count = 0;
  }
}

// No mini-batch seen yet: no heavy keys.
__global__ void __launch_bounds__(256) init_heavy_set(HeavySet* set) {
  for (u32 i = threadIdx.x; i <= (u32)kMaxHeavy; i += 256) set->keys[i] = ~0ull;
  for (u32 i = threadIdx.x; i < (1u << kHeavyTopBits); i += 256) set->span[i] = 0;
  if (threadIdx.x == 0) set->count = 0;
}

// Bits of a wave-wide ballot that belong to this lane's 8-lane group.
__device__ __forceinline__ u32 group_bits(u64 ballot) {
  return (u32)(ballot >> (lane_id() & ~7u)) & 0xFFu;
}

__device__ __forceinline__ u64 load_slot_key(const u64* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Fill kernels (no memset nodes: safe to capture in a graph).
__global__ void __launch_bounds__(256) fill_u64(u64* __restrict__ p, u64 n, u64 v) {
  for (u64 i = (u64)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (u64)gridDim.x * blockDim.x)
    p[i] = v;
}
__global__ void __launch_bounds__(64) reset_state(TableState* st) {
  if (threadIdx.x == 0) {
    st->size = 0;
    st->inserted = 0;
    st->error = 0;
    st->absent = 0;
    st->dump_count = 0;
  }
  if (threadIdx.x < kCountShards) st->miss_shard[threadIdx.x] = st->made_shard[threadIdx.x] = 0;
  if (threadIdx.x == 0) st->miss_overflow = 0;
}
__global__ void __launch_bounds__(64) clear_error(TableState* st) {
  if (threadIdx.x == 0) { st->error = 0; st->miss_overflow = 0; }
  if (threadIdx.x < kCountShards) st->miss_shard[threadIdx.x] = st->made_shard[threadIdx.x] = 0;
}
__global__ void clear_dump_count(TableState* st) { st->dump_count = 0; }
__global__ void __launch_bounds__(64) set_ctx_empty(PullCtx* ctx, u32* seg_off) {
  if (threadIdx.x == 0) {
    ctx->n_unique = 0;
    ctx->n_long = 0;
    ctx->n_chunk_items = 0;
    ctx->n_evidence = 0;
    ctx->sort_error = 0;
    ctx->n_slow = 0;
    ctx->n_slow_one_key = 0;
    ctx->n_hot = 0;
    ctx->n_total = 0;
    ctx->by_id = 0;
    seg_off[0] = 0;
  }
  if (threadIdx.x < kCountShards) ctx->med_count[threadIdx.x] = 0;
}

// Adds the rows insert_missing created to the table size and clears the counters.
// Called by one whole wave, after insert_missing has finished.
__device__ __forceinline__ void commit_insert_wave(TableState* st) {
  const u32 lane = lane_id();
  u32 made = lane < kCountShards ? st->made_shard[lane] : 0;
#pragma unroll
  for (int d = 1; d < kWave; d <<= 1) made += __shfl_xor(made, d, kWave);
  if (lane < kCountShards) st->miss_shard[lane] = st->made_shard[lane] = 0;
  if (lane == 0) {
    st->size += made;
    st->inserted = made;
    st->miss_overflow = 0;
  }
}
__global__ void __launch_bounds__(64) commit_insert(TableState* st) { commit_insert_wave(st); }

// After a lookup that creates nothing (accumulate): the number of keys not found
// goes to st->absent, the counters are cleared.
__global__ void __launch_bounds__(256) commit_absent(TableState* st, HeavyRing* ring, u32 slot) {
  if (ring) finalize_heavy(ring, slot);
  if (threadIdx.x >= kWave) return;
  const u32 lane = lane_id();
  u32 missing = lane < kCountShards ? st->miss_shard[lane] : 0;
#pragma unroll
  for (int d = 1; d < kWave; d <<= 1) missing += __shfl_xor(missing, d, kWave);
  if (lane < kCountShards) st->miss_shard[lane] = 0;
  if (lane == 0) {
    st->absent = (int)missing;
    st->miss_overflow = 0;
  }
}

// Walks key's probe sequence from `line` on.  Returns the slot of the key, or
// kNoRow with `line` left at the first line that has a free slot (slot_key holds
// this lane's slot of that line).  All 8 lanes of the group call it together.
// No kernel that calls it changes slot keys, so plain (cacheable) loads are enough.
__device__ __forceinline__ u32 probe_find(const TableView& t, u64 key, u32 sub, u64& line,
                                          u64& slot_key) {
  for (u64 step = 0; step < t.n_lines; ++step) {
    const u32 hit = group_bits(__ballot(slot_key == key));
    if (hit) return (u32)(line * kSlotsPerLine + (__ffs(hit) - 1));
    if (group_bits(__ballot(slot_key == kEmptyKey))) return kNoRow;
    line = line + 1 == t.n_lines ? 0 : line + 1;
    slot_key = t.keys[line * kSlotsPerLine + sub];
  }
  return kNoRow;
}

// Where a key's probe sequence starts: an even line (n_lines is even), so that a 128-byte
// memory line holds the first two lines of the sequence.
__device__ __forceinline__ u64 home_line(const TableView& t, u64 key) {
  return 2 * __umul64hi(slot_hash(key), t.n_lines >> 1);
}

// The same for a group of kLookupLanes lanes: lane `sub` holds slots 2 * sub and 2 * sub + 1 of
// the line in `pair`.
__device__ __forceinline__ u32 group4_bits(u64 ballot) {
  return (u32)(ballot >> (lane_id() & ~3u)) & 0xFu;
}
__device__ __forceinline__ ulonglong2 load_slot_pair(const TableView& t, u64 line, u32 sub) {
  return reinterpret_cast<const ulonglong2*>(t.keys)[line * (kSlotsPerLine / 2) + sub];
}
__device__ __forceinline__ u32 probe_find4(const TableView& t, u64 key, u32 sub, u64& line,
                                           ulonglong2& pair) {
  for (u64 step = 0; step < t.n_lines; ++step) {
    // bit s: lane s's first slot, bit 4 + s: its second
    const u32 hit = group4_bits(__ballot(pair.x == key)) | (group4_bits(__ballot(pair.y == key)) << 4);
    if (hit) {
      const u32 b = __ffs(hit) - 1;
      return (u32)(line * kSlotsPerLine + 2 * (b & 3u) + (b >> 2));
    }
    if (group4_bits(__ballot(pair.x == kEmptyKey || pair.y == kEmptyKey))) return kNoRow;
    line = line + 1 == t.n_lines ? 0 : line + 1;
    pair = load_slot_pair(t, line, sub);
  }
  return kNoRow;
}

// Finds the key or claims a free slot for it.  *created tells which.
__device__ __forceinline__ u32 probe_find_or_claim(const TableView& t, u64 key, u32 sub, u64 line,
                                                   u64 slot_key, bool* created) {
  *created = false;
  for (u64 step = 0; step < 2 * t.n_lines; ++step) {
    const u32 hit = group_bits(__ballot(slot_key == key));
    if (hit) return (u32)(line * kSlotsPerLine + (__ffs(hit) - 1));
    const u32 free_slots = group_bits(__ballot(slot_key == kEmptyKey));
    if (free_slots) {
      const u32 target = __ffs(free_slots) - 1;
      u64 seen = 0;
      if (sub == target)
        seen = atomicCAS((unsigned long long*)&t.keys[line * kSlotsPerLine + target],
                         (unsigned long long)kEmptyKey, (unsigned long long)key);
      seen = __shfl(seen, (int)((lane_id() & ~7u) + target), kWave);
      if (seen == kEmptyKey) { *created = true; return (u32)(line * kSlotsPerLine + target); }
      if (seen == key) return (u32)(line * kSlotsPerLine + target);
      slot_key = load_slot_key(&t.keys[line * kSlotsPerLine + sub]);   // another key took it
      continue;
    }
    line = line + 1 == t.n_lines ? 0 : line + 1;
    slot_key = load_slot_key(&t.keys[line * kSlotsPerLine + sub]);
  }
  return kNoRow;
}

// For a group of kLookupLanes lanes, after probe_find4 has returned kNoRow: claims a free slot
// for the key, starting at `line` (whose slots `pair` holds; they may be out of date, the
// compare-and-swap decides).  No other group creates the same key at the same time (the
// keys of a pull are distinct), so only the free slot is raced for.  `seen` is what a first
// compare-and-swap on slot `target` of the line returned (issued by the caller, so that
// several keys' first attempts are in flight together).
__device__ __forceinline__ u32 claim_after4(const TableView& t, u64 key, u32 sub, u64 line, u32 target,
                                            u64 seen) {
  if (seen == kEmptyKey) return (u32)(line * kSlotsPerLine + target);
  for (u64 step = 0; step < 2 * t.n_lines; ++step) {
    // another key took the slot, or the line is full: look at the line as it is now
    const u64 x = load_slot_key(&t.keys[line * kSlotsPerLine + 2 * sub]);
    const u64 y = load_slot_key(&t.keys[line * kSlotsPerLine + 2 * sub + 1]);
    const u32 free_slots = group4_bits(__ballot(x == kEmptyKey)) | (group4_bits(__ballot(y == kEmptyKey)) << 4);
    if (!free_slots) { line = line + 1 == t.n_lines ? 0 : line + 1; continue; }
    const u32 b = __ffs(free_slots) - 1;
    const u32 slot = 2 * (b & 3u) + (b >> 2);
    u64 got = 0;
    if (sub == (b & 3u))
      got = atomicCAS((unsigned long long*)&t.keys[line * kSlotsPerLine + slot],
                      (unsigned long long)kEmptyKey, (unsigned long long)key);
    got = __shfl(got, (int)((lane_id() & ~3u) + (b & 3u)), kWave);
    if (got == kEmptyKey) return (u32)(line * kSlotsPerLine + slot);
  }
  return kNoRow;
}

// MODE 1  bulk insert, initial rows: missing keys counted, nothing written
// MODE 2  bulk insert with values: present keys overwritten, missing keys counted
// MODE 3  get: copy the row out, found flags
// (The pull has a kernel of its own: pull_lookup.)
template <int MODE>
__global__ void __launch_bounds__(kProbeThreads)
lookup_keys(TableView t, const u64* __restrict__ keys, u64 n_keys_host,
            const u32* __restrict__ n_keys_dev,
            const float* __restrict__ w_in, const float* __restrict__ acc_in,
            float* __restrict__ w_out, float* __restrict__ acc_out,
            uint8_t* __restrict__ found_out) {
  __shared__ u32 s_missing;
  const u64 n_keys = n_keys_dev ? (u64)*n_keys_dev : n_keys_host;
  if (load_error(t.st) != 0) return;
  if (threadIdx.x == 0) s_missing = 0;
  __syncthreads();
  const u32 sub = threadIdx.x % kLookupLanes;
  const u64 group = (u64)blockIdx.x * kLookupGroups + threadIdx.x / kLookupLanes;
  const u64 n_groups = (u64)gridDim.x * kLookupGroups;
  u32 missing = 0;
  for (u64 u0 = group; u0 < n_keys; u0 += n_groups * kProbeInFlight) {
    u64 key[kProbeInFlight], line[kProbeInFlight];
    ulonglong2 pair[kProbeInFlight];
#pragma unroll
    for (int k = 0; k < kProbeInFlight; ++k) {
      const u64 u = u0 + (u64)k * n_groups;
      key[k] = u < n_keys ? keys[u] : 0;
      line[k] = home_line(t, key[k]);
    }
#pragma unroll
    for (int k = 0; k < kProbeInFlight; ++k) {
      const u64 u = u0 + (u64)k * n_groups;
      pair[k] = u < n_keys ? load_slot_pair(t, line[k], sub) : make_ulonglong2(0, 0);
    }
#pragma unroll
    for (int k = 0; k < kProbeInFlight; ++k) {
      const u64 u = u0 + (u64)k * n_groups;
      if (u >= n_keys) continue;
      if (key[k] == kEmptyKey) {
        if (MODE != 3) raise_error(t.st, kErrReserved);
        if (MODE == 3 && sub == 0) found_out[u] = 0;
        continue;
      }
      const u32 row = probe_find4(t, key[k], sub, line[k], pair[k]);
      if (row == kNoRow && MODE != 3) ++missing;
      if (MODE == 2 && row != kNoRow) {
        for (u32 j = sub; j < t.dim; j += kLookupLanes) store_w(t, row, j, w_in[u * t.dim + j]);
        float* ar = acc_row(t, row);
        for (u32 j = sub; j < t.acc_len; j += kLookupLanes)
          ar[j] = acc_in ? acc_value(acc_in[u * t.acc_len + j]) : t.init_acc;
      }
      if (MODE == 3) {
        if (sub == 0) found_out[u] = row != kNoRow;
        if (row != kNoRow) {
          for (u32 j = sub; j < t.dim; j += kLookupLanes) w_out[u * t.dim + j] = load_w(t, row, j);
          const float* ar = acc_row(t, row);
          for (u32 j = sub; j < t.acc_len; j += kLookupLanes) acc_out[u * t.acc_len + j] = acc_value(ar[j]);
        }
      }
    }
  }
  if (MODE == 1 || MODE == 2) {
    if (sub == 0 && missing) atomicAdd(&s_missing, missing);
    __syncthreads();
    if (threadIdx.x == 0 && s_missing) atomicAdd(&t.st->miss_shard[blockIdx.x % kCountShards], s_missing);
  }
}

// ---- the pull's lookup -------------------------------------------------------------------
// A key's probe sequence starts at an even line, so that its first two lines are one 128-byte
// memory line (what a miss fetches anyway): four lanes look at those 16 slots at once.
struct BucketSlots {
  ulonglong2 a, b;      // lane sub: slots 2 sub and 2 sub + 1 of the even line (a) and of the odd one (b)
};
__device__ __forceinline__ BucketSlots load_bucket(const TableView& t, u64 line, u32 sub) {
  BucketSlots s;
  s.a = load_slot_pair(t, line, sub);
  s.b = load_slot_pair(t, line + 1, sub);
  return s;
}
__device__ __forceinline__ u32 slot_of_bit(u32 b) { return 2 * (b & 3u) + (b >> 2); }

// Data movement inside a group of four lanes (a quad): full-rate DPP moves, no LDS.
template <int CTRL> __device__ __forceinline__ u32 quad_perm(u32 v) {
  return (u32)__builtin_amdgcn_mov_dpp((int)v, CTRL, 0xF, 0xF, true);
}
// The value lane k of the quad holds (k = 0..3, a constant after unrolling).
__device__ __forceinline__ u32 quad_lane(u32 v, int k) {
  switch (k) {
    case 0: return quad_perm<0x00>(v);
    case 1: return quad_perm<0x55>(v);
    case 2: return quad_perm<0xAA>(v);
    default: return quad_perm<0xFF>(v);
  }
}
__device__ __forceinline__ u64 quad_lane(u64 v, int k) {
  return (u64)quad_lane((u32)v, k) | ((u64)quad_lane((u32)(v >> 32), k) << 32);
}
// Bitwise or over the quad, in every lane.
__device__ __forceinline__ u32 quad_or(u32 v) {
  v |= quad_perm<0xB1>(v);      // lanes 1 0 3 2
  v |= quad_perm<0x4E>(v);      // lanes 2 3 0 1
  return v;
}

// What a bucket holds for a key, as one word in every lane of the group: byte 0 = slots of the
// even line that hold the key, byte 1 = free slots of the even line, bytes 2 and 3 the same for
// the odd line; within a byte, bit b stands for slot 2 * (b & 3) + (b >> 2) (slot_of_bit).
__device__ __forceinline__ u32 bucket_bits(const BucketSlots& s, u64 key, u32 sub) {
  const u32 lo = 1u << sub, hi = 16u << sub;
  u32 m = (s.a.x == key ? lo : 0u) | (s.a.y == key ? hi : 0u);
  m |= (s.a.x == kEmptyKey ? lo << 8 : 0u) | (s.a.y == kEmptyKey ? hi << 8 : 0u);
  m |= (s.b.x == key ? lo << 16 : 0u) | (s.b.y == key ? hi << 16 : 0u);
  m |= (s.b.x == kEmptyKey ? lo << 24 : 0u) | (s.b.y == kEmptyKey ? hi << 24 : 0u);
  return quad_or(m);
}

// rows[u] = the slot of unique key u, for u < *n_keys_dev.  Keys the table does not hold:
//  - create == 0 (accumulate): rows[u] = kNoRow, counted in st->miss_shard;
//  - create != 0 and the table has room for all the keys even if every one of them is new: the
//    key is created right here, with its initial row (the line is at hand, and so are its free
//    slots), counted in st->made_shard;
//  - create != 0 otherwise (a pull that might overfill the table): rows[u] = kNoRow and the key
//    is listed for insert_missing, which creates all the listed keys or none: block b appends to
//    shard b % 64 of miss_list (shard_cap entries each); if a list does not fit, the overflow
//    flag makes insert_missing scan all keys instead.
// Also sorts the keys into the push's work lists by their number of occurrences.
//
// A group of four lanes looks at a bucket at once and has four keys in flight, one per lane:
// each lane loads and hashes its own key and, at the end, stores its own key's row and lists it
// (one key per lane: full waves); in between the group goes through its four keys together.
// Every phase runs for all four keys before the next phase starts: a wave waits for memory once
// per phase and round, not once per key (16 groups share a wave, and nearly always one of them
// has a key that needs the next bucket, or has to be created).
__global__ void __launch_bounds__(kProbeThreads)
pull_lookup(TableView t, const u64* __restrict__ keys, const u32* __restrict__ n_keys_dev,
            u32* __restrict__ rows, u32* __restrict__ miss_list, u32 shard_cap, u32 create,
            u32 new_cap, OftenLists often) {
  // new_cap <= kNewLdsCap: how much of the block's list of created keys is used (all of it,
  // except in tests of what happens when it is full)
  constexpr int K = kPullInFlight;            // keys a group has in flight
  constexpr int OWN = K / kLookupLanes;       // of which each lane owns this many
  __shared__ u32 s_missing, s_base, s_med, s_med_base, s_made, s_new, s_long;
  __shared__ uint4 s_long_list[kLongLdsCap];  // (key, first chunk item, chunks) of the block's very frequent keys
  __shared__ u32 s_list[kMissLdsCap];
  __shared__ u32 s_med_list[kMedLdsCap];
  __shared__ u64 s_new_key[kNewLdsCap];       // keys created by this block, and their rows
  __shared__ u32 s_new_row[kNewLdsCap];
  const u64 n_keys = *n_keys_dev;
  if (often.report && blockIdx.x == 0 && threadIdx.x == 0) {
    const PullCtx* c = often.ctx;
    const u32 flags = (c->by_id ? kReportBucket : 0u) | ((u64)c->n_slow * 8 > c->n_total ? kReportSlow : 0u) |
                      ((u64)c->n_slow_one_key * 2 >= c->n_slow ? kReportOneKey : 0u) |
                      (!c->by_id && c->n_evidence > kMaxEvidence ? kReportMixed : 0u);
    __hip_atomic_store(often.report, (unsigned long long)often.serial | ((unsigned long long)flags << 32),
                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
  }
  if (often.ctx->sort_error != 0) {     // the dedup before this lookup failed
    if (threadIdx.x == 0) raise_error(t.st, kErrInternal);
    return;
  }
  if (load_error(t.st) != 0) return;
  if (threadIdx.x == 0) { s_missing = 0; s_med = 0; s_made = 0; s_new = 0; s_long = 0; }
  __syncthreads();
  // (the size does not change while this kernel runs: every thread decides the same)
  const bool create_here = create && t.st->size + n_keys <= t.capacity;
  const u32 sub = threadIdx.x % kLookupLanes;
  const u32 lane0 = lane_id() & ~3u;          // the group's first lane
  const u64 group = (u64)blockIdx.x * kLookupGroups + threadIdx.x / kLookupLanes;
  const u64 n_groups = (u64)gridDim.x * kLookupGroups;
  u32 made = 0;
  // (the bound is the same for all lanes of a group, so a group stays together)
  for (u64 u0 = group; u0 < n_keys; u0 += n_groups * K) {
    // Key k of the group's K is owned by lane k % 4 (as its number k / 4): that lane keeps the
    // key, where its search stands and its row; the group fetches them from it when needed.
    u64 my_key[OWN], my_line[OWN];
    u32 my_len[OWN], my_row[OWN], my_free[OWN];
#pragma unroll
    for (int o = 0; o < OWN; ++o) {
      const u64 u = u0 + (u64)(o * kLookupLanes + sub) * n_groups;
      my_key[o] = u < n_keys ? keys[u] : kEmptyKey;
      my_len[o] = u < n_keys ? often.seg_off[u + 1] - often.seg_off[u] : 0u;
      if (u < n_keys && my_key[o] == kEmptyKey) raise_error(t.st, kErrReserved);
    }
#pragma unroll
    for (int o = 0; o < OWN; ++o) {
      my_line[o] = home_line(t, my_key[o]);
      my_row[o] = kNoRow;
      my_free[o] = 0;
    }
    u32 open = 0;                 // bit k: key k is still being searched for
    BucketSlots slots[K];
#pragma unroll
    for (int k = 0; k < K; ++k) {
      const u64 key = quad_lane(my_key[k / kLookupLanes], k % kLookupLanes);
      const u64 line = quad_lane(my_line[k / kLookupLanes], k % kLookupLanes);
      if (key != kEmptyKey) {
        open |= 1u << k;
        slots[k] = load_bucket(t, line, sub);
      }
    }
    // rounds: look at the buckets at hand, fetch the next ones for the keys not settled
    u32 to_create = 0;            // bit k: key k is absent; its owner's my_free names the slot for it
    for (u64 step = 0; step < t.n_lines; step += 2) {
#pragma unroll
      for (int k = 0; k < K; ++k) {
        if (!(open >> k & 1u)) continue;
        const int o = k / kLookupLanes;
        const bool mine = sub == (u32)(k % kLookupLanes);
        const u64 key = quad_lane(my_key[o], k % kLookupLanes);
        const u32 bits = bucket_bits(slots[k], key, sub);
        const u32 hit_a = bits & 0xFFu, free_a = (bits >> 8) & 0xFFu;
        const u32 hit_b = (bits >> 16) & 0xFFu, free_b = bits >> 24;
        // (a key sits in the first line of its sequence that had a free slot when it came: if
        // the even line has a free slot the key is not in the odd one)
        if (hit_a) {
          if (mine) my_row[o] = (u32)(my_line[o] * kSlotsPerLine + slot_of_bit(__ffs(hit_a) - 1));
          open &= ~(1u << k);
        } else if (free_a) {
          if (mine) my_free[o] = slot_of_bit(__ffs(free_a) - 1);
          to_create |= 1u << k;
          open &= ~(1u << k);
        } else if (hit_b) {
          if (mine) my_row[o] = (u32)((my_line[o] + 1) * kSlotsPerLine + slot_of_bit(__ffs(hit_b) - 1));
          open &= ~(1u << k);
        } else if (free_b) {
          if (mine) my_free[o] = 8u | slot_of_bit(__ffs(free_b) - 1);
          to_create |= 1u << k;
          open &= ~(1u << k);
        } else if (mine) {
          my_line[o] = my_line[o] + 2 >= t.n_lines ? 0 : my_line[o] + 2;
        }
      }
      if (!__any(open != 0)) break;
#pragma unroll
      for (int k = 0; k < K; ++k) {
        const u64 line = quad_lane(my_line[k / kLookupLanes], k % kLookupLanes);
        if (open >> k & 1u) slots[k] = load_bucket(t, line, sub);
      }
    }
    // keys to create: all first attempts in flight together, then whatever is left of each
    if (create_here && __any(to_create != 0)) {
      u64 seen[K];
#pragma unroll
      for (int o = 0; o < OWN; ++o) my_line[o] += my_free[o] >> 3;        // the line of the free slot
#pragma unroll
      for (int k = 0; k < K; ++k) {
        const int o = k / kLookupLanes;
        const u64 key = quad_lane(my_key[o], k % kLookupLanes);
        const u64 line = quad_lane(my_line[o], k % kLookupLanes);
        const u32 slot = quad_lane(my_free[o], k % kLookupLanes) & 7u;
        seen[k] = 0;
        if ((to_create >> k & 1u) && sub == slot >> 1)
          seen[k] = atomicCAS((unsigned long long*)&t.keys[line * kSlotsPerLine + slot],
                              (unsigned long long)kEmptyKey, (unsigned long long)key);
      }
#pragma unroll
      for (int k = 0; k < K; ++k) {
        const int o = k / kLookupLanes;
        const u64 key = quad_lane(my_key[o], k % kLookupLanes);
        const u64 line = quad_lane(my_line[o], k % kLookupLanes);
        const u32 slot = quad_lane(my_free[o], k % kLookupLanes) & 7u;
        if (!(to_create >> k & 1u)) continue;
        const u64 got = __shfl(seen[k], (int)(lane0 + (slot >> 1)), kWave);
        const u32 row = claim_after4(t, key, sub, line, slot, got);
        if (row == kNoRow) {
          raise_error(t.st, kErrInternal);            // (cannot happen: the table has room)
          continue;
        }
        // The new row's initial values are left to the end of the kernel, where all lanes of
        // the block share the work (here four lanes of the wave would do it while sixty wait);
        // only a key that finds the block's list full gets them right away.
        u32 at = 0;
        if (sub == (u32)(k % kLookupLanes)) {
          my_row[o] = row;
          ++made;
          at = atomicAdd(&s_new, 1u);
          if (at < new_cap) { s_new_key[at] = key; s_new_row[at] = row; }
        }
        if (quad_lane(at, k % kLookupLanes) >= new_cap) {
          const u64 base = mix64(key ^ t.init_seed);
          for (u32 j = sub; j < t.dim; j += kLookupLanes) store_w(t, row, j, init_weight(base, j, t.init_range));
          float* ar = acc_row(t, row);
          for (u32 j = sub; j < t.acc_len; j += kLookupLanes) ar[j] = t.init_acc;
        }
      }
    }
    // every lane: the rows of its own keys, and the push's work lists
#pragma unroll
    for (int o = 0; o < OWN; ++o) {
      const u64 u = u0 + (u64)(o * kLookupLanes + sub) * n_groups;
      if (u >= n_keys) continue;
      rows[u] = my_row[o];
      if (my_key[o] == kEmptyKey) continue;
      if (my_row[o] == kNoRow) {
        const u32 at = atomicAdd(&s_missing, 1u);
        if (at < kMissLdsCap) s_list[at] = (u32)u;
      }
      const u32 len = my_len[o];
      if (len >= often.heavy_min) {
        const u32 at = atomicAdd(&often.heavy_raw->count, 1u);
        if (at < (u32)kMaxHeavy) often.heavy_raw->keys[at] = my_key[o];
      }
      if (len >= often.hot_min && my_row[o] != kNoRow) {
        const u32 at = atomicAdd(&often.ctx->n_hot, 1u);
        if (at < often.hot_cap) often.hot_list[at] = make_uint2((u32)u, my_row[o]);
      }
      if (len > kMedSeg) {
        const u32 n_chunks = (len + kChunk - 1) / kChunk;
        const u32 first = atomicAdd(&often.ctx->n_chunk_items, n_chunks);
        often.long_list[atomicAdd(&often.ctx->n_long, 1u)] = make_uint2((u32)u, first);
        // the key's chunk items are written at the end of the kernel by all lanes of the block
        // (a key that fills thousands of chunks would keep this lane, and its wave, for long)
        const u32 at = atomicAdd(&s_long, 1u);
        if (at < kLongLdsCap) {
          s_long_list[at] = make_uint4((u32)u, first, n_chunks, 0u);
        } else {
          for (u32 c = 0; c < n_chunks; ++c) often.chunk_items[first + c] = make_uint2((u32)u, c);
        }
      } else if (len > kShortSeg) {
        const u32 at = atomicAdd(&s_med, 1u);
        if (at < kMedLdsCap) {
          s_med_list[at] = (u32)u;
        } else {      // buffer full: append straight to the shard
          const u32 shard = blockIdx.x % kCountShards;
          const u32 pos = atomicAdd(&often.ctx->med_count[shard], 1u);
          if (pos < often.med_cap) often.med_list[(u64)shard * often.med_cap + pos] = (u32)u;
        }
      }
    }
  }
  if (made) atomicAdd(&s_made, made);
  __syncthreads();
  if (threadIdx.x == 0 && s_made) atomicAdd(&t.st->made_shard[blockIdx.x % kCountShards], s_made);
  {
    const u32 n_long_here = min(s_long, kLongLdsCap);
    for (u32 e = 0; e < n_long_here; ++e) {
      const uint4 it = s_long_list[e];
      for (u32 c = threadIdx.x; c < it.z; c += kProbeThreads) often.chunk_items[it.y + c] = make_uint2(it.x, c);
    }
  }
  // the initial rows of the keys created above: one float4 of one row per lane and turn
  const u32 n_new = min(s_new, new_cap);
  const u32 dim4 = t.dim >> 2;
  for (u32 e = threadIdx.x; e < n_new * dim4; e += kProbeThreads) {
    const u32 i = e / dim4, col = e % dim4;
    const u64 base = mix64(s_new_key[i] ^ t.init_seed);
    store_w4(t, s_new_row[i], col,
             make_float4(init_weight(base, 4 * col, t.init_range), init_weight(base, 4 * col + 1, t.init_range),
                         init_weight(base, 4 * col + 2, t.init_range), init_weight(base, 4 * col + 3, t.init_range)));
  }
  for (u32 e = threadIdx.x; e < n_new * t.acc_len; e += kProbeThreads)
    acc_row(t, s_new_row[e / t.acc_len])[e % t.acc_len] = t.init_acc;
  const u32 n_med = min(s_med, kMedLdsCap);
  if (n_med) {
    const u32 shard = blockIdx.x % kCountShards;
    if (threadIdx.x == 0) s_med_base = atomicAdd(&often.ctx->med_count[shard], n_med);
    __syncthreads();
    for (u32 i = threadIdx.x; i < n_med; i += kProbeThreads)
      if (s_med_base + i < often.med_cap)
        often.med_list[(u64)shard * often.med_cap + s_med_base + i] = s_med_list[i];
  }
  const u32 cnt = s_missing;
  if (cnt == 0) return;
  if (threadIdx.x == 0) s_base = atomicAdd(&t.st->miss_shard[blockIdx.x % kCountShards], cnt);
  __syncthreads();
  const u32 base = s_base;
  if (cnt > kMissLdsCap || base + cnt > shard_cap) {
    if (threadIdx.x == 0) t.st->miss_overflow = 1;
    return;
  }
  u32* dst = miss_list + (u64)(blockIdx.x % kCountShards) * shard_cap + base;
  for (u32 i = threadIdx.x; i < cnt; i += kProbeThreads) dst[i] = s_list[i];
}

// Creates the keys lookup_keys found missing, if the table has room for all of them
// (a key that occurs twice in a bulk insert is counted twice for this check).
// rows != null (pull): the listed missing keys are visited (or, after a list overflow,
// all keys with rows[u] == kNoRow); rows[u] is set.
// rows == null (bulk insert): every key is probed again.
// w_in == null: new rows get the deterministic initial row; else the given values.
__global__ void __launch_bounds__(kProbeThreads)
insert_missing(TableView t, const u64* __restrict__ keys, u64 n_keys_host,
               const u32* __restrict__ n_keys_dev, u32* __restrict__ rows,
               const float* __restrict__ w_in, const float* __restrict__ acc_in,
               const u32* __restrict__ miss_list, u32 shard_cap) {
  __shared__ u32 s_total, s_made, s_mine;
  const u32 block = blockIdx.x, n_blocks = gridDim.x;
  if (load_error(t.st) != 0) return;
  if (threadIdx.x < kWave) {
    const u32 mine = threadIdx.x < kCountShards ? t.st->miss_shard[threadIdx.x] : 0;
    u32 c = mine;
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) c += __shfl_xor(c, d, kWave);
    if (threadIdx.x == 0) { s_total = c; s_made = 0; }
    if (threadIdx.x == block % kCountShards) s_mine = mine;
  }
  __syncthreads();
  const u32 total = s_total;
  if (total == 0) return;
  // st->size does not change while this kernel runs: every block decides the same
  if (t.st->size + total > t.capacity) {
    if (threadIdx.x == 0) raise_error(t.st, kErrFull);
    return;
  }
  const u64 n_keys = n_keys_dev ? (u64)*n_keys_dev : n_keys_host;
  const u32 sub = threadIdx.x & 7;
  const u64 group = (u64)block * kProbeGroups + (threadIdx.x >> 3);
  const u64 n_groups = (u64)n_blocks * kProbeGroups;
  u32 made = 0;
  const bool listed = rows != nullptr && t.st->miss_overflow == 0;
  // listed: this block's share of its shard's list; else every key
  const u32 shard = block % kCountShards;
  const u32 shard_blocks = (n_blocks - shard + kCountShards - 1) / kCountShards;
  const u64 first = listed ? (u64)(block / kCountShards) * kProbeGroups + (threadIdx.x >> 3) : group;
  const u64 stride = listed ? (u64)shard_blocks * kProbeGroups : n_groups;
  const u64 count = listed ? (u64)s_mine : n_keys;
  for (u64 e = first; e < count; e += stride) {
    const u64 u = listed ? (u64)miss_list[(u64)shard * shard_cap + e] : e;
    if (!listed && rows && rows[u] != kNoRow) continue;
    const u64 key = keys[u];
    if (key == kEmptyKey) continue;
    const u64 line = home_line(t, key);
    const u64 slot_key = load_slot_key(&t.keys[line * kSlotsPerLine + sub]);
    bool created;
    const u32 row = probe_find_or_claim(t, key, sub, line, slot_key, &created);
    if (rows && sub == 0) rows[u] = row;
    if (!created) continue;
    ++made;
    float* ar = acc_row(t, row);
    if (w_in) {
      for (u32 j = sub; j < t.dim; j += 8) store_w(t, row, j, w_in[u * t.dim + j]);
      for (u32 j = sub; j < t.acc_len; j += 8)
        ar[j] = acc_in ? acc_value(acc_in[u * t.acc_len + j]) : t.init_acc;
    } else {
      const u64 base = mix64(key ^ t.init_seed);
      for (u32 j = sub; j < t.dim; j += 8) store_w(t, row, j, init_weight(base, j, t.init_range));
      for (u32 j = sub; j < t.acc_len; j += 8) ar[j] = t.init_acc;
    }
  }
  if (sub == 0 && made) atomicAdd(&s_made, made);
  __syncthreads();
  if (threadIdx.x == 0 && s_made) atomicAdd(&t.st->made_shard[block % kCountShards], s_made);
}

// dump: every occupied slot (DIRTY: every occupied slot whose row is marked as
// updated; the mark of a row that is written out is cleared), compacted through one
// counter per block of slots (order unspecified).
template <bool DIRTY>
__global__ void __launch_bounds__(256)
dump_rows(TableView t, u64* __restrict__ keys_out, float* __restrict__ w_out,
          float* __restrict__ acc_out, u64 max_rows, unsigned long long* __restrict__ counter) {
  __shared__ u32 scratch[256 / kWave + 1];
  __shared__ unsigned long long s_base;
  const u64 n_slots = t.n_lines * kSlotsPerLine;
  const u64 n_rounds = (n_slots + 255) / 256;
  for (u64 round = blockIdx.x; round < n_rounds; round += gridDim.x) {
    const u64 s = round * 256 + threadIdx.x;
    const u64 key = s < n_slots ? t.keys[s] : kEmptyKey;
    bool used = key != kEmptyKey;
    if (DIRTY && used) used = acc_is_marked(*acc_row(t, s));
    u32 total;
    const u32 before = block_excl_sum<256>(used ? 1u : 0u, scratch, &total);
    if (threadIdx.x == 0 && total) s_base = atomicAdd(counter, (unsigned long long)total);
    __syncthreads();
    if (used) {
      const u64 o = s_base + before;
      if (o < max_rows) {
        keys_out[o] = key;
        for (u32 j = 0; j < t.dim; ++j) w_out[o * t.dim + j] = load_w(t, s, j);
        for (u32 j = 0; j < t.acc_len; ++j) acc_out[o * t.acc_len + j] = acc_value(acc_row(t, s)[j]);
        if (DIRTY) *acc_row(t, s) = acc_value(*acc_row(t, s));
      }
    }
    __syncthreads();
  }
}

// How many buckets (pairs of lines: 128 bytes) a lookup reads to find each stored key (1 = the
// key sits in the bucket its hash names): sum and maximum over all stored keys, into st->probe_sum / probe_max (zero on
// entry).
__global__ void __launch_bounds__(256) probe_length_scan(TableView t) {
  __shared__ unsigned long long s_sum, s_max;
  if (threadIdx.x == 0) { s_sum = 0; s_max = 0; }
  __syncthreads();
  const u64 n_slots = t.n_lines * kSlotsPerLine;
  unsigned long long sum = 0, most = 0;
  for (u64 s = (u64)blockIdx.x * blockDim.x + threadIdx.x; s < n_slots; s += (u64)gridDim.x * blockDim.x) {
    const u64 key = t.keys[s];
    if (key == kEmptyKey) continue;
    const u64 home = home_line(t, key), line = s / kSlotsPerLine;
    const u64 lines = (line >= home ? line - home : line + t.n_lines - home) / 2 + 1;
    sum += lines;
    most = max(most, (unsigned long long)lines);
  }
#pragma unroll
  for (int d = 1; d < kWave; d <<= 1) {
    sum += __shfl_xor(sum, d, kWave);
    most = max(most, (unsigned long long)__shfl_xor(most, d, kWave));
  }
  if (lane_id() == 0) { atomicAdd(&s_sum, sum); atomicMax(&s_max, most); }
  __syncthreads();
  if (threadIdx.x == 0) { atomicAdd(&t.st->probe_sum, s_sum); atomicMax(&t.st->probe_max, s_max); }
}
__global__ void clear_probe_lengths(TableState* st) { st->probe_sum = 0; st->probe_max = 0; }

}  // namespace hps
