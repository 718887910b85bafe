// The HBM hash table: open addressing over 64-byte lines of 8 slots, linear
// probing line by line, one 8-lane group per key (each lane looks at one slot of
// the line), lock-free insertion by 64-bit compare-and-swap on the slot's key.
//
// Layout (structure of arrays, row index = slot index):
//   keys[n_slots]            u64, kEmptyKey when free
//   w[n_slots][dim]          f32
//   acc[n_slots][acc_len]    f32
#pragma once

#include "common.cuh"

namespace hps {

struct TableView {
  u64* keys;
  float* w;
  float* acc;
  TableState* st;
  u64 n_lines;      // n_slots / 8
  u64 capacity;
  u32 dim;
  u32 acc_len;
  float init_acc;
  float init_range;
  u64 init_seed;
};

constexpr int kProbeThreads = 256;
constexpr int kProbeGroups = kProbeThreads / kSlotsPerLine;   // keys in flight per block
constexpr int kProbeKeysPerGroup = 4;
constexpr int kProbeKeysPerBlock = kProbeGroups * kProbeKeysPerGroup;

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
__global__ void __launch_bounds__(256) fill_f32(float* __restrict__ p, u64 n, float v) {
  for (u64 i = (u64)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (u64)gridDim.x * blockDim.x)
    p[i] = v;
}
__global__ void reset_state(TableState* st) {
  st->size = 0;
  st->inserted = 0;
  st->error = 0;
  st->pad = 0;
  st->dump_count = 0;
}
__global__ void clear_error(TableState* st) { st->error = 0; }
__global__ void clear_inserted(TableState* st) { st->inserted = 0; }
__global__ void clear_dump_count(TableState* st) { st->dump_count = 0; }
__global__ void set_ctx_empty(PullCtx* ctx, u32* seg_off) {
  ctx->n_unique = 0;
  ctx->n_long = 0;
  ctx->n_chunk_items = 0;
  ctx->n_evidence = 0;
  ctx->sort_error = 0;
  seg_off[0] = 0;
}

// Look up `n_keys` keys (the count is read from *n_keys_dev when that pointer is
// not null, so that a pull needs no host round trip for U); MODE:
//   0  find only                       -> rows[u] = slot or kNoRow
//   1  find or insert the initial row  -> rows[u] = slot (kNoRow if the table is full)
//   2  insert/overwrite given values   -> rows[u] = slot
//   3  find and copy the row out        -> w_out[u], acc_out[u], found_out[u]
// In modes 1 and 2 the keys handed to one block's groups are first looked up, the
// block then reserves room for all its missing keys with ONE atomic add on the
// table size, and only then claims slots.
template <int MODE>
__global__ void __launch_bounds__(kProbeThreads)
probe_keys(TableView t, const u64* __restrict__ keys, u64 n_keys_host,
           const u32* __restrict__ n_keys_dev, u32* __restrict__ rows,
           const float* __restrict__ w_in, const float* __restrict__ acc_in,
           float* __restrict__ w_out, float* __restrict__ acc_out,
           uint8_t* __restrict__ found_out) {
  __shared__ u32 s_need;
  __shared__ int s_ok;
  const u64 n_keys = n_keys_dev ? (u64)*n_keys_dev : n_keys_host;
  const u64 block_first = (u64)blockIdx.x * kProbeKeysPerBlock;
  if (block_first >= n_keys) return;
  if (load_error(t.st) != 0) return;
  if (threadIdx.x == 0) { s_need = 0; s_ok = 1; }
  __syncthreads();

  const u32 sub = threadIdx.x & 7;
  const u32 group = threadIdx.x >> 3;
  u64 key[kProbeKeysPerGroup];
  u64 line[kProbeKeysPerGroup];
  u64 slot_key[kProbeKeysPerGroup];
  u32 row[kProbeKeysPerGroup];
  bool live[kProbeKeysPerGroup];

#pragma unroll
  for (int k = 0; k < kProbeKeysPerGroup; ++k) {
    const u64 u = block_first + (u64)k * kProbeGroups + group;
    live[k] = u < n_keys;
    key[k] = live[k] ? keys[u] : 0;
    line[k] = __umul64hi(slot_hash(key[k]), t.n_lines);
    row[k] = kNoRow;
    slot_key[k] = live[k] ? load_slot_key(&t.keys[line[k] * kSlotsPerLine + sub]) : 0;
  }

  // Phase 1: walk each key's probe sequence to its match or to the first line with a free slot.
  u32 missing = 0;
#pragma unroll
  for (int k = 0; k < kProbeKeysPerGroup; ++k) {
    if (!live[k]) continue;
    if (key[k] == kEmptyKey) { raise_error(t.st, kErrReserved); live[k] = false; continue; }
    for (u64 step = 0; step < t.n_lines; ++step) {
      const u32 hit = group_bits(__ballot(slot_key[k] == key[k]));
      if (hit) { row[k] = (u32)(line[k] * kSlotsPerLine + (__ffs(hit) - 1)); break; }
      const u32 free_slots = group_bits(__ballot(slot_key[k] == kEmptyKey));
      if (free_slots) break;
      line[k] = line[k] + 1 == t.n_lines ? 0 : line[k] + 1;
      slot_key[k] = load_slot_key(&t.keys[line[k] * kSlotsPerLine + sub]);
    }
    if (row[k] == kNoRow) ++missing;
  }

  if (MODE == 1 || MODE == 2) {
    if (sub == 0 && missing) atomicAdd(&s_need, missing);
    __syncthreads();
    if (threadIdx.x == 0 && s_need) {
      const unsigned long long before = atomicAdd(&t.st->size, (unsigned long long)s_need);
      if (before + s_need > t.capacity) {
        atomicAdd(&t.st->size, (unsigned long long)(-(long long)s_need));
        raise_error(t.st, kErrFull);
        s_ok = 0;
      } else {
        atomicAdd(&t.st->inserted, (unsigned long long)s_need);
      }
    }
    __syncthreads();

    // Phase 2: claim a slot for each missing key.
#pragma unroll
    for (int k = 0; k < kProbeKeysPerGroup; ++k) {
      if (!live[k] || row[k] != kNoRow || !s_ok) continue;
      bool created = false;
      for (u64 step = 0; step < 2 * t.n_lines; ++step) {
        const u32 hit = group_bits(__ballot(slot_key[k] == key[k]));
        if (hit) { row[k] = (u32)(line[k] * kSlotsPerLine + (__ffs(hit) - 1)); break; }
        const u32 free_slots = group_bits(__ballot(slot_key[k] == kEmptyKey));
        if (free_slots) {
          const u32 target = __ffs(free_slots) - 1;
          u64 seen = 0;
          if (sub == target)
            seen = atomicCAS((unsigned long long*)&t.keys[line[k] * kSlotsPerLine + target],
                             (unsigned long long)kEmptyKey, (unsigned long long)key[k]);
          seen = __shfl(seen, (lane_id() & ~7u) + target, kWave);
          if (seen == kEmptyKey) {
            row[k] = (u32)(line[k] * kSlotsPerLine + target);
            created = true;
            break;
          }
          if (seen == key[k]) { row[k] = (u32)(line[k] * kSlotsPerLine + target); break; }
          // another key took the slot: look at the line again
          slot_key[k] = load_slot_key(&t.keys[line[k] * kSlotsPerLine + sub]);
          continue;
        }
        line[k] = line[k] + 1 == t.n_lines ? 0 : line[k] + 1;
        slot_key[k] = load_slot_key(&t.keys[line[k] * kSlotsPerLine + sub]);
      }
      if (!created && sub == 0) {
        // the key turned out to be present (duplicate in a bulk insert): give the room back
        atomicAdd(&t.st->size, (unsigned long long)(-1ll));
        atomicAdd(&t.st->inserted, (unsigned long long)(-1ll));
      }
      if (created && MODE == 1) {
        const u64 base = mix64(key[k] ^ t.init_seed);
        float* wr = t.w + (u64)row[k] * t.dim;
        for (u32 j = sub; j < t.dim; j += 8) wr[j] = init_weight(base, j, t.init_range);
        float* ar = t.acc + (u64)row[k] * t.acc_len;
        for (u32 j = sub; j < t.acc_len; j += 8) ar[j] = t.init_acc;
      }
    }
  }

#pragma unroll
  for (int k = 0; k < kProbeKeysPerGroup; ++k) {
    const u64 u = block_first + (u64)k * kProbeGroups + group;
    if (u >= n_keys) continue;
    if (MODE == 2 && row[k] != kNoRow) {
      float* wr = t.w + (u64)row[k] * t.dim;
      const float* ws = w_in + u * t.dim;
      for (u32 j = sub; j < t.dim; j += 8) wr[j] = ws[j];
      float* ar = t.acc + (u64)row[k] * t.acc_len;
      for (u32 j = sub; j < t.acc_len; j += 8) ar[j] = acc_in ? acc_in[u * t.acc_len + j] : t.init_acc;
    }
    if (MODE == 3) {
      if (sub == 0) found_out[u] = row[k] != kNoRow;
      if (row[k] != kNoRow) {
        const float* wr = t.w + (u64)row[k] * t.dim;
        for (u32 j = sub; j < t.dim; j += 8) w_out[u * t.dim + j] = wr[j];
        const float* ar = t.acc + (u64)row[k] * t.acc_len;
        for (u32 j = sub; j < t.acc_len; j += 8) acc_out[u * t.acc_len + j] = ar[j];
      }
    }
    if (rows && sub == 0) rows[u] = row[k];
  }
}

// dump: every occupied slot, compacted through one counter (order unspecified).
__global__ void __launch_bounds__(256)
dump_rows(TableView t, u64* __restrict__ keys_out, float* __restrict__ w_out,
          float* __restrict__ acc_out, u64 max_rows, unsigned long long* __restrict__ counter) {
  const u64 n_slots = t.n_lines * kSlotsPerLine;
  for (u64 s = (u64)blockIdx.x * blockDim.x + threadIdx.x; s < n_slots + (kWave - 1);
       s += (u64)gridDim.x * blockDim.x) {
    const u64 key = s < n_slots ? t.keys[s] : kEmptyKey;
    const bool used = key != kEmptyKey;
    const u64 m = __ballot(used);
    if (m == 0) continue;
    unsigned long long base = 0;
    if (lane_id() == 0) base = atomicAdd(counter, (unsigned long long)__popcll(m));
    base = __shfl(base, 0, kWave);
    if (!used) continue;
    const u64 o = base + __popcll(m & lanemask_lt());
    if (o >= max_rows) continue;
    keys_out[o] = key;
    for (u32 j = 0; j < t.dim; ++j) w_out[o * t.dim + j] = t.w[s * t.dim + j];
    for (u32 j = 0; j < t.acc_len; ++j) acc_out[o * t.acc_len + j] = t.acc[s * t.acc_len + j];
  }
}

}  // namespace hps
