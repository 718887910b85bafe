// Key dedup, bucket form, part 1: ordering the key occurrences by bucket id without any
// workgroup waiting for another.
//
// A key's bucket id (sort.hpp: bucket_id) has at most 16 bits; the occurrences are ordered by
// it with one or two stable 8-bit passes, least significant byte first.  Each pass is three
// launches, none of which waits for anything but its own input:
//
//   bucket_count / digit_count   every tile (kPartTile consecutive occurrences) counts its
//                                digits; the counts go to a digit-major matrix
//                                hist[digit][tile];
//   scan_tiles                   one workgroup per digit: exclusive prefix over the tiles
//                                (in place) and the digit's total;
//   scatter_pass                 a tile ranks its elements (wave ballots: stable), adds the
//                                tile's prefix and the digit's base, stages the tile in LDS
//                                and writes every digit's run contiguously.
//
// bucket_count also works out the mini-batch's key range (from samples), every key's bucket
// id (id16, read again by the first scatter) and bag_of[i]; the first scatter of a two-pass
// plan leaves the ids' high bytes in sorted order (dig), so that the second pass's count
// reads one byte per occurrence.  region_borders then cuts the ordered array into the
// regions that bucket.hpp finishes.
#pragma once

#include "common.hpp"
#include "sort.hpp"

namespace hps {

constexpr int kPartThreads = 256;
constexpr int kPartWaves = kPartThreads / kWave;
constexpr int kPartItems = 12;                          // per thread
constexpr int kPartTile = kPartThreads * kPartItems;    // 3072 occurrences
constexpr int kPartWaveSpan = kWave * kPartItems;       // 768 consecutive occurrences per wave
constexpr u32 kRegionSpan = 2048;                       // positions between nominal region cuts
static_assert(kPartTile == kSortTile, "the workspace is sized in tiles of kSortTile");
static_assert(kRadix == kPartThreads, "thread d owns digit d");

// First kernel of a bucket-form dedup.  The first count_blocks blocks loop over the tiles:
// bucket id of every key (id16) and the tile's counts of the ids' low bytes
// (hist[digit * n_tiles + tile]); the blocks behind them write bag_of.  Block 0 also resets
// the pull context and the tickets and leaves the key range in ctx->range.
__global__ void __launch_bounds__(kPrepThreads)
bucket_count(const u64* __restrict__ keys, u32 n, SortPlan plan, u32* __restrict__ tickets,
             PullCtx* __restrict__ ctx, const i32* __restrict__ offsets, u32 n_bags,
             i32* __restrict__ bag_of, const HeavySet* __restrict__ heavy_set,
             uint16_t* __restrict__ id16, u32* __restrict__ hist, u32 n_tiles, u32 count_blocks) {
  if (blockIdx.x >= count_blocks) {
    expand_bags(offsets, n_bags, n, bag_of, blockIdx.x - count_blocks, gridDim.x - count_blocks);
    return;
  }
  __shared__ u32 h[kRadix];
  __shared__ HeavyLds hv;
  __shared__ u64 s_lo[kPrepThreads / kWave], s_hi[kPrepThreads / kWave];
  // The block's first tile is requested before anything waits for the samples, so that the
  // two round trips to memory overlap (count_blocks <= n_tiles: every block has a tile).
  u64 first_keys[kPartItems];
#pragma unroll
  for (int k = 0; k < kPartItems; ++k) {
    const u32 i = blockIdx.x * kPartTile + k * kPrepThreads + threadIdx.x;
    first_keys[k] = i < n ? keys[i] : 0;
  }
  sample_key_range(keys, n, s_lo, s_hi);
  load_heavy(hv, heavy_set, plan.max_heavy);
  h[threadIdx.x] = 0;
  if (blockIdx.x == 0) {
    if (threadIdx.x < kMaxPasses + 2) tickets[threadIdx.x] = 0;
    reset_ctx(ctx, n, 1u);
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    u64 lo = s_lo[0], hi = s_hi[0];
    for (int w = 1; w < kPrepThreads / kWave; ++w) { lo = min(lo, s_lo[w]); hi = max(hi, s_hi[w]); }
    if (lo > hi) lo = hi = 0;            // n == 0
    hv.range = make_range(lo, hi, plan);
    if (blockIdx.x == 0) ctx->range = hv.range;
  }
  __syncthreads();
  for (u32 tile = blockIdx.x; tile < n_tiles; tile += count_blocks) {
    const u32 base = tile * kPartTile;
#pragma unroll
    for (int k = 0; k < kPartItems; ++k) {
      const u32 i = base + k * kPrepThreads + threadIdx.x;
      if (i < n) {
        const u64 key = tile == blockIdx.x ? first_keys[k] : keys[i];
        bool heavy;
        const u32 id = bucket_id(key, hv, &heavy);
        id16[i] = (uint16_t)id;
        atomicAdd(&h[id & (kRadix - 1)], 1u);
      }
    }
    __syncthreads();
    hist[(u64)threadIdx.x * n_tiles + tile] = h[threadIdx.x];
    h[threadIdx.x] = 0;
    __syncthreads();
  }
}

// Counts of the second pass: dig[j] is the id's high byte of the occurrence at position j
// after the first pass.  One tile per block.
__global__ void __launch_bounds__(kPartThreads)
digit_count(const uint8_t* __restrict__ dig, u32 n, u32* __restrict__ hist, u32 n_tiles) {
  __shared__ u32 h[kRadix];
  h[threadIdx.x] = 0;
  __syncthreads();
  const u32 tile = blockIdx.x;
  // four consecutive digits per load (tiles start at multiples of four)
  const u32* dig4 = reinterpret_cast<const u32*>(dig);
  const u32 base4 = tile * (kPartTile / 4);
#pragma unroll
  for (int k = 0; k < kPartItems / 4; ++k) {
    const u32 q = base4 + k * kPartThreads + threadIdx.x;
    const u32 i = q * 4;
    if (i + 3 < n) {
      const u32 v = dig4[q];
      atomicAdd(&h[v & 255u], 1u);
      atomicAdd(&h[(v >> 8) & 255u], 1u);
      atomicAdd(&h[(v >> 16) & 255u], 1u);
      atomicAdd(&h[v >> 24], 1u);
    } else {
      for (u32 e = i; e < n; ++e) atomicAdd(&h[dig[e]], 1u);
    }
  }
  __syncthreads();
  hist[(u64)threadIdx.x * n_tiles + tile] = h[threadIdx.x];
}

// One workgroup per digit: hist[digit][0 .. n_tiles) becomes its own exclusive prefix, tot[digit]
// the digit's total.  The launch also clears `n_clear` words at `clear` (status words of the
// kernel that finishes the dedup: nothing of an earlier dedup may be left in them).
__global__ void __launch_bounds__(kPartThreads)
scan_tiles(u32* __restrict__ hist, u32 n_tiles, u32* __restrict__ tot, u32* __restrict__ clear,
           u32 n_clear) {
  __shared__ u32 scratch[kPartThreads / kWave + 1];
  for (u32 i = blockIdx.x * kPartThreads + threadIdx.x; i < n_clear; i += gridDim.x * kPartThreads)
    clear[i] = 0;
  u32* row = hist + (u64)blockIdx.x * n_tiles;
  u32 running = 0;
  for (u32 base = 0; base < n_tiles; base += kPartThreads) {
    const u32 t = base + threadIdx.x;
    const u32 v = t < n_tiles ? row[t] : 0;
    u32 total;
    const u32 ex = block_excl_sum<kPartThreads>(v, scratch, &total);
    if (t < n_tiles) row[t] = running + ex;
    running += total;
  }
  if (threadIdx.x == 0) tot[blockIdx.x] = running;
}

// One stable pass over (key, payload) pairs by one byte of the bucket id; payload =
// occurrence index | bag << 32.  One tile per block.
//   FIRST: reads keys / id16 / bag_of in arrival order, sorts by the id's low byte and, if
//          dig_out is not null (two-pass plan), leaves the high byte of every occurrence at
//          its new position there.
//   else:  reads the pairs and dig_in (the first pass's dig_out), sorts by that byte.
//   hist   [digit][tile] exclusive prefixes and tot[digit] totals of this pass (scan_tiles)
//   ORDERED: how the elements are ranked (sort.hpp: digit_rank)
template <bool FIRST, bool ORDERED>
__global__ void __launch_bounds__(kPartThreads)
scatter_pass(const u64* __restrict__ keys_in, const u64* __restrict__ pay_in,
             const i32* __restrict__ bag_of, const uint16_t* __restrict__ id16,
             const uint8_t* __restrict__ dig_in, u64* __restrict__ keys_out,
             u64* __restrict__ pay_out, uint8_t* __restrict__ dig_out, u32 n,
             const u32* __restrict__ hist, u32 n_tiles, const u32* __restrict__ tot) {
  __shared__ u32 wave_cnt[kPartWaves][kRadix];   // per-wave digit counts, then wave offsets
  __shared__ u32 local_start[kRadix];            // first staged position of each digit
  __shared__ u32 out_base[kRadix];               // global position of the digit's run - local_start
  __shared__ u32 scratch[kPartThreads / kWave + 1];
  __shared__ u64 stage[kPartTile];               // keys first, then the payloads
  __shared__ uint8_t stage_digit[kPartTile];     // digit of each staged element
  __shared__ uint8_t stage_next[kPartTile];      // FIRST: its id's high byte

  const u32 tid = threadIdx.x;
  const u32 tile = blockIdx.x;
  const u32 wave = tid / kWave, lane = tid & (kWave - 1);
  const u32 tile_base = tile * kPartTile;
  const u32 tile_n = min((u32)kPartTile, n - tile_base);
  const u32 wave_base = tile_base + wave * kPartWaveSpan;
#pragma unroll
  for (int w = 0; w < kPartWaves; ++w) wave_cnt[w][tid] = 0;
  // what thread d needs about digit d, requested early
  const u32 tile_prefix = hist[(u64)tid * n_tiles + tile];
  const u32 digit_count_all = tot[tid];

  u64 key[kPartItems];
  u64 pay[kPartItems];
  u32 dg[kPartItems];      // digit | next digit << 8
#pragma unroll
  for (int r = 0; r < kPartItems; ++r) {
    const u32 i = wave_base + r * kWave + lane;
    key[r] = (i < n) ? keys_in[i] : ~0ull;
    if (FIRST) {
      pay[r] = (i < n) ? ((u64)i | ((u64)(u32)bag_of[i] << 32)) : 0ull;
      dg[r] = (i < n) ? (u32)id16[i] : 0u;
    } else {
      pay[r] = (i < n) ? pay_in[i] : 0ull;
      dg[r] = (i < n) ? (u32)dig_in[i] : 0u;
    }
  }
  __syncthreads();
  u32 rank[kPartItems];
  {
    const u64 lt = lanemask_lt();
#pragma unroll
    for (int r = 0; r < kPartItems; ++r) {
      const u32 i = wave_base + r * kWave + lane;
      const u32 d = dg[r] & (kRadix - 1);
      rank[r] = digit_rank<ORDERED>(&wave_cnt[wave][d], d, i < n, lt);
    }
  }
  __syncthreads();
  // Thread d owns digit d: the waves' offsets inside the run, the run's place.
  u32 digit_total = 0;
#pragma unroll
  for (int w = 0; w < kPartWaves; ++w) {
    const u32 c = wave_cnt[w][tid];
    wave_cnt[w][tid] = digit_total;
    digit_total += c;
  }
  u32 total;
  const u32 gbase = block_excl_sum<kPartThreads>(digit_count_all, scratch, &total);
  const u32 start = block_excl_sum<kPartThreads>(digit_total, scratch, &total);
  local_start[tid] = start;
  out_base[tid] = gbase + tile_prefix - start;
  __syncthreads();

  u32 pos[kPartItems];
#pragma unroll
  for (int r = 0; r < kPartItems; ++r) {
    const u32 i = wave_base + r * kWave + lane;
    pos[r] = 0;
    if (i < n) {
      const u32 d = dg[r] & (kRadix - 1);
      pos[r] = local_start[d] + wave_cnt[wave][d] + rank[r];
      stage[pos[r]] = key[r];
      stage_digit[pos[r]] = (uint8_t)d;
      if (FIRST) stage_next[pos[r]] = (uint8_t)(dg[r] >> kRadixBits);
    }
  }
  __syncthreads();
  u32 dest[kPartItems];
#pragma unroll
  for (int k = 0; k < kPartItems; ++k) {
    const u32 p = k * kPartThreads + tid;
    dest[k] = 0;
    if (p < tile_n) {
      dest[k] = out_base[stage_digit[p]] + p;
      keys_out[dest[k]] = stage[p];
      if (FIRST && dig_out) dig_out[dest[k]] = stage_next[p];
    }
  }
  __syncthreads();
#pragma unroll
  for (int r = 0; r < kPartItems; ++r) {
    const u32 i = wave_base + r * kWave + lane;
    if (i < n) stage[pos[r]] = pay[r];
  }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < kPartItems; ++k) {
    const u32 p = k * kPartThreads + tid;
    if (p < tile_n) pay_out[dest[k]] = stage[p];
  }
}

// ---- regions ---------------------------------------------------------------------------
// A region may start where the bucket id changes, or anywhere inside a heavy key's bucket
// (it holds one key).  border(p0) = the first such position >= p0, n if there is none; region
// c is [border(c * kRegionSpan), border((c + 1) * kRegionSpan)), border(0) = 0.  One wave per
// border, 256 positions per round; borders[0 .. n_regions] out.
__global__ void __launch_bounds__(kPartThreads)
region_borders(const u64* __restrict__ skeys, u32 n, u32 n_regions, u32 max_heavy,
               const HeavySet* __restrict__ heavy_set, const PullCtx* __restrict__ ctx,
               u32* __restrict__ borders) {
  __shared__ HeavyLds hv;
  load_heavy(hv, heavy_set, max_heavy);
  if (threadIdx.x == 0) hv.range = ctx->range;
  __syncthreads();
  const u32 lane = lane_id();
  const u32 c = blockIdx.x * kPartWaves + threadIdx.x / kWave;
  if (c > n_regions) return;
  if (c == 0 || c == n_regions) {
    if (lane == 0) borders[c] = c == 0 ? 0u : n;
    return;
  }
  const u32 p0 = c * kRegionSpan;       // 0 < p0 < n
  u32 found = n;
  for (u32 base = p0; base < n && found == n; base += 4 * kWave) {
    // positions base + 4 * lane + q, q = 0..3, and the one before them
    u32 id[5];
    bool heavy[5];
#pragma unroll
    for (int q = 0; q < 5; ++q) {
      const u32 p = base + 4 * lane + q - 1;       // >= p0 - 1 >= 0
      const u64 key = skeys[min(p, n - 1)];
      id[q] = bucket_id(key, hv, &heavy[q]);
    }
    u32 mine = n;
#pragma unroll
    for (int q = 3; q >= 0; --q) {
      const u32 p = base + 4 * lane + q;
      if (p < n && (id[q + 1] != id[q] || (p == p0 && heavy[q + 1]))) mine = p;
    }
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) mine = min(mine, (u32)__shfl_xor((int)mine, d, kWave));
    found = mine;
  }
  if (lane == 0) borders[c] = found;
}

}  // namespace hps
