// Key dedup, part 2: from the occurrence indices sorted by key to
//   uniq[U]      ascending unique keys
//   inverse[N]   rank of each occurrence's key among them
//   perm[N]      occurrence indices grouped by key (ascending key)
//   seg_off[U+1] start of each key's group in perm
// Three kernels over tiles of kHeadTile sorted positions: count group heads per
// tile, scan the tile counts (one block), emit.
#pragma once

#include "common.cuh"

namespace hps {

constexpr int kHeadThreads = 256;
constexpr int kHeadItems = 8;
constexpr int kHeadTile = kHeadThreads * kHeadItems;

// skeys[j] = key of the j-th sorted occurrence; tile_heads[tile] = number of
// positions in the tile whose key differs from the previous position's.
__global__ void __launch_bounds__(kHeadThreads)
heads_count(const u64* __restrict__ sorted_pairs, const u64* __restrict__ keys, u32 n,
            u64* __restrict__ skeys, u32* __restrict__ tile_heads) {
  __shared__ u32 scratch[kHeadThreads / kWave + 1];
  const u32 first = blockIdx.x * kHeadTile + threadIdx.x * kHeadItems;
  u64 prev = 0;
  if (first > 0 && first < n) prev = keys[(u32)sorted_pairs[first - 1]];
  u32 heads = 0;
#pragma unroll
  for (int k = 0; k < kHeadItems; ++k) {
    const u32 j = first + k;
    if (j < n) {
      const u64 key = keys[(u32)sorted_pairs[j]];
      skeys[j] = key;
      heads += (j == 0 || key != prev) ? 1u : 0u;
      prev = key;
    }
  }
  u32 total;
  block_excl_sum<kHeadThreads>(heads, scratch, &total);
  if (threadIdx.x == 0) tile_heads[blockIdx.x] = total;
}

// Exclusive scan of the tile counts; publishes U and seg_off[U] = n.
__global__ void __launch_bounds__(1024)
heads_scan(u32* __restrict__ tile_heads, u32 n_tiles, u32 n, PullCtx* __restrict__ ctx,
           u32* __restrict__ seg_off) {
  __shared__ u32 scratch[1024 / kWave + 1];
  const u32 per = (n_tiles + 1023) / 1024;
  const u32 lo = min(threadIdx.x * per, n_tiles), hi = min(lo + per, n_tiles);
  u32 s = 0;
  for (u32 i = lo; i < hi; ++i) s += tile_heads[i];
  u32 total;
  u32 run = block_excl_sum<1024>(s, scratch, &total);
  for (u32 i = lo; i < hi; ++i) {
    const u32 c = tile_heads[i];
    tile_heads[i] = run;
    run += c;
  }
  if (threadIdx.x == 0) {
    ctx->n_unique = total;
    ctx->n_long = 0;
    ctx->n_chunk_items = 0;
    seg_off[total] = n;
  }
}

__global__ void __launch_bounds__(kHeadThreads)
heads_emit(const u64* __restrict__ sorted_pairs, const u64* __restrict__ skeys, u32 n,
           const u32* __restrict__ tile_base, u64* __restrict__ uniq, i32* __restrict__ inverse,
           u32* __restrict__ perm, u32* __restrict__ seg_off, TableState* __restrict__ st) {
  __shared__ u32 scratch[kHeadThreads / kWave + 1];
  const u32 first = blockIdx.x * kHeadTile + threadIdx.x * kHeadItems;
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
  u32 total;
  u32 rank = tile_base[blockIdx.x] + block_excl_sum<kHeadThreads>(heads, scratch, &total);
  // rank = number of heads before this thread's first position
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
      const u32 idx = (u32)sorted_pairs[j];
      perm[j] = idx;
      inverse[idx] = (i32)(rank - 1);
    }
  }
}

}  // namespace hps
