// Gradient reduce-by-key fused with the Adagrad row update.
//
// The dedup left the occurrences grouped by unique key: seg_off[u] .. seg_off[u+1]
// are the sorted positions of key u, and bagperm[j] is the bag of the occurrence at
// sorted position j.  The gradient of a sum-pooled bag reaches every occurrence
// unchanged, so the gradient of key u is the sum of grads[bagperm[j]] over its
// positions.  Keys are handled by how often they occur; the pull's lookup already
// sorted the frequent ones into work lists (table.hpp, OftenLists):
//
//   push_main   one launch, blocks take one of three roles:
//                 short   a group of LPR lanes per key with at most kShortSeg
//                         occurrences: reduced and updated on the spot;
//                 medium  one wave per listed key (up to kMedSeg occurrences): its
//                         lane groups stride over the positions, then add up;
//                 chunks  one block per listed chunk (kChunk positions of a still more
//                         frequent key): tree-reduced partial sum;
//   push_long   one block per chunked key: sums its chunks' partials in chunk order
//               (tree) and updates the row.
// Every sum has a fixed shape, so results do not depend on scheduling.
#pragma once

#include "common.hpp"
#include "table.hpp"

namespace hps {

constexpr int kPushThreads = 256;
constexpr int kPushShortBlocks = 1024;   // fixed grids: groups, waves and blocks loop (more short blocks measured slower)
constexpr int kPushMediumBlocks = 512;   // a multiple of kCountShards
// (one block per chunk, as many as the mini-batch could have, up to this: with 512 the skewed
// workload, most of whose occurrences are chunks of very frequent keys, ran its push at two
// waves per SIMD, 0.55 ms instead of 0.32; blocks without a chunk return at once)
constexpr int kPushChunkBlocks = 4096;
constexpr int kPushLongBlocks = 256;
constexpr int kPushInFlight = 8;  // gradient rows a lane group has in flight
constexpr u32 kBagMask = 0x7FFFFFFFu;
constexpr int kStepRowwise = 0;      // Adagrad, one accumulator per row
constexpr int kStepElementwise = 1;  // Adagrad, one accumulator per element
constexpr int kStepAdd = 2;          // Section 4.1 accumulate: the summed values are added

struct PushArgs {
  const u32* seg_off;
  const u32* bagperm;
  const u32* rows;
  const float* grads;
  const float* inv_len;   // != null (mean pooling): per bag, the share of its gradient an occurrence gets
  const PullCtx* ctx;
  const u32* med_list;  // unique indices, kCountShards shards of med_cap entries
  u32 med_cap;
  const uint2* long_list;     // (unique index, first chunk item)
  const uint2* chunk_items;   // (unique index, chunk number)
  u32 short_blocks, medium_blocks;   // roles of push_main's blocks: short, medium, chunks
  float* partials;      // [chunk item][dim]
  float lr, eps;
  int kind;   // what a touched row takes: kStepRowwise, kStepElementwise or kStepAdd
  HeavyRing* ring;   // != null: one more block puts the pull's list of frequent keys in order
  u32 ring_slot;
};

// One step on row r with the row's summed gradient (or summed values) held as
// float4 columns spread over the LPR lanes of a group.  Marks the row as updated.
template <int LPR, int COLS>
__device__ __forceinline__ void adagrad_row(const TableView& t, u32 r, const float4* g, u32 sub,
                                            float lr, float eps, int kind) {
  const u32 dim4 = t.dim >> 2;
  if (kind == kStepAdd) {
#pragma unroll
    for (int c = 0; c < COLS; ++c) {
      const u32 col = sub + c * LPR;
      if (col < dim4) {
        float4 v = load_w4(t, r, col);
        v.x += g[c].x; v.y += g[c].y; v.z += g[c].z; v.w += g[c].w;
        store_w4(t, r, col, v);
      }
    }
    if (sub == 0) {
      float* G = acc_row(t, r);
      *G = acc_marked(*G);
    }
  } else if (kind == kStepRowwise) {
    float ss = 0.f;
#pragma unroll
    for (int c = 0; c < COLS; ++c)
      if (sub + c * LPR < dim4) ss += g[c].x * g[c].x + g[c].y * g[c].y + g[c].z * g[c].z + g[c].w * g[c].w;
#pragma unroll
    for (int d = LPR / 2; d > 0; d >>= 1) ss += __shfl_xor(ss, d, kWave);
    float* G = acc_row(t, r);
    const float Gn = acc_value(*G) + ss / (float)t.dim;
    const float scale = lr / (sqrtf(Gn) + eps);
#pragma unroll
    for (int c = 0; c < COLS; ++c) {
      const u32 col = sub + c * LPR;
      if (col < dim4) {
        float4 v = load_w4(t, r, col);
        v.x -= scale * g[c].x; v.y -= scale * g[c].y; v.z -= scale * g[c].z; v.w -= scale * g[c].w;
        store_w4(t, r, col, v);
      }
    }
    if (sub == 0) *G = acc_marked(Gn);
  } else {
    float4* G = reinterpret_cast<float4*>(acc_row(t, r));
#pragma unroll
    for (int c = 0; c < COLS; ++c) {
      const u32 col = sub + c * LPR;
      if (col < dim4) {
        float4 a = G[col], v = load_w4(t, r, col);
        a.x = acc_value(a.x) + g[c].x * g[c].x; a.y += g[c].y * g[c].y; a.z += g[c].z * g[c].z; a.w += g[c].w * g[c].w;
        v.x -= lr * g[c].x / (sqrtf(a.x) + eps);
        v.y -= lr * g[c].y / (sqrtf(a.y) + eps);
        v.z -= lr * g[c].z / (sqrtf(a.z) + eps);
        v.w -= lr * g[c].w / (sqrtf(a.w) + eps);
        if (col == 0) a.x = acc_marked(a.x);
        G[col] = a;
        store_w4(t, r, col, v);
      }
    }
  }
}

// Adds the bag gradients of positions lo, lo+stride, ... < hi, kPushInFlight positions
// in flight at a time; each batch is summed as a balanced tree, then added.
template <int LPR, int COLS>
__device__ __forceinline__ void add_positions(float4* g, const PushArgs& a, u32 lo, u32 hi,
                                              u32 stride, u32 dim, u32 sub) {
  const u32 dim4 = dim >> 2;
  for (u32 j0 = lo; j0 < hi; j0 += kPushInFlight * stride) {
    u32 bag[kPushInFlight];
    bool on[kPushInFlight];
#pragma unroll
    for (int k = 0; k < kPushInFlight; ++k) {
      const u32 j = j0 + k * stride;
      on[k] = j < hi;
      bag[k] = on[k] ? (a.bagperm[j] & kBagMask) : 0u;
    }
    float4 v[kPushInFlight][COLS];
    float share[kPushInFlight];
#pragma unroll
    for (int k = 0; k < kPushInFlight; ++k) share[k] = (a.inv_len && on[k]) ? a.inv_len[bag[k]] : 1.0f;
#pragma unroll
    for (int k = 0; k < kPushInFlight; ++k) {
      const float4* row = reinterpret_cast<const float4*>(a.grads + (u64)bag[k] * dim);
#pragma unroll
      for (int c = 0; c < COLS; ++c) {
        const u32 col = sub + c * LPR;
        v[k][c] = (on[k] && col < dim4) ? row[col] : make_float4(0.f, 0.f, 0.f, 0.f);
      }
    }
    if (a.inv_len) {
#pragma unroll
      for (int k = 0; k < kPushInFlight; ++k)
#pragma unroll
        for (int c = 0; c < COLS; ++c) {
          v[k][c].x *= share[k]; v[k][c].y *= share[k]; v[k][c].z *= share[k]; v[k][c].w *= share[k];
        }
    }
#pragma unroll
    for (int c = 0; c < COLS; ++c) {
#pragma unroll
      for (int w = 1; w < kPushInFlight; w <<= 1) {
#pragma unroll
        for (int k = 0; k + w < kPushInFlight; k += 2 * w) {
          v[k][c].x += v[k + w][c].x; v[k][c].y += v[k + w][c].y;
          v[k][c].z += v[k + w][c].z; v[k][c].w += v[k + w][c].w;
        }
      }
      g[c].x += v[0][c].x; g[c].y += v[0][c].y; g[c].z += v[0][c].z; g[c].w += v[0][c].w;
    }
  }
}

template <int LPR, int COLS>
__device__ __forceinline__ void push_short_role(const TableView& t, const PushArgs& a, u32 block,
                                                u32 n_blocks) {
  const u32 sub = threadIdx.x % LPR;
  const u32 n_unique = a.ctx->n_unique;
  const u32 n_groups = n_blocks * (kPushThreads / LPR);
  for (u32 u = (block * kPushThreads + threadIdx.x) / LPR; u < n_unique; u += n_groups) {
    const u32 lo = a.seg_off[u], hi = a.seg_off[u + 1];
    if (hi - lo > kShortSeg) continue;      // on one of the lists
    const u32 r = a.rows[u];
    if (r == kNoRow) continue;
    float4 g[COLS];
#pragma unroll
    for (int c = 0; c < COLS; ++c) g[c] = make_float4(0.f, 0.f, 0.f, 0.f);
    add_positions<LPR, COLS>(g, a, lo, hi, 1, t.dim, sub);
    adagrad_row<LPR, COLS>(t, r, g, sub, a.lr, a.eps, a.kind);
  }
}

template <int LPR, int COLS>
__device__ __forceinline__ void push_medium_role(const TableView& t, const PushArgs& a, u32 block,
                                                 u32 n_blocks) {
  constexpr u32 kGroups = kWave / LPR;
  constexpr u32 kWavesPerBlock = kPushThreads / kWave;
  const u32 group = lane_id() / LPR, sub = lane_id() % LPR;
  // block b serves list shard b % 64, together with the other blocks of that residue
  const u32 shard = block % kCountShards;
  const u32 shard_blocks = (n_blocks - shard + kCountShards - 1) / kCountShards;
  const u32 count = min(a.ctx->med_count[shard], a.med_cap);
  const u32* list = a.med_list + (u64)shard * a.med_cap;
  for (u32 m = (block / kCountShards) * kWavesPerBlock + threadIdx.x / kWave; m < count;
       m += shard_blocks * kWavesPerBlock) {
    const u32 u = list[m];
    float4 g[COLS];
#pragma unroll
    for (int c = 0; c < COLS; ++c) g[c] = make_float4(0.f, 0.f, 0.f, 0.f);
    add_positions<LPR, COLS>(g, a, a.seg_off[u] + group, a.seg_off[u + 1], kGroups, t.dim, sub);
#pragma unroll
    for (int c = 0; c < COLS; ++c) {
#pragma unroll
      for (int d = LPR; d < kWave; d <<= 1) {
        g[c].x += __shfl_xor(g[c].x, d, kWave);
        g[c].y += __shfl_xor(g[c].y, d, kWave);
        g[c].z += __shfl_xor(g[c].z, d, kWave);
        g[c].w += __shfl_xor(g[c].w, d, kWave);
      }
    }
    const u32 r = a.rows[u];
    if (group == 0 && r != kNoRow) adagrad_row<LPR, COLS>(t, r, g, sub, a.lr, a.eps, a.kind);
  }
}

// Sums, over the kPushThreads/LPR groups of the block, the float4 columns each
// group holds; the result is valid in group 0.  `lds` holds kPushThreads float4.
template <int LPR, int COLS>
__device__ __forceinline__ void block_tree_sum(float4* g, float4* lds, u32 dim4) {
  constexpr int kGroups = kPushThreads / LPR;
  const u32 group = threadIdx.x / LPR, sub = threadIdx.x % LPR;
#pragma unroll
  for (int c = 0; c < COLS; ++c) {
    if ((u32)(c * LPR) >= dim4) break;       // block-uniform: no columns left
    const bool has = sub + c * LPR < dim4;
    for (int s = kGroups / 2; s > 0; s >>= 1) {
      __syncthreads();
      if (has && group >= (u32)s && group < (u32)(2 * s)) lds[(group - s) * LPR + sub] = g[c];
      __syncthreads();
      if (has && group < (u32)s) {
        const float4 v = lds[group * LPR + sub];
        g[c].x += v.x; g[c].y += v.y; g[c].z += v.z; g[c].w += v.w;
      }
    }
  }
}

template <int LPR, int COLS>
__device__ __forceinline__ void push_chunks_role(const TableView& t, const PushArgs& a, u32 block,
                                                 u32 n_blocks, float4* lds) {
  constexpr int kGroups = kPushThreads / LPR;
  const u32 n_items = a.ctx->n_chunk_items;
  const u32 group = threadIdx.x / LPR, sub = threadIdx.x % LPR;
  for (u32 item = block; item < n_items; item += n_blocks) {
    const uint2 it = a.chunk_items[item];
    const u32 lo = a.seg_off[it.x] + it.y * kChunk;
    const u32 hi = min(lo + kChunk, a.seg_off[it.x + 1]);
    float4 g[COLS];
#pragma unroll
    for (int c = 0; c < COLS; ++c) g[c] = make_float4(0.f, 0.f, 0.f, 0.f);
    add_positions<LPR, COLS>(g, a, lo + group, hi, kGroups, t.dim, sub);
    block_tree_sum<LPR, COLS>(g, lds, t.dim >> 2);
    if (group == 0) {
      float4* out = reinterpret_cast<float4*>(a.partials + (u64)item * t.dim);
#pragma unroll
      for (int c = 0; c < COLS; ++c)
        if (sub + c * LPR < (t.dim >> 2)) out[sub + c * LPR] = g[c];
    }
  }
}

template <int LPR, int COLS>
__global__ void __launch_bounds__(kPushThreads) push_main(TableView t, PushArgs a) {
  __shared__ float4 lds[kPushThreads];
  if (load_error(t.st) != 0) return;
  if (a.ring && blockIdx.x == 0) {
    // Not part of the push: the list of frequent keys the pull's lookup left (common.hpp) is
    // put in order here, where it costs nothing -- the next dedup that reads it starts after
    // this push, and the push takes several times longer than this block.  (The first block,
    // so that it starts at once: behind thousands of others it would end the kernel late.)
    finalize_heavy(a.ring, a.ring_slot);
    return;
  }
  const u32 b = a.ring ? blockIdx.x - 1 : blockIdx.x;
  const u32 role_blocks = a.ring ? gridDim.x - 1 : gridDim.x;
  if (b < a.short_blocks) {
    push_short_role<LPR, COLS>(t, a, b, a.short_blocks);
  } else if (b < a.short_blocks + a.medium_blocks) {
    push_medium_role<LPR, COLS>(t, a, b - a.short_blocks, a.medium_blocks);
  } else {
    push_chunks_role<LPR, COLS>(t, a, b - a.short_blocks - a.medium_blocks,
                          role_blocks - a.short_blocks - a.medium_blocks, lds);
  }
}

template <int LPR, int COLS>
__global__ void __launch_bounds__(kPushThreads) push_long(TableView t, PushArgs a) {
  __shared__ float4 lds[kPushThreads];
  constexpr int kGroups = kPushThreads / LPR;
  if (load_error(t.st) != 0) return;
  const u32 n_long = a.ctx->n_long;
  const u32 group = threadIdx.x / LPR, sub = threadIdx.x % LPR;
  for (u32 l = blockIdx.x; l < n_long; l += gridDim.x) {
  const uint2 seg = a.long_list[l];
  const u32 len = a.seg_off[seg.x + 1] - a.seg_off[seg.x];
  const u32 n_chunks = (len + kChunk - 1) / kChunk;
  float4 g[COLS];
#pragma unroll
  for (int c = 0; c < COLS; ++c) g[c] = make_float4(0.f, 0.f, 0.f, 0.f);
  // (eight partial rows requested at a time, added in chunk order: a key that fills thousands of
  // chunks would otherwise wait for every row in turn)
  for (u32 c0 = group; c0 < n_chunks; c0 += kPushInFlight * kGroups) {
    float4 v[kPushInFlight][COLS];
#pragma unroll
    for (int k = 0; k < kPushInFlight; ++k) {
      const u32 c = c0 + k * kGroups;
      const float4* row = reinterpret_cast<const float4*>(a.partials + (u64)(seg.y + (c < n_chunks ? c : c0)) * t.dim);
#pragma unroll
      for (int q = 0; q < COLS; ++q) {
        const u32 col = sub + q * LPR;
        v[k][q] = (c < n_chunks && col < (t.dim >> 2)) ? row[col] : make_float4(0.f, 0.f, 0.f, 0.f);
      }
    }
#pragma unroll
    for (int k = 0; k < kPushInFlight; ++k)
#pragma unroll
      for (int q = 0; q < COLS; ++q) {
        g[q].x += v[k][q].x; g[q].y += v[k][q].y; g[q].z += v[k][q].z; g[q].w += v[k][q].w;
      }
  }
  block_tree_sum<LPR, COLS>(g, lds, t.dim >> 2);
  const u32 r = a.rows[seg.x];
  if (group == 0 && r != kNoRow) adagrad_row<LPR, COLS>(t, r, g, sub, a.lr, a.eps, a.kind);
  }
}

}  // namespace hps
