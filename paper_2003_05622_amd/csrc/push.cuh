// Gradient reduce-by-key fused with the Adagrad row update.
//
// The dedup left the occurrences grouped by unique key: seg_off[u] .. seg_off[u+1]
// are the sorted positions of key u, and bagperm[j] is the bag of the occurrence at
// sorted position j.  The gradient of a sum-pooled bag reaches every occurrence
// unchanged, so the gradient of key u is the sum of grads[bagperm[j]] over its
// positions.  Keys are handled by how often they occur:
//
//   push_short    a group of LPR lanes per key; keys with at most kShortSeg
//                 occurrences are reduced and updated on the spot, the others are
//                 queued: up to kMedSeg occurrences on the medium list, more as
//                 chunks of kChunk positions;
//   push_medium   one wave per queued key: its lane groups stride over the positions,
//                 then add up across the wave;
//   push_chunks   one block per queued chunk: tree-reduced partial sum;
//   push_long     one block per chunked key: sums its chunks' partials in chunk order
//                 (tree) and updates the row.
// Every sum has a fixed shape, so results do not depend on scheduling.
#pragma once

#include "common.cuh"
#include "table.cuh"

namespace hps {

constexpr int kPushThreads = 256;
constexpr int kPushShortBlocks = 2048;   // fixed grids: groups, waves and blocks loop
constexpr int kPushMediumBlocks = 1024;
constexpr int kPushChunkBlocks = 1024;
constexpr int kPushLongBlocks = 256;
constexpr u32 kShortSeg = 16;     // occurrences handled serially by one lane group
constexpr u32 kMedSeg = 512;      // occurrences handled by one wave
constexpr u32 kChunk = 1024;      // occurrences per queued chunk of a longer key
constexpr int kMaxCols = 4;       // float4 columns per lane
constexpr u32 kBagMask = 0x7FFFFFFFu;

struct PushArgs {
  const u32* seg_off;
  const u32* bagperm;
  const u32* rows;
  const float* grads;
  PullCtx* ctx;
  u32* med_list;        // unique indices
  uint2* long_list;     // (unique index, first chunk item)
  uint2* chunk_items;   // (unique index, chunk number)
  float* partials;      // [chunk item][dim]
  float lr, eps;
  int elementwise;
};

// One optimizer step on row r with the row's summed gradient held as float4
// columns spread over the LPR lanes of a group.
template <int LPR>
__device__ __forceinline__ void adagrad_row(const TableView& t, u32 r, const float4* g, u32 sub,
                                            float lr, float eps, int elementwise) {
  const u32 dim4 = t.dim >> 2;
  float4* w = reinterpret_cast<float4*>(t.w + (u64)r * t.dim);
  if (!elementwise) {
    float ss = 0.f;
#pragma unroll
    for (int c = 0; c < kMaxCols; ++c)
      if (sub + c * LPR < dim4) ss += g[c].x * g[c].x + g[c].y * g[c].y + g[c].z * g[c].z + g[c].w * g[c].w;
#pragma unroll
    for (int d = LPR / 2; d > 0; d >>= 1) ss += __shfl_xor(ss, d, kWave);
    float* G = t.acc + (u64)r;
    const float Gn = *G + ss / (float)t.dim;
    const float scale = lr / (sqrtf(Gn) + eps);
#pragma unroll
    for (int c = 0; c < kMaxCols; ++c) {
      const u32 col = sub + c * LPR;
      if (col < dim4) {
        float4 v = w[col];
        v.x -= scale * g[c].x; v.y -= scale * g[c].y; v.z -= scale * g[c].z; v.w -= scale * g[c].w;
        w[col] = v;
      }
    }
    if (sub == 0) *G = Gn;
  } else {
    float4* G = reinterpret_cast<float4*>(t.acc + (u64)r * t.dim);
#pragma unroll
    for (int c = 0; c < kMaxCols; ++c) {
      const u32 col = sub + c * LPR;
      if (col < dim4) {
        float4 a = G[col], v = w[col];
        a.x += g[c].x * g[c].x; a.y += g[c].y * g[c].y; a.z += g[c].z * g[c].z; a.w += g[c].w * g[c].w;
        v.x -= lr * g[c].x / (sqrtf(a.x) + eps);
        v.y -= lr * g[c].y / (sqrtf(a.y) + eps);
        v.z -= lr * g[c].z / (sqrtf(a.z) + eps);
        v.w -= lr * g[c].w / (sqrtf(a.w) + eps);
        G[col] = a;
        w[col] = v;
      }
    }
  }
}

template <int LPR>
__device__ __forceinline__ void add_grad_row(float4* g, const float* grads, u32 bag, u32 dim,
                                             u32 sub) {
  const float4* row = reinterpret_cast<const float4*>(grads + (u64)bag * dim);
  const u32 dim4 = dim >> 2;
#pragma unroll
  for (int c = 0; c < kMaxCols; ++c) {
    const u32 col = sub + c * LPR;
    if (col < dim4) {
      const float4 v = row[col];
      g[c].x += v.x; g[c].y += v.y; g[c].z += v.z; g[c].w += v.w;
    }
  }
}

// Adds the bag gradients of positions lo, lo+stride, ... < hi, four positions in
// flight at a time.
template <int LPR>
__device__ __forceinline__ void add_positions(float4* g, const PushArgs& a, u32 lo, u32 hi,
                                              u32 stride, u32 dim, u32 sub) {
  u32 j = lo;
  for (; j + 3 * stride < hi; j += 4 * stride) {
    const u32 b0 = a.bagperm[j] & kBagMask, b1 = a.bagperm[j + stride] & kBagMask;
    const u32 b2 = a.bagperm[j + 2 * stride] & kBagMask, b3 = a.bagperm[j + 3 * stride] & kBagMask;
    float4 t0[kMaxCols], t1[kMaxCols], t2[kMaxCols], t3[kMaxCols];
#pragma unroll
    for (int c = 0; c < kMaxCols; ++c) t0[c] = t1[c] = t2[c] = t3[c] = make_float4(0.f, 0.f, 0.f, 0.f);
    add_grad_row<LPR>(t0, a.grads, b0, dim, sub);
    add_grad_row<LPR>(t1, a.grads, b1, dim, sub);
    add_grad_row<LPR>(t2, a.grads, b2, dim, sub);
    add_grad_row<LPR>(t3, a.grads, b3, dim, sub);
#pragma unroll
    for (int c = 0; c < kMaxCols; ++c) {
      g[c].x += (t0[c].x + t1[c].x) + (t2[c].x + t3[c].x);
      g[c].y += (t0[c].y + t1[c].y) + (t2[c].y + t3[c].y);
      g[c].z += (t0[c].z + t1[c].z) + (t2[c].z + t3[c].z);
      g[c].w += (t0[c].w + t1[c].w) + (t2[c].w + t3[c].w);
    }
  }
  for (; j < hi; j += stride) add_grad_row<LPR>(g, a.grads, a.bagperm[j] & kBagMask, dim, sub);
}

template <int LPR>
__global__ void __launch_bounds__(kPushThreads) push_short(TableView t, PushArgs a) {
  const u32 sub = threadIdx.x % LPR;
  if (load_error(t.st) != 0) return;
  const u32 n_unique = a.ctx->n_unique;
  const u32 n_groups = gridDim.x * (kPushThreads / LPR);
  for (u32 u = (blockIdx.x * kPushThreads + threadIdx.x) / LPR; u < n_unique; u += n_groups) {
  const u32 lo = a.seg_off[u], hi = a.seg_off[u + 1];
  const u32 len = hi - lo;
  if (len > kShortSeg) {
    if (len <= kMedSeg) {
      if (sub == 0) a.med_list[atomicAdd(&a.ctx->n_medium, 1u)] = u;
      continue;
    }
    const u32 n_chunks = (len + kChunk - 1) / kChunk;
    u32 base = 0;
    if (sub == 0) {
      base = atomicAdd(&a.ctx->n_chunk_items, n_chunks);
      a.long_list[atomicAdd(&a.ctx->n_long, 1u)] = make_uint2(u, base);
    }
    base = __shfl(base, (int)(lane_id() - sub), kWave);
    for (u32 c = sub; c < n_chunks; c += LPR) a.chunk_items[base + c] = make_uint2(u, c);
    continue;
  }
  const u32 r = a.rows[u];
  if (r == kNoRow) continue;
  float4 g[kMaxCols];
#pragma unroll
  for (int c = 0; c < kMaxCols; ++c) g[c] = make_float4(0.f, 0.f, 0.f, 0.f);
  add_positions<LPR>(g, a, lo, hi, 1, t.dim, sub);
  adagrad_row<LPR>(t, r, g, sub, a.lr, a.eps, a.elementwise);
  }
}

template <int LPR>
__global__ void __launch_bounds__(kPushThreads) push_medium(TableView t, PushArgs a) {
  constexpr u32 kGroups = kWave / LPR;
  if (load_error(t.st) != 0) return;
  const u32 n_medium = a.ctx->n_medium;
  const u32 n_waves = gridDim.x * (kPushThreads / kWave);
  const u32 group = lane_id() / LPR, sub = lane_id() % LPR;
  for (u32 m = (blockIdx.x * kPushThreads + threadIdx.x) / kWave; m < n_medium; m += n_waves) {
  const u32 u = a.med_list[m];
  float4 g[kMaxCols];
#pragma unroll
  for (int c = 0; c < kMaxCols; ++c) g[c] = make_float4(0.f, 0.f, 0.f, 0.f);
  add_positions<LPR>(g, a, a.seg_off[u] + group, a.seg_off[u + 1], kGroups, t.dim, sub);
#pragma unroll
  for (int c = 0; c < kMaxCols; ++c) {
#pragma unroll
    for (int d = LPR; d < kWave; d <<= 1) {
      g[c].x += __shfl_xor(g[c].x, d, kWave);
      g[c].y += __shfl_xor(g[c].y, d, kWave);
      g[c].z += __shfl_xor(g[c].z, d, kWave);
      g[c].w += __shfl_xor(g[c].w, d, kWave);
    }
  }
  const u32 r = a.rows[u];
  if (group == 0 && r != kNoRow) adagrad_row<LPR>(t, r, g, sub, a.lr, a.eps, a.elementwise);
  }
}

// Sums, over the kPushThreads/LPR groups of the block, the float4 columns each
// group holds; the result is valid in group 0.  `lds` holds kPushThreads float4.
template <int LPR>
__device__ __forceinline__ void block_tree_sum(float4* g, float4* lds, u32 dim4) {
  constexpr int kGroups = kPushThreads / LPR;
  const u32 group = threadIdx.x / LPR, sub = threadIdx.x % LPR;
#pragma unroll
  for (int c = 0; c < kMaxCols; ++c) {
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

template <int LPR>
__global__ void __launch_bounds__(kPushThreads) push_chunks(TableView t, PushArgs a) {
  __shared__ float4 lds[kPushThreads];
  constexpr int kGroups = kPushThreads / LPR;
  if (load_error(t.st) != 0) return;
  const u32 n_items = a.ctx->n_chunk_items;
  const u32 group = threadIdx.x / LPR, sub = threadIdx.x % LPR;
  for (u32 item = blockIdx.x; item < n_items; item += gridDim.x) {
  const uint2 it = a.chunk_items[item];
  const u32 lo = a.seg_off[it.x] + it.y * kChunk;
  const u32 hi = min(lo + kChunk, a.seg_off[it.x + 1]);
  float4 g[kMaxCols];
#pragma unroll
  for (int c = 0; c < kMaxCols; ++c) g[c] = make_float4(0.f, 0.f, 0.f, 0.f);
  add_positions<LPR>(g, a, lo + group, hi, kGroups, t.dim, sub);
  block_tree_sum<LPR>(g, lds, t.dim >> 2);
  if (group == 0) {
    float4* out = reinterpret_cast<float4*>(a.partials + (u64)item * t.dim);
#pragma unroll
    for (int c = 0; c < kMaxCols; ++c)
      if (sub + c * LPR < (t.dim >> 2)) out[sub + c * LPR] = g[c];
  }
  }
}

template <int LPR>
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
  float4 g[kMaxCols];
#pragma unroll
  for (int c = 0; c < kMaxCols; ++c) g[c] = make_float4(0.f, 0.f, 0.f, 0.f);
  for (u32 c = group; c < n_chunks; c += kGroups)
    add_grad_row<LPR>(g, a.partials, seg.y + c, t.dim, sub);
  block_tree_sum<LPR>(g, lds, t.dim >> 2);
  const u32 r = a.rows[seg.x];
  if (group == 0 && r != kNoRow) adagrad_row<LPR>(t, r, g, sub, a.lr, a.eps, a.elementwise);
  }
}

}  // namespace hps
