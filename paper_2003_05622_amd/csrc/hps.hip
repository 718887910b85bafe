// Host side of the C ABI declared in include/hps.h: argument checks, carving of
// the caller's storage and workspace, and the kernel launch sequences of
// insert / pull / push / get / dump.  No device memory is allocated here.

#include "../../include/hps.h"
#include "../../include/hps_measure.h"
#include "../../include/hps_mem.h"

#include <hip/hip_runtime.h>

#include <cstddef>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include <algorithm>

#include "common.hpp"
#include "bucket.hpp"
#include "dedup.hpp"
#include "partition.hpp"
#include "pool.hpp"
#include "push.hpp"
#include "sort.hpp"
#include "table.hpp"
#include "mem_tier.hpp"

using namespace hps;

namespace {

constexpr double kLoadFactor = 0.7;
constexpr size_t kAlign = 256;
constexpr uint64_t kMaxSlots = 0xFFFFFFF0ull;   // row indices are 32-bit, kNoRow is reserved
constexpr uint32_t kMinTileGroup = 8;

size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

uint64_t slots_for(uint64_t capacity) {
  uint64_t s = (uint64_t)((double)capacity / kLoadFactor) + 1;
  if (s < capacity + kSlotsPerLine) s = capacity + kSlotsPerLine;
  // a whole number of 128-byte memory lines (two lines of slots each)
  return (s + 2 * kSlotsPerLine - 1) / (2 * kSlotsPerLine) * (2 * kSlotsPerLine);
}

bool valid_opt(const hps_optimizer* o) {
  return o && (o->kind == HPS_OPT_ADAGRAD_ROWWISE || o->kind == HPS_OPT_ADAGRAD_ELEMENTWISE) &&
         (o->row_format == HPS_ROWS_F32 || o->row_format == HPS_ROWS_BF16 ||
          o->row_format == HPS_ROWS_F32_WIDE) &&
         o->init_range >= 0.f && o->eps >= 0.f && o->init_acc >= 0.f;
}

bool valid_shape(uint64_t capacity, uint32_t dim) {
  return capacity >= 1 && dim >= 4 && dim <= 1024 && dim % 4 == 0 &&
         slots_for(capacity) <= kMaxSlots;
}

struct StorageLayout {
  size_t keys, w, acc, state, total;
  uint32_t w_pitch, acc_pitch;     // bytes from one row to the next
};

// Weights and accumulators of a row side by side (table.hpp: TableView)?
bool rows_side_by_side(uint32_t dim, uint32_t acc_len, int row_format) {
  const uint32_t pair = 8 * dim;
  const char* env = std::getenv("HPS_ROWS");          // "apart": always two arrays (for comparison)
  if (env && std::strcmp(env, "apart") == 0) return false;
  return row_format == HPS_ROWS_F32 && acc_len == dim && (pair % 128 == 0 || 128 % pair == 0);
}

StorageLayout storage_layout(uint64_t n_slots, uint32_t dim, uint32_t acc_len, int row_format) {
  StorageLayout L;
  size_t o = 0;
  L.keys = o;  o = align_up(o + n_slots * sizeof(uint64_t));
  const uint32_t w_bytes = dim * (row_format == HPS_ROWS_BF16 ? 2 : 4), acc_bytes = acc_len * 4;
  if (row_format == HPS_ROWS_F32_WIDE) {
    // one record per row, whole memory lines
    const uint32_t pitch = (w_bytes + acc_bytes + 127) / 128 * 128;
    L.w = o;   L.acc = o + w_bytes;
    L.w_pitch = L.acc_pitch = pitch;
    o = align_up(o + n_slots * (size_t)pitch);
  } else if (rows_side_by_side(dim, acc_len, row_format)) {
    L.w = o;   L.acc = o + w_bytes;
    L.w_pitch = L.acc_pitch = w_bytes + acc_bytes;
    o = align_up(o + n_slots * (size_t)(w_bytes + acc_bytes));
  } else {
    L.w = o;   o = align_up(o + n_slots * (size_t)w_bytes);
    L.acc = o; o = align_up(o + n_slots * (size_t)acc_bytes);
    L.w_pitch = w_bytes;
    L.acc_pitch = acc_bytes;
  }
  L.state = o; o = align_up(o + sizeof(TableState));
  L.total = o;
  return L;
}

// Per pull context (two of them, so that the dedup of the next mini-batch can run
// while the current one is still between pull and push).
struct ContextLayout {
  size_t ctx, uniq, rows, inverse, bagperm, seg_off, inv_len, hot_list;
};

struct WorkspaceLayout {
  size_t keys_a, keys_b, keys_c, idx_a, idx_b, idx_c, id16, dig, part_hist, part_tot, borders, heavy_raw, ghist,
      tickets, tile_rows, group_rows, head_rows, head_groups, evidence, bag_of, miss_list, med_list, long_list,
      chunk_items, partials, total;
  ContextLayout c[2];
  uint64_t med_cap, max_long, max_items, sort_tiles, head_tiles, shard_cap;
};

WorkspaceLayout workspace_layout(uint64_t n, uint64_t bags, uint32_t dim) {
  WorkspaceLayout L;
  const uint64_t n1 = n ? n : 1;
  L.sort_tiles = (n1 + kSortTile - 1) / kSortTile;
  L.head_tiles = (n1 + kHeadTile - 1) / kHeadTile;
  L.med_cap = n1 / kCountShards + 2048;     // per shard: no shard's blocks see more keys
  L.max_long = n1 / (kMedSeg + 1) + 1;      // keys with more than kMedSeg occurrences
  L.max_items = n1 / kChunk + L.max_long + 1;
  size_t o = 0;
  L.keys_a = o;      o = align_up(o + n1 * 8);
  L.keys_b = o;      o = align_up(o + n1 * 8);
  L.keys_c = o;      o = align_up(o + n1 * 8);    // scratch of a region ordered the slow way
  L.idx_a = o;       o = align_up(o + n1 * 8);    // payloads: occurrence index | bag << 32
  L.idx_b = o;       o = align_up(o + n1 * 8);
  L.idx_c = o;       o = align_up(o + n1 * 8);
  L.id16 = o;        o = align_up(o + n1 * 2);    // bucket id of every occurrence
  L.dig = o;         o = align_up(o + n1 + 4);    // the ids' high bytes, ordered by the low bytes
  L.part_hist = o;   o = align_up(o + (size_t)kRadix * L.sort_tiles * 4);   // [digit][tile] counts of a pass
  L.part_tot = o;    o = align_up(o + kRadix * 4);
  L.borders = o;     o = align_up(o + (n1 / kRegionSpan + 3) * 4);
  // from here to `evidence`: cleared at creation, never again (see sort.hpp)
  L.ghist = o;       o = align_up(o + 2 * (size_t)kHistWords * 4);
  L.tickets = o;     o = align_up(o + (kMaxPasses + 2) * 4);
  L.tile_rows = o;   o = align_up(o + (size_t)kMaxPasses * L.sort_tiles * kRadix * 4);
  L.group_rows = o;  o = align_up(o + (size_t)kMaxPasses * (L.sort_tiles / kMinTileGroup + 1) * kRadix * 4);
  L.head_rows = o;   o = align_up(o + 2 * L.head_tiles * 4);
  L.head_groups = o; o = align_up(o + 2 * (L.head_tiles / kMinTileGroup + 1) * 4);
  L.evidence = o;    o = align_up(o + kMaxEvidence * 4);
  L.heavy_raw = o;   o = align_up(o + sizeof(HeavyRing));
  L.bag_of = o;      o = align_up(o + n1 * 4);
  L.shard_cap = n1 / kCountShards + kMissLdsCap;
  L.miss_list = o;   o = align_up(o + (size_t)kCountShards * L.shard_cap * 4);
  for (int k = 0; k < 2; ++k) {
    L.c[k].ctx = o;     o = align_up(o + sizeof(PullCtx));
    L.c[k].uniq = o;    o = align_up(o + n1 * 8);
    L.c[k].rows = o;    o = align_up(o + n1 * 4);
    L.c[k].inverse = o; o = align_up(o + n1 * 4);
    L.c[k].bagperm = o; o = align_up(o + n1 * 4);
    L.c[k].seg_off = o; o = align_up(o + (n1 + 1) * 4);
    L.c[k].inv_len = o; o = align_up(o + (bags ? bags : 1) * 4);    // mean pooling: 1 / bag length
    L.c[k].hot_list = o; o = align_up(o + kMaxHot * 8);             // (unique index, row) of the most frequent keys
  }
  L.med_list = o;    o = align_up(o + (size_t)kCountShards * L.med_cap * 4);
  L.long_list = o;   o = align_up(o + L.max_long * 8);
  L.chunk_items = o; o = align_up(o + L.max_items * 8);
  L.partials = o;    o = align_up(o + L.max_items * (size_t)dim * 4);
  L.total = o;
  return L;
}

// Tiles per look-back group: about the square root of the tile count.
uint32_t tile_group(uint64_t n_tiles) {
  uint32_t g = kMinTileGroup;
  while (g < kMaxTileGroup && (uint64_t)g * g < n_tiles) ++g;
  return g;
}

// Largest dedup the bucket path takes: beyond it a heavy key the hint misses could
// hold more occurrences than a region has room for.
constexpr uint64_t kBucketPathMaxKeys = 12ull << 20;
constexpr uint64_t kPlainHold = 32;      // dedups in the plain form after the bucket form disappointed
constexpr uint64_t kHintLag = 3;         // ... after a surprise that the next lists of frequent keys will cover
static_assert(kChunkSpan + 2 * kNaturalBucket + kBucketPathMaxKeys / kHeavyShare + 64 <= kChunkThreads * kChunkItems,
              "a region must have room for its span, a natural bucket and one heavy key the hint missed");

// Bucket path: enough leading key bits that a natural bucket holds kNaturalBucket
// occurrences on average at most; the passes sort by the bytes of the bucket id.  Up to
// kOnePassMaxKeys occurrences 7 leading bits and 63 heavy keys do: ids below 256, one pass.
constexpr uint64_t kOnePassMaxKeys = 1ull << 16;

SortPlan bucket_plan(uint64_t n) {
  SortPlan p;
  int bits = 1;
  while (bits < 15 && ((n + kNaturalBucket - 1) / kNaturalBucket) > (1ull << bits)) ++bits;
  p.max_heavy = kMaxHeavy;
  p.n_pass = 2;      // ids stay below 2^16 for every n the bucket path takes
  if (n <= kOnePassMaxKeys) {
    if (bits > 7) bits = 7;
    p.max_heavy = 63;
    p.n_pass = 1;
  }
  p.low_shift = 0;
  p.group = tile_group((n + kSortTile - 1) / kSortTile);
  p.by_id = 1;
  p.nat_shift = 64 - bits;
  return p;
}

// Plain form.  How many 8-bit digits to sort for n occurrences: enough that two different
// keys rarely agree in all sorted bits.  With b sorted bits about n^2 / 2^(b+1) pairs of
// distinct hashed keys collide; b >= 2*log2(n) - 2 keeps that near one in a few
// batches, and every collision is repaired anyway (dedup.hpp).
// all_bits: every bit of the keys is sorted (eight passes), whatever the keys look like.
SortPlan sort_plan(uint64_t n, bool all_bits) {
  SortPlan p;
  p.by_id = 0;
  p.nat_shift = 0;
  p.max_heavy = 0;
  int log2n = 1;
  while ((1ull << log2n) < n) ++log2n;
  int want = (2 * log2n - 2 + 7) / 8;
  if (want < 2) want = 2;
  if (want > kMaxPasses || all_bits) want = kMaxPasses;
  p.n_pass = want;
  p.low_shift = 64 - 8 * want;
  p.group = tile_group((n + kSortTile - 1) / kSortTile);
  return p;
}

unsigned grid_for(uint64_t work_items, uint64_t items_per_block, unsigned max_blocks) {
  uint64_t b = (work_items + items_per_block - 1) / items_per_block;
  if (b < 1) b = 1;
  return (unsigned)(b < max_blocks ? b : max_blocks);
}

int lanes_per_row(uint32_t dim) {
  int l = 1;
  while (l < 64 && (uint32_t)l * 4 < dim) l <<= 1;
  return l;
}

bool launch_ok() { return hipGetLastError() == hipSuccess; }

}  // namespace

// ---- the one entry point that allocates nothing (hps_accumulate_static) ------------------
// Its workspace: a file-scope device array, one copy per GPU, held until the process ends.
// Room for the workspace of HPS_STATIC_MAX_KEYS pairs with rows of up to 1024 floats.
constexpr size_t kStaticScratchBytes = 10u << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
struct StaticScratch {
  char* ptr;                // this device's address of `scratch` (hipGetSymbolAddress), null until first used
  bool ring_ready;          // its lists of frequent keys have been initialised
  uint64_t lookup_serial;   // lookups run on it so far (they take turns on its three lists)
};
static StaticScratch g_static[kMaxDevices];

struct hps_table {
  uint64_t capacity, n_slots, max_keys, max_bags;
  uint32_t dim, acc_len;
  hps_optimizer opt;
  TableView view;
  char* ws;
  WorkspaceLayout wl;
  int lpr;
  bool mean_pooling;        // bags are averaged instead of summed (hps_set_pooling)
  uint64_t lookup_serial;   // lookups so far; lookup s lists its frequent keys in ring slot s % 3
  int dedup_mode;      // 0: by size and history; 1: plain radix passes always; 2: bucket path whenever it can
  bool ordered_rank;   // the GPU's LDS atomics serve a wave's lanes in lane order (sort.hpp: digit_rank)
  // How much of pull_lookup's per-block list of created keys is used: all of it, unless
  // HPS_LOOKUP_NEW_LIST says less (tests of what happens when it is full).
  u32 lookup_new_cap;
  // The pooling kernel keeps the most frequent keys' rows in LDS (HPS_POOL=lds).  Off unless
  // asked for: measured slower than reading them through L2 on every workload (the hash probe
  // per occurrence costs more than the L2 hits it saves, and the LDS halves the occupancy).
  bool hot_rows;
  uint64_t serial;     // number of dedups so far (status words carry it modulo kEpochMod)
  uint64_t plain_serial;   // ... of them in the plain form
  // Pinned host word the lookups report into (table.hpp: OftenLists::report).  When a dedup
  // of the bucket form had to order much of its input the slow way (keys bunched inside
  // their range, or frequent keys that change from one mini-batch to the next), the
  // following dedups take the plain form, which copes with both: for kPlainHold dedups, and
  // twice as long each time in a row the bucket form then disappoints again.
  unsigned long long* report;
  uint32_t report_seen;     // serial of the last report acted on
  uint32_t strikes;
  uint64_t plain_until;     // dedups numbered below this take the plain form
  uint64_t n_fallbacks;     // times plain_until was pushed out
  // The same for the plain form itself: after a dedup whose keys agreed in all the bits the
  // plain form sorts by (table.hpp: kReportMixed), the following ones sort by all 64 bits.
  uint32_t full_strikes;
  uint64_t full_until;
  uint64_t n_full_fallbacks;

  // Pull contexts.  `current` is the context of the outstanding pull (-1: none),
  // `prepared` the one whose dedup has been enqueued but not yet pulled (-1: none).
  struct Context {
    uint64_t n_keys, n_bags;
    const int32_t* d_offsets;
    bool mean;            // pooling of this pull (fixed when it is prepared)
    hipEvent_t ready;     // recorded after the dedup kernels
    hipEvent_t released;  // recorded after the push that used the context
    bool ready_set, released_set;
  } cx[2];
  int current, prepared;
  hipEvent_t scratch_free;   // the last dedup's end: the sort scratch is shared
  bool scratch_set;
  uint64_t last_n_keys;      // of the most recent pull, for hps_stats

  // stage timing (measurement only)
  uint32_t timing_mask;
  std::vector<hipEvent_t> ev_pool[HPS_N_STAGES];   // begin/end alternate
  size_t ev_used[HPS_N_STAGES];

  template <typename T> T* w(size_t off) const { return reinterpret_cast<T*>(ws + off); }
  PullCtx* ctx(int c) const { return w<PullCtx>(wl.c[c].ctx); }
};

namespace {
constexpr size_t kMaxEventPairs = 4096;

void stage_mark(hps_table* t, int stage, hipStream_t s) {
  if (!(t->timing_mask & (1u << stage))) return;
  std::vector<hipEvent_t>& pool = t->ev_pool[stage];
  if (t->ev_used[stage] >= 2 * kMaxEventPairs) return;
  if (t->ev_used[stage] == pool.size()) {
    hipEvent_t e;
    if (hipEventCreate(&e) != hipSuccess) return;
    pool.push_back(e);
  }
  (void)hipEventRecord(pool[t->ev_used[stage]++], s);
}
}  // namespace

// Rows of frequent keys the pooling kernel keeps in LDS: as many as fit kHotBytes.  A key is
// listed by the lookup if it has at least n / (8 * cap) occurrences, so that at most 8 * cap
// keys can qualify and usually far fewer do.
static u32 hot_capacity(uint32_t dim) {
  const u32 cap = kHotBytes / (dim * 4);
  return cap < kMaxHot ? cap : kMaxHot;
}

template <int LPR>
static void launch_pool(hps_table* t, int c, float* d_pooled, hipStream_t s) {
  const hps_table::Context& cx = t->cx[c];
  // (a block has 256 / LPR lane groups with eight rows in flight each: wide rows need more
  // blocks for as many rows in flight; d = 64: 0.293 ms with 1024 blocks, 0.247 with 4096, while
  // d = 16 runs the same with 1024 to 3072)
  const unsigned blocks = grid_for(cx.n_bags, kPoolThreads / LPR, kPoolMaxBlocks * (LPR > 4 ? LPR / 4 : 1));
  float* inv_len = cx.mean ? t->w<float>(t->wl.c[c].inv_len) : nullptr;
  const u32 cap = hot_capacity(t->dim);
  const bool hot = t->hot_rows && cap >= 8;
#define HPS_POOL(COLS, HOT)                                                                     \
  pool_bags<LPR, COLS, HOT><<<blocks, kPoolThreads, 0, s>>>(                                    \
      t->view, cx.d_offsets, (u32)cx.n_bags, (u32)cx.n_keys, t->w<i32>(t->wl.c[c].inverse),     \
      t->w<u32>(t->wl.c[c].rows), d_pooled, inv_len, t->w<uint2>(t->wl.c[c].hot_list),          \
      &t->ctx(c)->n_hot, cap)
  if (t->dim <= (uint32_t)LPR * 4) {
    if (hot) HPS_POOL(1, true); else HPS_POOL(1, false);
  } else {
    if (hot) HPS_POOL(4, true); else HPS_POOL(4, false);
  }
#undef HPS_POOL
}

template <int LPR>
static void launch_push(hps_table* t, uint64_t n, PushArgs& a, hipStream_t s) {
  a.short_blocks = grid_for(n, kPushThreads / LPR, kPushShortBlocks);
  a.medium_blocks = kPushMediumBlocks;
  const unsigned chunk_blocks = grid_for(n / kChunk + 1, 1, kPushChunkBlocks);
  const unsigned main_blocks = a.short_blocks + a.medium_blocks + chunk_blocks + (a.ring ? 1 : 0);
  const unsigned long_blocks = grid_for(n / (kMedSeg + 1) + 1, 1, kPushLongBlocks);
  if (t->dim <= (uint32_t)LPR * 4) {
    push_main<LPR, 1><<<main_blocks, kPushThreads, 0, s>>>(t->view, a);
    push_long<LPR, 1><<<long_blocks, kPushThreads, 0, s>>>(t->view, a);
  } else {
    push_main<LPR, 4><<<main_blocks, kPushThreads, 0, s>>>(t->view, a);
    push_long<LPR, 4><<<long_blocks, kPushThreads, 0, s>>>(t->view, a);
  }
}

// a1 for context c: the kernels that turn (keys, offsets) into uniq / inverse / bagperm /
// seg_off.  d_offsets == nullptr: every occurrence is its own bag.
static void launch_dedup(hps_table* t, int c, const uint64_t* d_keys, u32 n,
                         const int32_t* d_offsets, u32 n_bags, hipStream_t s) {
  const WorkspaceLayout& L = t->wl;
  const ContextLayout& C = L.c[c];
  PullCtx* ctx = t->ctx(c);
  if (n == 0) {
    set_ctx_empty<<<1, 64, 0, s>>>(ctx, t->w<u32>(C.seg_off));
  } else {
    // a1: order the occurrences by the top bits of their keys
    stage_mark(t, HPS_STAGE_SORT, s);
    ++t->serial;
    const u32 epoch = (u32)(t->serial % kEpochMod) + 1;
    if (epoch == 1 && t->serial >= kEpochMod)   // the epochs start over: forget the old words
      fill_u64<<<1024, 256, 0, s>>>(t->w<u64>(L.tile_rows), (L.evidence - L.tile_rows) / 8, 0);
    // The bucket path needs to know the heavy keys, which it learns from the lookups: the
    // first two dedups of a table take the plain passes, as do very large ones.
    if (t->dedup_mode == 0) {
      const unsigned long long r = __atomic_load_n(t->report, __ATOMIC_RELAXED);
      const uint32_t serial = (uint32_t)r, flags = (uint32_t)(r >> 32);
      if (serial != t->report_seen) {
        t->report_seen = serial;
        if ((flags & kReportBucket) && (flags & kReportSlow) && (flags & kReportOneKey)) {
          // a few keys turned frequent without warning: plain until the hint has caught up
          t->plain_until = t->serial + kHintLag;
          ++t->n_fallbacks;
        } else if ((flags & kReportBucket) && (flags & kReportSlow)) {
          t->plain_until = t->serial + ((uint64_t)kPlainHold << (t->strikes < 7 ? t->strikes : 7));
          ++t->strikes;
          ++t->n_fallbacks;
        } else if (flags & kReportBucket) {
          t->strikes = 0;
        }
        if (flags & kReportMixed) {
          // the plain form's sorted bits did not tell the keys apart: all 64 bits for a while
          t->full_until = t->serial + ((uint64_t)kPlainHold << (t->full_strikes < 7 ? t->full_strikes : 7));
          ++t->full_strikes;
          ++t->n_full_fallbacks;
        } else if (!(flags & kReportBucket) && t->serial >= t->full_until) {
          t->full_strikes = 0;       // the plain form with its usual passes did well
        }
      }
    }
    const bool buckets = n <= kBucketPathMaxKeys && t->dedup_mode != 1 &&
                         (t->dedup_mode == 2 || (t->lookup_serial >= 2 && t->serial >= t->plain_until));
    const SortPlan plan = buckets ? bucket_plan(n) : sort_plan(n, t->dedup_mode != 2 && t->serial < t->full_until);
    u64* kcur = t->w<u64>(L.keys_a);
    u64* kalt = t->w<u64>(L.keys_b);
    u64* pcur = t->w<u64>(L.idx_a);
    u64* palt = t->w<u64>(L.idx_b);
    u32* tickets = t->w<u32>(L.tickets);
    const unsigned n_tiles = (n + kSortTile - 1) / kSortTile;
    const unsigned bag_blocks = grid_for(d_offsets ? n_bags : n, kPrepThreads, 256);
    if (buckets) {
      // the most recent list of frequent keys that is certainly complete (common.hpp)
      const HeavySet* heavy =
          &t->w<HeavyRing>(L.heavy_raw)->set[(t->lookup_serial + kHeavyRing - 1) % kHeavyRing];
      const unsigned count_blocks = n_tiles < 1024 ? n_tiles : 1024;
      const unsigned n_regions = (n + kRegionSpan - 1) / kRegionSpan;
      u32* hist = t->w<u32>(L.part_hist);
      u32* tot = t->w<u32>(L.part_tot);
      uint8_t* dig = plan.n_pass == 2 ? t->w<uint8_t>(L.dig) : nullptr;
      bucket_count<<<count_blocks + bag_blocks, kPrepThreads, 0, s>>>(
          d_keys, n, plan, tickets, ctx, d_offsets, n_bags, t->w<i32>(L.bag_of), heavy,
          t->w<uint16_t>(L.id16), hist, n_tiles, count_blocks);
      // (the first scan also clears the status words of region_sort_emit: one per region and
      // one per group of regions, laid out back to back)
      scan_tiles<<<kRadix, kPartThreads, 0, s>>>(hist, n_tiles, tot, t->w<u32>(L.head_rows),
                                                 (u32)((L.evidence - L.head_rows) / 4));
#define HPS_SCATTER(FIRST, ...)                                                          \
  do {                                                                                  \
    if (t->ordered_rank) scatter_pass<FIRST, true><<<n_tiles, kPartThreads, 0, s>>>(__VA_ARGS__);  \
    else scatter_pass<FIRST, false><<<n_tiles, kPartThreads, 0, s>>>(__VA_ARGS__);      \
  } while (0)
      HPS_SCATTER(true, d_keys, nullptr, t->w<i32>(L.bag_of), t->w<uint16_t>(L.id16), nullptr, kcur, pcur,
                  dig, n, hist, n_tiles, tot);
      if (plan.n_pass == 2) {
        digit_count<<<n_tiles, kPartThreads, 0, s>>>(dig, n, hist, n_tiles);
        scan_tiles<<<kRadix, kPartThreads, 0, s>>>(hist, n_tiles, tot, nullptr, 0);
        HPS_SCATTER(false, kcur, pcur, nullptr, nullptr, dig, kalt, palt, nullptr, n, hist, n_tiles, tot);
        u64* tk = kcur; kcur = kalt; kalt = tk;
        tk = pcur; pcur = palt; palt = tk;
      }
      stage_mark(t, HPS_STAGE_SORT, s);
      // a1: unique keys, ranks, grouping
      stage_mark(t, HPS_STAGE_UNIQUE, s);
      u32* borders = t->w<u32>(L.borders);
      region_borders<<<(n_regions + 1 + kPartWaves - 1) / kPartWaves, kPartThreads, 0, s>>>(
          kcur, n, n_regions, plan.max_heavy, heavy, ctx, borders);
#undef HPS_SCATTER
      // region_sort's notes for region_emit: heads per region and per group of regions (the
      // status words the first scan cleared), how each region was ordered, and the order itself
      // (in bag_of, which the first scatter has finished with)
      u32* region_heads = t->w<u32>(L.head_rows);
      u32* region_kind = t->w<u32>(L.head_rows) + L.head_tiles;
      u32* group_heads = t->w<u32>(L.head_groups);
      u32* order = t->w<u32>(L.bag_of);
#define HPS_REGIONS(ORDERED)                                                                       \
  region_sort<kChunkItems, ORDERED><<<n_regions, kChunkThreads, 0, s>>>(                           \
      kcur, pcur, kalt, palt, t->w<u64>(L.keys_c), t->w<u64>(L.idx_c), n, borders, region_kind,    \
      region_heads, group_heads, order, ctx)
      if (t->ordered_rank) HPS_REGIONS(true);
      else HPS_REGIONS(false);
#undef HPS_REGIONS
      region_emit<<<n_regions, kChunkThreads, 0, s>>>(
          kcur, pcur, kalt, palt, t->w<u64>(L.keys_c), t->w<u64>(L.idx_c), n, borders, region_kind,
          region_heads, group_heads, order, n_bags, t->w<u64>(C.uniq), t->w<i32>(C.inverse),
          t->w<u32>(C.bagperm), t->w<u32>(C.seg_off), ctx, t->view.st);
    } else {
      // two sets of digit histograms: a plain dedup counts into one and clears the other for
      // the next plain dedup
      ++t->plain_serial;
      u32* ghist = t->w<u32>(L.ghist) + (t->plain_serial & 1) * kHistWords;
      u32* ghist_next = t->w<u32>(L.ghist) + ((t->plain_serial + 1) & 1) * kHistWords;
      const unsigned hist_blocks = n_tiles < 768 ? n_tiles : 768;
      sort_prepare<<<hist_blocks + bag_blocks, kPrepThreads, 0, s>>>(
          d_keys, n, plan, ghist, ghist_next, tickets, ctx, d_offsets, n_bags, t->w<i32>(L.bag_of),
          hist_blocks);
      for (int p = 0; p < plan.n_pass; ++p) {
        u32* tile_rows = t->w<u32>(L.tile_rows) + (size_t)p * L.sort_tiles * kRadix;
        u32* group_rows = t->w<u32>(L.group_rows) + (size_t)p * (L.sort_tiles / kMinTileGroup + 1) * kRadix;
        const int shift = p * kRadixBits;     // within the key's sorted prefix
        if (p == 0) {
          onesweep_pass<true><<<n_tiles, kSortThreads, 0, s>>>(
              d_keys, nullptr, t->w<i32>(L.bag_of), kcur, pcur, n, shift, ghist + p * kRadix, tile_rows,
              group_rows, plan.group, tickets + p, epoch, ctx);
        } else {
          onesweep_pass<false><<<n_tiles, kSortThreads, 0, s>>>(
              kcur, pcur, t->w<i32>(L.bag_of), kalt, palt, n, shift, ghist + p * kRadix, tile_rows,
              group_rows, plan.group, tickets + p, epoch, ctx);
          u64* tk = kcur; kcur = kalt; kalt = tk;
          tk = pcur; pcur = palt; palt = tk;
        }
      }
      stage_mark(t, HPS_STAGE_SORT, s);
      // a1: unique keys, ranks, grouping; the second unique_emit only acts after a repair
      stage_mark(t, HPS_STAGE_UNIQUE, s);
      const unsigned head_tiles = (n + kHeadTile - 1) / kHeadTile;
      const u32 head_group = tile_group(head_tiles);
      u32* evidence = t->w<u32>(L.evidence);
      unique_emit<false><<<head_tiles, kHeadThreads, 0, s>>>(
          kcur, pcur, n, t->w<u32>(L.head_rows), t->w<u32>(L.head_groups), head_group,
          tickets + kMaxPasses, epoch, n_bags, t->w<u64>(C.uniq),
          t->w<i32>(C.inverse), t->w<u32>(C.bagperm), t->w<u32>(C.seg_off), ctx, evidence, t->view.st);
      fix_mixed_runs<<<1, kFixThreads, 0, s>>>(kcur, pcur, kalt, palt, n, ctx, evidence);
      unique_emit<true><<<head_tiles, kHeadThreads, 0, s>>>(
          kcur, pcur, n, t->w<u32>(L.head_rows) + L.head_tiles,
          t->w<u32>(L.head_groups) + (L.head_tiles / kMinTileGroup + 1), head_group,
          tickets + kMaxPasses + 1, epoch, n_bags, t->w<u64>(C.uniq),
          t->w<i32>(C.inverse), t->w<u32>(C.bagperm), t->w<u32>(C.seg_off), ctx, evidence, t->view.st);
    }
    stage_mark(t, HPS_STAGE_UNIQUE, s);
  }
}

// a2 without creating anything, for context c: rows of the unique keys (kNoRow for a
// key the table does not hold) and the push's work lists.
static void launch_lookup(hps_table* t, int c, uint64_t n_keys, bool create, hipStream_t s) {
  const ContextLayout& C = t->wl.c[c];
  PullCtx* ctx = t->ctx(c);
  OftenLists often;
  often.seg_off = t->w<u32>(C.seg_off);
  often.ctx = ctx;
  often.med_list = t->w<u32>(t->wl.med_list);
  often.med_cap = (u32)t->wl.med_cap;
  often.long_list = t->w<uint2>(t->wl.long_list);
  often.chunk_items = t->w<uint2>(t->wl.chunk_items);
  ++t->lookup_serial;
  often.heavy_raw = &t->w<HeavyRing>(t->wl.heavy_raw)->raw[t->lookup_serial % kHeavyRing];
  often.heavy_min = (u32)(n_keys / kHeavyShare > kHeavyMin ? n_keys / kHeavyShare : kHeavyMin);
  often.hot_list = t->w<uint2>(C.hot_list);
  often.hot_cap = hot_capacity(t->dim);
  // at most 8 * cap keys can have this many occurrences; 0 occurrences never qualify
  often.hot_min = ~0u;                       // nothing is listed
  if (t->hot_rows && often.hot_cap >= 8)
    often.hot_min = (u32)(n_keys / (8ull * often.hot_cap) > 8 ? n_keys / (8ull * often.hot_cap) : 8);
  often.report = t->report;
  often.serial = (u32)t->lookup_serial;
  const unsigned probe_blocks = grid_for(n_keys, kLookupGroups * kPullInFlight, kProbeMaxBlocks);
  pull_lookup<<<probe_blocks, kProbeThreads, 0, s>>>(
      t->view, t->w<u64>(C.uniq), &ctx->n_unique, t->w<u32>(C.rows), t->w<u32>(t->wl.miss_list),
      (u32)t->wl.shard_cap, create ? 1u : 0u, t->lookup_new_cap, often);

}

static void fill_push_args(hps_table* t, int c, const float* d_rows, int kind, PushArgs& a) {
  const WorkspaceLayout& L = t->wl;
  a.seg_off = t->w<u32>(L.c[c].seg_off);
  a.bagperm = t->w<u32>(L.c[c].bagperm);
  a.rows = t->w<u32>(L.c[c].rows);
  a.grads = d_rows;
  a.inv_len = nullptr;
  a.ctx = t->ctx(c);
  a.med_list = t->w<u32>(L.med_list);
  a.med_cap = (u32)L.med_cap;
  a.long_list = t->w<uint2>(L.long_list);
  a.chunk_items = t->w<uint2>(L.chunk_items);
  a.partials = t->w<float>(L.partials);
  a.lr = t->opt.lr;
  a.eps = t->opt.eps;
  a.kind = kind;
  a.ring = nullptr;
  a.ring_slot = 0;
}

// Whether the GPU's LDS atomics serve the lanes of one instruction in ascending lane order
// (sort.hpp: digit_rank), measured once per device: 0 not yet, 1 yes, 2 no.  uses the table's (not yet
// initialised) state block for the result; waits for the stream.  HPS_RANK=ballot / ordered overrides
// the measurement (comparison runs, tests).
static int g_lane_order[64];

static bool lane_order_holds(TableState* st, hipStream_t s) {
  static_assert(offsetof(TableState, miss_overflow) % 8 == 0 &&
                    offsetof(TableState, probe_bad) == offsetof(TableState, miss_overflow) + 4,
                "the two words are cleared as one");
  u32* word = &st->probe_bad;
  const char* force = std::getenv("HPS_RANK");
  if (force && std::strcmp(force, "ballot") == 0) return false;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) { (void)hipGetLastError(); return false; }
  int state = __atomic_load_n(&g_lane_order[dev], __ATOMIC_ACQUIRE);
  if (state == 0) {
    u32 bad = 1;
    fill_u64<<<1, 64, 0, s>>>(reinterpret_cast<u64*>(&st->miss_overflow), 1, 0);
    probe_lane_order<<<256, kSortThreads, 0, s>>>(64, word);
    if (hipMemcpyAsync(&bad, word, sizeof(bad), hipMemcpyDeviceToHost, s) != hipSuccess ||
        hipStreamSynchronize(s) != hipSuccess) {
      (void)hipGetLastError();
      return false;
    }
    state = bad == 0 ? 1 : 2;
    __atomic_store_n(&g_lane_order[dev], state, __ATOMIC_RELEASE);
  }
  return state == 1;
}

#define HPS_DISPATCH_LPR(lpr, CALL)            \
  switch (lpr) {                               \
    case 1: CALL(1); break;                    \
    case 2: CALL(2); break;                    \
    case 4: CALL(4); break;                    \
    case 8: CALL(8); break;                    \
    case 16: CALL(16); break;                  \
    case 32: CALL(32); break;                  \
    default: CALL(64); break;                  \
  }

extern "C" {

const char* hps_strerror(hps_status s) {
  switch (s) {
    case HPS_OK: return "ok";
    case HPS_EINVAL: return "invalid argument";
    case HPS_EFULL: return "table full";
    case HPS_ERESERVED: return "reserved key 0xFFFFFFFFFFFFFFFF in input";
    case HPS_ESTATE: return "call not valid in this state";
    case HPS_EDEVICE: return "HIP call failed or no usable GPU";
    case HPS_ENOMEM: return "buffer too small";
  }
  return "unknown status";
}

size_t hps_table_bytes(uint64_t capacity_keys, uint32_t dim, const hps_optimizer* opt) {
  if (!valid_opt(opt) || !valid_shape(capacity_keys, dim)) return 0;
  const uint32_t acc_len = opt->kind == HPS_OPT_ADAGRAD_ELEMENTWISE ? dim : 1;
  return storage_layout(slots_for(capacity_keys), dim, acc_len, opt->row_format).total;
}

size_t hps_workspace_bytes(uint64_t max_keys, uint64_t max_bags, uint32_t dim) {
  if (max_keys >= (1ull << 30) || max_bags >= (1ull << 31) || dim < 4 || dim > 1024 || dim % 4)
    return 0;
  return workspace_layout(max_keys, max_bags, dim).total;
}

hps_status hps_create(hps_table** out, uint64_t capacity_keys, uint32_t dim,
                      const hps_optimizer* opt, void* d_storage, size_t storage_bytes,
                      void* d_workspace, size_t workspace_bytes, uint64_t max_keys,
                      uint64_t max_bags, void* stream) {
  if (!out) return HPS_EINVAL;
  *out = nullptr;
  if (!valid_opt(opt) || !valid_shape(capacity_keys, dim)) return HPS_EINVAL;
  if (!d_storage || !d_workspace) return HPS_EINVAL;
  if ((uintptr_t)d_storage % kAlign || (uintptr_t)d_workspace % kAlign) return HPS_EINVAL;
  if (max_keys >= (1ull << 30) || max_bags >= (1ull << 31)) return HPS_EINVAL;
  const uint32_t acc_len = opt->kind == HPS_OPT_ADAGRAD_ELEMENTWISE ? dim : 1;
  const uint64_t n_slots = slots_for(capacity_keys);
  const StorageLayout sl = storage_layout(n_slots, dim, acc_len, opt->row_format);
  const WorkspaceLayout wl = workspace_layout(max_keys, max_bags, dim);
  if (storage_bytes < sl.total || workspace_bytes < wl.total) return HPS_ENOMEM;
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return HPS_EDEVICE; }

  hps_table* t = new (std::nothrow) hps_table();
  if (!t) return HPS_ENOMEM;
  t->capacity = capacity_keys;
  t->n_slots = n_slots;
  t->max_keys = max_keys;
  t->max_bags = max_bags;
  t->dim = dim;
  t->acc_len = acc_len;
  t->opt = *opt;
  char* base = static_cast<char*>(d_storage);
  t->view.keys = reinterpret_cast<u64*>(base + sl.keys);
  t->view.w = base + sl.w;
  t->view.acc = base + sl.acc;
  t->view.w_pitch = sl.w_pitch;
  t->view.acc_pitch = sl.acc_pitch;
  t->view.st = reinterpret_cast<TableState*>(base + sl.state);
  t->view.n_lines = n_slots / kSlotsPerLine;
  t->view.capacity = capacity_keys;
  t->view.dim = dim;
  t->view.acc_len = acc_len;
  t->view.init_acc = opt->init_acc;
  t->view.init_range = opt->init_range;
  t->view.init_seed = opt->init_seed;
  t->view.bf16 = opt->row_format == HPS_ROWS_BF16 ? 1u : 0u;
  t->ws = static_cast<char*>(d_workspace);
  t->wl = wl;
  t->lpr = lanes_per_row(dim);
  t->current = t->prepared = -1;
  t->last_n_keys = 0;
  t->scratch_set = false;
  bool events_ok = hipEventCreateWithFlags(&t->scratch_free, hipEventDisableTiming) == hipSuccess;
  for (int k = 0; k < 2; ++k) {
    t->cx[k].n_keys = t->cx[k].n_bags = 0;
    t->cx[k].d_offsets = nullptr;
    t->cx[k].ready_set = t->cx[k].released_set = false;
    events_ok = events_ok &&
                hipEventCreateWithFlags(&t->cx[k].ready, hipEventDisableTiming) == hipSuccess &&
                hipEventCreateWithFlags(&t->cx[k].released, hipEventDisableTiming) == hipSuccess;
  }
  t->report = nullptr;
  if (!events_ok) { (void)hipGetLastError(); hps_destroy(t); return HPS_EDEVICE; }
  t->timing_mask = 0;
  for (int i = 0; i < HPS_N_STAGES; ++i) t->ev_used[i] = 0;
  t->serial = 0;
  t->plain_serial = 0;
  t->mean_pooling = false;
  t->lookup_serial = 0;
  t->report_seen = 0;
  t->strikes = 0;
  t->plain_until = 0;
  t->n_fallbacks = 0;
  t->full_strikes = 0;
  t->full_until = 0;
  t->n_full_fallbacks = 0;
  t->report = nullptr;
  if (hipHostMalloc(reinterpret_cast<void**>(&t->report), 64, hipHostMallocDefault) != hipSuccess) {
    (void)hipGetLastError();
    hps_destroy(t);
    return HPS_EDEVICE;
  }
  *t->report = 0;
  {
    // HPS_DEDUP=radix / bucket pins the dedup to one of its two forms (comparison runs, tests)
    const char* mode = std::getenv("HPS_DEDUP");
    t->dedup_mode = !mode ? 0 : std::strcmp(mode, "radix") == 0 ? 1 : std::strcmp(mode, "bucket") == 0 ? 2 : 0;
  }

  t->lookup_new_cap = kNewLdsCap;
  if (const char* cap = std::getenv("HPS_LOOKUP_NEW_LIST")) {
    const unsigned n = (unsigned)std::strtoul(cap, nullptr, 10);
    t->lookup_new_cap = n < kNewLdsCap ? n : kNewLdsCap;
  }
  {
    const char* pool = std::getenv("HPS_POOL");
    t->hot_rows = pool && std::strcmp(pool, "lds") == 0;
  }
  hipStream_t s = static_cast<hipStream_t>(stream);
  t->ordered_rank = lane_order_holds(t->view.st, s);
  fill_u64<<<4096, 256, 0, s>>>(t->view.keys, n_slots, kEmptyKey);
  // look-back status words and digit histograms start at zero
  fill_u64<<<1024, 256, 0, s>>>(t->w<u64>(wl.ghist), (wl.bag_of - wl.ghist) / 8, 0);
  for (u32 k = 0; k < kHeavyRing; ++k)
    init_heavy_set<<<1, 256, 0, s>>>(&t->w<HeavyRing>(wl.heavy_raw)->set[k]);
  reset_state<<<1, 64, 0, s>>>(t->view.st);
  for (int k = 0; k < 2; ++k)
    set_ctx_empty<<<1, 64, 0, s>>>(t->ctx(k), t->w<u32>(wl.c[k].seg_off));
  if (!launch_ok()) { hps_destroy(t); return HPS_EDEVICE; }
  *out = t;
  return HPS_OK;
}

hps_status hps_destroy(hps_table* t) {
  if (!t) return HPS_EINVAL;
  for (int i = 0; i < HPS_N_STAGES; ++i)
    for (hipEvent_t e : t->ev_pool[i]) (void)hipEventDestroy(e);
  // (a table whose creation failed half way holds null handles)
  if (t->scratch_free) (void)hipEventDestroy(t->scratch_free);
  for (int k = 0; k < 2; ++k) {
    if (t->cx[k].ready) (void)hipEventDestroy(t->cx[k].ready);
    if (t->cx[k].released) (void)hipEventDestroy(t->cx[k].released);
  }
  if (t->report) (void)hipHostFree(t->report);     // waits for the device: no lookup still writes to it
  delete t;
  return HPS_OK;
}

hps_status hps_clear(hps_table* t, void* stream) {
  if (!t) return HPS_EINVAL;
  if (t->current >= 0 || t->prepared >= 0) return HPS_ESTATE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  // rows and accumulators need no clearing: a slot's row is written when its key is
  // claimed, and the marks of updated rows live in the accumulators
  fill_u64<<<4096, 256, 0, s>>>(t->view.keys, t->n_slots, kEmptyKey);
  reset_state<<<1, 64, 0, s>>>(t->view.st);
  return launch_ok() ? HPS_OK : HPS_EDEVICE;
}

hps_status hps_insert(hps_table* t, const uint64_t* d_keys, uint64_t n, const float* d_weights,
                      const float* d_acc, void* stream) {
  if (!t || (n && !d_keys) || (d_acc && !d_weights)) return HPS_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const unsigned blocks = grid_for(n, kProbeGroups * kProbeInFlight, kProbeMaxBlocks);
  const unsigned lookup_blocks = grid_for(n, kLookupGroups * kProbeInFlight, kProbeMaxBlocks);
  if (n) {
    if (d_weights)
      lookup_keys<2><<<lookup_blocks, kProbeThreads, 0, s>>>(t->view, d_keys, n, nullptr, d_weights, d_acc,
                                                             nullptr, nullptr, nullptr);
    else
      lookup_keys<1><<<lookup_blocks, kProbeThreads, 0, s>>>(t->view, d_keys, n, nullptr, nullptr, nullptr,
                                                             nullptr, nullptr, nullptr);
    insert_missing<<<blocks, kProbeThreads, 0, s>>>(t->view, d_keys, n, nullptr, nullptr, d_weights,
                                                    d_acc, nullptr, 0);
  }
  commit_insert<<<1, 64, 0, s>>>(t->view.st);
  return launch_ok() ? HPS_OK : HPS_EDEVICE;
}

static bool mini_batch_ok(const hps_table* t, const uint64_t* d_keys, uint64_t n_keys,
                          const int32_t* d_offsets, uint32_t n_examples, uint32_t n_slots) {
  if (!t || !d_offsets || (n_keys && !d_keys)) return false;
  if (n_keys > t->max_keys || (uint64_t)n_examples * n_slots > t->max_bags) return false;
  if (n_keys && (uint64_t)n_examples * n_slots == 0) return false;      // keys, but no bag to hold them
  return (uintptr_t)d_keys % 8 == 0 && (uintptr_t)d_offsets % 4 == 0;
}

hps_status hps_prepare(hps_table* t, const uint64_t* d_keys, uint64_t n_keys,
                       const int32_t* d_offsets, uint32_t n_examples, uint32_t n_slots,
                       void* stream) {
  if (!mini_batch_ok(t, d_keys, n_keys, d_offsets, n_examples, n_slots)) return HPS_EINVAL;
  const uint64_t n_bags = (uint64_t)n_examples * n_slots;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int c = t->current == 0 ? 1 : 0;        // the context the outstanding pull does not use
  hps_table::Context& cx = t->cx[c];
  const u32 n = (u32)n_keys;
  // order after the push that last read this context, and after the previous dedup
  // (the sort scratch is shared); both may have run on other streams
  if (cx.released_set && hipStreamWaitEvent(s, cx.released, 0) != hipSuccess) return HPS_EDEVICE;
  if (t->scratch_set && hipStreamWaitEvent(s, t->scratch_free, 0) != hipSuccess) return HPS_EDEVICE;

  launch_dedup(t, c, d_keys, n, d_offsets, (u32)n_bags, s);
  if (!launch_ok()) return HPS_EDEVICE;
  if (hipEventRecord(cx.ready, s) != hipSuccess || hipEventRecord(t->scratch_free, s) != hipSuccess)
    return HPS_EDEVICE;
  cx.ready_set = true;
  t->scratch_set = true;
  cx.n_keys = n_keys;
  cx.n_bags = n_bags;
  cx.d_offsets = d_offsets;
  cx.mean = t->mean_pooling;
  t->prepared = c;
  return HPS_OK;
}

hps_status hps_pull_prepared(hps_table* t, float* d_pooled, void* stream) {
  if (!t) return HPS_EINVAL;
  if (t->prepared < 0 || t->current >= 0) return HPS_ESTATE;
  const int c = t->prepared;
  const hps_table::Context& cx = t->cx[c];
  if (cx.n_bags && !d_pooled) return HPS_EINVAL;
  if ((uintptr_t)d_pooled % 16) return HPS_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const ContextLayout& C = t->wl.c[c];
  PullCtx* ctx = t->ctx(c);
  if (hipStreamWaitEvent(s, cx.ready, 0) != hipSuccess) return HPS_EDEVICE;
  // the lookup rewrites the work lists that both contexts share and the pooling reads rows: order
  // them after the push of the mini-batch before, should that have run on another stream
  const hps_table::Context& other = t->cx[1 - c];
  if (other.released_set && hipStreamWaitEvent(s, other.released, 0) != hipSuccess) return HPS_EDEVICE;
  // a2: look up every unique key, create the missing ones
  stage_mark(t, HPS_STAGE_LOOKUP, s);
  if (cx.n_keys) {
    const unsigned probe_blocks = grid_for(cx.n_keys, kProbeGroups * kProbeInFlight, kProbeMaxBlocks);
    u32* miss_list = t->w<u32>(t->wl.miss_list);
    const u32 shard_cap = (u32)t->wl.shard_cap;
    launch_lookup(t, c, cx.n_keys, true, s);
    insert_missing<<<probe_blocks, kProbeThreads, 0, s>>>(t->view, t->w<u64>(C.uniq), 0,
                                                          &ctx->n_unique, t->w<u32>(C.rows), nullptr,
                                                          nullptr, miss_list, shard_cap);
  }
  if (!cx.n_bags) commit_insert<<<1, 64, 0, s>>>(t->view.st);   // else the pooling kernel does it
  stage_mark(t, HPS_STAGE_LOOKUP, s);
  // a3: gather rows and pool per bag
  if (cx.n_bags) {
    stage_mark(t, HPS_STAGE_POOL, s);
#define CALL(LPR) launch_pool<LPR>(t, c, d_pooled, s)
    HPS_DISPATCH_LPR(t->lpr, CALL)
#undef CALL
    stage_mark(t, HPS_STAGE_POOL, s);
  }
  if (!launch_ok()) return HPS_EDEVICE;
  t->current = c;
  t->prepared = -1;
  t->last_n_keys = cx.n_keys;
  return HPS_OK;
}

hps_status hps_pull(hps_table* t, const uint64_t* d_keys, uint64_t n_keys,
                    const int32_t* d_offsets, uint32_t n_examples, uint32_t n_slots,
                    float* d_pooled, void* stream) {
  if ((uint64_t)n_examples * n_slots && !d_pooled) return HPS_EINVAL;
  if ((uintptr_t)d_pooled % 16) return HPS_EINVAL;
  if (!mini_batch_ok(t, d_keys, n_keys, d_offsets, n_examples, n_slots)) return HPS_EINVAL;
  if (t->current >= 0) return HPS_ESTATE;
  const hps_status rc = hps_prepare(t, d_keys, n_keys, d_offsets, n_examples, n_slots, stream);
  return rc != HPS_OK ? rc : hps_pull_prepared(t, d_pooled, stream);
}

hps_status hps_push(hps_table* t, const float* d_pooled_grads, void* stream) {
  if (!t) return HPS_EINVAL;
  if (t->current < 0) return HPS_ESTATE;
  const int c = t->current;
  hps_table::Context& cx = t->cx[c];
  if (cx.n_bags && cx.n_keys && !d_pooled_grads) return HPS_EINVAL;
  if ((uintptr_t)d_pooled_grads % 16) return HPS_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(stream);
  t->current = -1;
  if (cx.n_keys && cx.n_bags) {
    PushArgs a;
    fill_push_args(t, c, d_pooled_grads,
                   t->opt.kind == HPS_OPT_ADAGRAD_ELEMENTWISE ? kStepElementwise : kStepRowwise, a);
    if (cx.mean) a.inv_len = t->w<float>(t->wl.c[c].inv_len);
    a.ring = t->w<HeavyRing>(t->wl.heavy_raw);       // the pull's lookup listed the frequent keys
    a.ring_slot = (u32)(t->lookup_serial % kHeavyRing);
    stage_mark(t, HPS_STAGE_PUSH, s);
#define CALL(LPR) launch_push<LPR>(t, cx.n_keys, a, s)
    HPS_DISPATCH_LPR(t->lpr, CALL)
#undef CALL
    stage_mark(t, HPS_STAGE_PUSH, s);
    if (!launch_ok()) return HPS_EDEVICE;
  }
  if (hipEventRecord(cx.released, s) != hipSuccess) return HPS_EDEVICE;
  cx.released_set = true;
  return HPS_OK;
}

hps_status hps_set_pooling(hps_table* t, int mean) {
  if (!t || (mean != 0 && mean != 1)) return HPS_EINVAL;
  if (t->current >= 0 || t->prepared >= 0) return HPS_ESTATE;
  t->mean_pooling = mean != 0;
  return HPS_OK;
}

// The kernels of an accumulate on context 0 of whatever workspace the table currently points to.
static hps_status accumulate_launches(hps_table* t, const uint64_t* d_keys, uint64_t n,
                                      const float* d_values, hipStream_t s) {
  const int c = 0;
  // every (key, value row) pair is a bag of its own: the dedup groups the pairs by key,
  // the push kernels sum each group's value rows and add the sum onto the row
  launch_dedup(t, c, d_keys, (u32)n, nullptr, (u32)n, s);
  if (n) {
    launch_lookup(t, c, n, false, s);
    commit_absent<<<1, 256, 0, s>>>(t->view.st, t->w<HeavyRing>(t->wl.heavy_raw),
                                   (u32)(t->lookup_serial % kHeavyRing));
    PushArgs a;
    fill_push_args(t, c, d_values, kStepAdd, a);
#define CALL(LPR) launch_push<LPR>(t, n, a, s)
    HPS_DISPATCH_LPR(t->lpr, CALL)
#undef CALL
  } else {
    commit_absent<<<1, 256, 0, s>>>(t->view.st, nullptr, 0);
  }
  return launch_ok() ? HPS_OK : HPS_EDEVICE;
}

hps_status hps_accumulate(hps_table* t, const uint64_t* d_keys, uint64_t n, const float* d_values,
                          void* stream) {
  if (!t || (n && (!d_keys || !d_values))) return HPS_EINVAL;
  if (n > t->max_keys || (uintptr_t)d_keys % 8 || (uintptr_t)d_values % 16) return HPS_EINVAL;
  if (t->current >= 0 || t->prepared >= 0) return HPS_ESTATE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  hps_table::Context& cx = t->cx[0];
  for (int k = 0; k < 2; ++k)      // after the last push of either context (shared work lists, table rows)
    if (t->cx[k].released_set && hipStreamWaitEvent(s, t->cx[k].released, 0) != hipSuccess) return HPS_EDEVICE;
  if (t->scratch_set && hipStreamWaitEvent(s, t->scratch_free, 0) != hipSuccess) return HPS_EDEVICE;
  const hps_status rc = accumulate_launches(t, d_keys, n, d_values, s);
  if (rc != HPS_OK) return rc;
  if (hipEventRecord(cx.released, s) != hipSuccess || hipEventRecord(t->scratch_free, s) != hipSuccess)
    return HPS_EDEVICE;
  cx.released_set = true;
  t->scratch_set = true;
  return HPS_OK;
}

hps_status hps_accumulate_static(hps_table* t, const uint64_t* d_keys, uint64_t n,
                                 const float* d_values, void* stream) {
  if (!t || (n && (!d_keys || !d_values))) return HPS_EINVAL;
  if (n > HPS_STATIC_MAX_KEYS || (uintptr_t)d_keys % 8 || (uintptr_t)d_values % 16) return HPS_EINVAL;
  if (t->current >= 0 || t->prepared >= 0) return HPS_ESTATE;
  const WorkspaceLayout wl = workspace_layout(HPS_STATIC_MAX_KEYS, HPS_STATIC_MAX_KEYS, t->dim);
  if (wl.total > kStaticScratchBytes) return HPS_EINVAL;       // rows too wide for the static array
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) { (void)hipGetLastError(); return HPS_EDEVICE; }
  StaticScratch& ss = g_static[dev];
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (!ss.ptr) {
    // this device's copy of the array: the name itself is no device address on the host
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) { (void)hipGetLastError(); return HPS_EDEVICE; }
    ss.ptr = static_cast<char*>(p);
    ss.ring_ready = false;
  }
  // The table works on the static array for the length of this call: its own workspace, and
  // what the host keeps about it, stay as they are.
  struct Saved {
    char* ws; WorkspaceLayout wl; uint64_t serial, plain_serial, lookup_serial, full_until;
    int dedup_mode; unsigned long long* report; uint32_t timing_mask;
  } keep = {t->ws, t->wl, t->serial, t->plain_serial, t->lookup_serial, t->full_until,
            t->dedup_mode, t->report, t->timing_mask};
  t->ws = ss.ptr;
  t->wl = wl;
  t->serial = t->plain_serial = 0;            // the status words are cleared below: any epoch will do
  t->lookup_serial = ss.lookup_serial;
  t->dedup_mode = 1;                           // plain passes ...
  t->full_until = ~0ull;                       // ... over all 64 key bits: exact whatever the keys, no history needed
  t->report = nullptr;
  t->timing_mask = 0;
  // what must start at zero: digit histograms, tickets, status words; once per device: the lists of frequent keys
  fill_u64<<<256, 256, 0, s>>>(t->w<u64>(wl.ghist), (wl.heavy_raw - wl.ghist) / 8, 0);
  if (!ss.ring_ready) {
    fill_u64<<<64, 256, 0, s>>>(t->w<u64>(wl.heavy_raw), (wl.bag_of - wl.heavy_raw) / 8, 0);
    for (u32 k = 0; k < kHeavyRing; ++k)
      init_heavy_set<<<1, 256, 0, s>>>(&t->w<HeavyRing>(wl.heavy_raw)->set[k]);
    ss.ring_ready = true;
  }
  set_ctx_empty<<<1, 64, 0, s>>>(t->ctx(0), t->w<u32>(wl.c[0].seg_off));
  const hps_status rc = accumulate_launches(t, d_keys, n, d_values, s);
  ss.lookup_serial = t->lookup_serial;
  t->ws = keep.ws;
  t->wl = keep.wl;
  t->serial = keep.serial;
  t->plain_serial = keep.plain_serial;
  t->lookup_serial = keep.lookup_serial;
  t->full_until = keep.full_until;
  t->dedup_mode = keep.dedup_mode;
  t->report = keep.report;
  t->timing_mask = keep.timing_mask;
  return rc;
}

hps_status hps_last_unique(hps_table* t, uint64_t* d_uniq_out, int32_t* d_inverse_out,
                           void* stream) {
  if (!t) return HPS_EINVAL;
  if (t->current < 0) return HPS_ESTATE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const ContextLayout& C = t->wl.c[t->current];
  const uint64_t n = t->cx[t->current].n_keys;
  if (n == 0) return HPS_OK;
  // U <= n is only known on the device: copy n entries, the caller reads the first U.
  if (d_uniq_out &&
      hipMemcpyAsync(d_uniq_out, t->w<u64>(C.uniq), n * 8, hipMemcpyDeviceToDevice, s) != hipSuccess)
    return HPS_EDEVICE;
  if (d_inverse_out &&
      hipMemcpyAsync(d_inverse_out, t->w<i32>(C.inverse), n * 4, hipMemcpyDeviceToDevice, s) != hipSuccess)
    return HPS_EDEVICE;
  return HPS_OK;
}

hps_status hps_get(hps_table* t, const uint64_t* d_keys, uint64_t n, float* d_weights_out,
                   float* d_acc_out, uint8_t* d_found_out, void* stream) {
  if (!t || (n && (!d_keys || !d_weights_out || !d_acc_out || !d_found_out))) return HPS_EINVAL;
  if (n == 0) return HPS_OK;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const unsigned blocks = grid_for(n, kLookupGroups * kProbeInFlight, kProbeMaxBlocks);
  lookup_keys<3><<<blocks, kProbeThreads, 0, s>>>(t->view, d_keys, n, nullptr, nullptr, nullptr,
                                                  d_weights_out, d_acc_out, d_found_out);
  return launch_ok() ? HPS_OK : HPS_EDEVICE;
}

static hps_status dump_impl(hps_table* t, bool dirty, uint64_t* d_keys_out, float* d_weights_out,
                            float* d_acc_out, uint64_t max_rows, uint64_t* h_n_rows, void* stream) {
  if (!t || !h_n_rows) return HPS_EINVAL;
  if (max_rows && (!d_keys_out || !d_weights_out || !d_acc_out)) return HPS_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(stream);
  clear_dump_count<<<1, 1, 0, s>>>(t->view.st);
  if (dirty)
    dump_rows<true><<<4096, 256, 0, s>>>(t->view, d_keys_out, d_weights_out, d_acc_out, max_rows,
                                         &t->view.st->dump_count);
  else
    dump_rows<false><<<4096, 256, 0, s>>>(t->view, d_keys_out, d_weights_out, d_acc_out, max_rows,
                                          &t->view.st->dump_count);
  if (!launch_ok()) return HPS_EDEVICE;
  unsigned long long count = 0;
  if (hipMemcpyAsync(&count, &t->view.st->dump_count, sizeof(count), hipMemcpyDeviceToHost, s) != hipSuccess)
    return HPS_EDEVICE;
  if (hipStreamSynchronize(s) != hipSuccess) return HPS_EDEVICE;
  *h_n_rows = count;
  return count > max_rows ? HPS_ENOMEM : HPS_OK;
}

hps_status hps_dump(hps_table* t, uint64_t* d_keys_out, float* d_weights_out, float* d_acc_out,
                    uint64_t max_rows, uint64_t* h_n_rows, void* stream) {
  return dump_impl(t, false, d_keys_out, d_weights_out, d_acc_out, max_rows, h_n_rows, stream);
}

hps_status hps_dump_dirty(hps_table* t, uint64_t* d_keys_out, float* d_weights_out,
                          float* d_acc_out, uint64_t max_rows, uint64_t* h_n_rows, void* stream) {
  if (t && t->current >= 0) return HPS_ESTATE;
  return dump_impl(t, true, d_keys_out, d_weights_out, d_acc_out, max_rows, h_n_rows, stream);
}

hps_status hps_stats(hps_table* t, hps_stats_t* h_out, void* stream) {
  if (!t || !h_out) return HPS_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(stream);
  TableState st;
  PullCtx ctx;
  if (hipMemcpyAsync(&st, t->view.st, sizeof(st), hipMemcpyDeviceToHost, s) != hipSuccess)
    return HPS_EDEVICE;
  const int which = t->current >= 0 ? t->current : (t->prepared >= 0 ? t->prepared : 0);
  if (hipMemcpyAsync(&ctx, t->ctx(which), sizeof(ctx), hipMemcpyDeviceToHost, s) != hipSuccess)
    return HPS_EDEVICE;
  if (hipStreamSynchronize(s) != hipSuccess) return HPS_EDEVICE;
  h_out->size = st.size;
  h_out->capacity = t->capacity;
  h_out->n_slots = t->n_slots;
  h_out->last_n_keys = t->last_n_keys;
  h_out->last_n_unique = ctx.n_unique;
  h_out->last_n_inserted = st.inserted;
  h_out->last_n_absent = (uint64_t)st.absent;
  h_out->n_plain_fallbacks = t->n_fallbacks;
  h_out->n_full_fallbacks = t->n_full_fallbacks;
  h_out->load_factor = (double)st.size / (double)t->n_slots;
  h_out->error = st.error;
  h_out->pull_outstanding = t->current >= 0 ? 1 : 0;
  return HPS_OK;
}

hps_status hps_probe_lengths(hps_table* t, double* h_mean, uint64_t* h_max, void* stream) {
  if (!t || !h_mean || !h_max) return HPS_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(stream);
  clear_probe_lengths<<<1, 1, 0, s>>>(t->view.st);
  probe_length_scan<<<4096, 256, 0, s>>>(t->view);
  if (!launch_ok()) return HPS_EDEVICE;
  TableState st;
  if (hipMemcpyAsync(&st, t->view.st, sizeof(st), hipMemcpyDeviceToHost, s) != hipSuccess ||
      hipStreamSynchronize(s) != hipSuccess)
    return HPS_EDEVICE;
  *h_mean = st.size ? (double)st.probe_sum / (double)st.size : 0.0;
  *h_max = st.probe_max;
  return HPS_OK;
}

hps_status hps_set_stage_timing(hps_table* t, uint32_t stage_mask) {
  if (!t || stage_mask >= (1u << HPS_N_STAGES)) return HPS_EINVAL;
  t->timing_mask = stage_mask;
  for (int i = 0; i < HPS_N_STAGES; ++i) t->ev_used[i] = 0;
  return HPS_OK;
}

hps_status hps_stage_times(hps_table* t, double* h_ms_sum, uint32_t* h_count) {
  if (!t || !h_ms_sum || !h_count) return HPS_EINVAL;
  hps_status rc = HPS_OK;
  for (int st = 0; st < HPS_N_STAGES; ++st) {
    h_ms_sum[st] = 0.0;
    h_count[st] = 0;
    const size_t pairs = t->ev_used[st] / 2;
    for (size_t p = 0; p < pairs; ++p) {
      float ms = 0.f;
      if (hipEventSynchronize(t->ev_pool[st][2 * p + 1]) != hipSuccess ||
          hipEventElapsedTime(&ms, t->ev_pool[st][2 * p], t->ev_pool[st][2 * p + 1]) != hipSuccess) {
        (void)hipGetLastError();
        rc = HPS_EDEVICE;
        continue;
      }
      h_ms_sum[st] += ms;
      h_count[st] += 1;
    }
    t->ev_used[st] = 0;
  }
  return rc;
}

hps_status hps_probe_random_rows(const void* d_rows, uint64_t n_rows, uint32_t row_bytes,
                                 uint64_t n_accesses, float* d_sink, void* stream) {
  if (!d_rows || !d_sink || n_rows == 0 || (uintptr_t)d_rows % 16) return HPS_EINVAL;
  if (row_bytes != 64 && row_bytes != 256) return HPS_EINVAL;
  const unsigned blocks = kPoolMaxBlocks;
  const uint64_t groups = (uint64_t)blocks * (kPoolThreads / (row_bytes / 16));
  uint64_t per_group = (n_accesses + groups - 1) / groups;
  per_group = (per_group + kPoolInFlight - 1) / kPoolInFlight * kPoolInFlight;
  if (per_group == 0 || per_group > 0xFFFFFFF0ull) return HPS_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (row_bytes == 64)
    random_row_probe<4><<<blocks, kPoolThreads, 0, s>>>(static_cast<const float4*>(d_rows), n_rows,
                                                        (u32)per_group, d_sink);
  else
    random_row_probe<16><<<blocks, kPoolThreads, 0, s>>>(static_cast<const float4*>(d_rows), n_rows,
                                                         (u32)per_group, d_sink);
  return launch_ok() ? HPS_OK : HPS_EDEVICE;
}

hps_status hps_clear_error(hps_table* t, void* stream) {
  if (!t) return HPS_EINVAL;
  clear_error<<<1, 64, 0, static_cast<hipStream_t>(stream)>>>(t->view.st);
  // While the status was set the kernels of a pull did nothing: what its context holds
  // (row numbers above all) may be an earlier mini-batch's, and a push must not use it.
  t->current = t->prepared = -1;
  return launch_ok() ? HPS_OK : HPS_EDEVICE;
}

// ---- the host-memory cache behind the table (include/hps_mem.h) --------------------------
struct hps_mem {
  hps::MemTier tier;
  hps_mem(uint32_t dim, uint32_t acc_len, uint64_t lru, uint64_t lfu) : tier(dim, acc_len, lru, lfu) {}
};

hps_status hps_mem_create(hps_mem** out, uint32_t dim, uint32_t acc_len, uint64_t lru_capacity,
                          uint64_t lfu_capacity) {
  if (!out) return HPS_EINVAL;
  *out = nullptr;
  if (dim == 0 || dim > 1024 || (acc_len != 1 && acc_len != dim)) return HPS_EINVAL;
  hps_mem* m = new (std::nothrow) hps_mem(dim, acc_len, lru_capacity, lfu_capacity);
  if (!m) return HPS_ENOMEM;
  *out = m;
  return HPS_OK;
}

hps_status hps_mem_fetch(hps_mem* m, const uint64_t* h_keys, uint64_t n, uint64_t batch, float* h_w,
                         float* h_acc, uint8_t* h_found) {
  if (!m || (n && (!h_keys || !h_w || !h_acc || !h_found))) return HPS_EINVAL;
  try { m->tier.fetch(h_keys, n, batch, h_w, h_acc, h_found); } catch (const std::bad_alloc&) { return HPS_ENOMEM; }
  return HPS_OK;
}

hps_status hps_mem_store(hps_mem* m, const uint64_t* h_keys, uint64_t n, const float* h_w,
                         const float* h_acc, uint64_t batch, int visit) {
  if (!m || (n && (!h_keys || !h_w || !h_acc)) || (visit != 0 && visit != 1)) return HPS_EINVAL;
  try { m->tier.store(h_keys, n, h_w, h_acc, batch, visit != 0); } catch (const std::bad_alloc&) { return HPS_ENOMEM; }
  return HPS_OK;
}

hps_status hps_mem_complete_batch(hps_mem* m, uint64_t batch) {
  if (!m) return HPS_EINVAL;
  try { m->tier.complete_batch(batch); } catch (const std::bad_alloc&) { return HPS_ENOMEM; }
  return HPS_OK;
}

hps_status hps_mem_take_evicted(hps_mem* m, uint64_t* h_keys, float* h_w, float* h_acc,
                                uint64_t max_rows, uint64_t* h_n) {
  if (!m || !h_n || (max_rows && (!h_keys || !h_w || !h_acc))) return HPS_EINVAL;
  *h_n = m->tier.take_evicted(h_keys, h_w, h_acc, max_rows);
  return m->tier.evicted_waiting() ? HPS_ENOMEM : HPS_OK;
}

hps_status hps_mem_list(hps_mem* m, int which, uint64_t* h_keys, uint64_t max, uint64_t* h_n) {
  if (!m || !h_n || (which != 0 && which != 1) || (max && !h_keys)) return HPS_EINVAL;
  *h_n = m->tier.list(which, h_keys, max);
  return HPS_OK;
}

hps_status hps_mem_stats(hps_mem* m, hps_mem_stats_t* h_out) {
  if (!m || !h_out) return HPS_EINVAL;
  h_out->lru_size = m->tier.lru_size();
  h_out->lfu_size = m->tier.lfu_size();
  h_out->pinned = m->tier.pinned();
  h_out->evicted_waiting = m->tier.evicted_waiting();
  h_out->hits = m->tier.hits();
  h_out->misses = m->tier.misses();
  return HPS_OK;
}

hps_status hps_mem_destroy(hps_mem* m) {
  if (!m) return HPS_EINVAL;
  delete m;
  return HPS_OK;
}

}  // extern "C"
