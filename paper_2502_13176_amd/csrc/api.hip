// C-ABI entry points of libbaklava (device part): context, split-K schedule, launches.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <new>
#include <numeric>
#include <vector>

#include "baklava.h"
#include "common.h"

using namespace baklava;

namespace {

thread_local int g_last_hip_error = 0;

inline bool hip_ok(hipError_t e) {
  if (e == hipSuccess) return true;
  g_last_hip_error = (int)e;
  return false;
}

constexpr int kMinChunk = 256;
constexpr int kSizingChunk = 256;  // the workspace is sized for chunks of at least this many rows
constexpr int kDefaultChunk = 512;        // launches over part of the model: shortest run (the item target lengthens it)
constexpr int kDefaultChunkWhole = 256;   // launches over the whole model: shortest run; longer ones come from the item target
constexpr int kWholeItemsPerCu = 5;       // whole-model launches aim at this many work items per compute unit
constexpr int kMaxChunk = 1 << 22; // row offsets inside a work item stay below 2^32 bytes
// Eviction: caches beyond this capacity are ranked by several workgroups.  One workgroup sweeps a cache
// five times out of the L2 and is bound by latency (about 80 us for 32768 rows); with thousands of
// caches in flight that latency is hidden and one workgroup per cache is the cheaper way up to about
// that size (measured on the 2048 llama32 caches: 175 us one workgroup each, 240 us with a threshold
// of 8192 rows), with a few caches (a prompt of one sequence: 8 caches of 32768 rows) it is not
// (82 us against 47 us tile by tile).
constexpr int kDefaultLongRows = 36864;
constexpr int kFewCaches = 512;  // below this many caches every cache beyond one tile is ranked tile by tile

inline size_t align256(size_t x) { return (x + 255) & ~size_t(255); }

int64_t count_items(const int32_t* cap, int64_t n_caches, int chunk) {
  int64_t n = 0;
  for (int64_t c = 0; c < n_caches; ++c) n += std::max<int64_t>(1, ((int64_t)cap[c] + chunk - 1) / chunk);
  return n;
}

struct WorkspacePlan {
  // index 0: schedule for launches over a layer sub-range, 1: for launches over the whole model
  size_t items[2], multi[2];
  size_t part_o, part_ml, final_ml, lag_q, lag_ml, lag_n, lag_cnt, status, kept, info, order_all, order_layer;
  size_t segs, seg_split, halo_k, halo_v, halo_score, halo_pos, tiles, tile_hist, sel_state, total;
  int64_t n_segs, halo_rows, n_tiles, n_long;
  int64_t max_items;
};

bool shape_ok(const baklava_desc* d) {
  if (!d) return false;
  if (d->L <= 0 || d->Hq <= 0 || d->Hkv <= 0 || d->batch <= 0) return false;
  if (d->D != 64 && d->D != 128) return false;
  if (d->dtype != BAKLAVA_BF16 && d->dtype != BAKLAVA_F32) return false;
  if (d->Hq % d->Hkv) return false;
  const int G = d->Hq / d->Hkv;
  if (G > 16 || (d->dtype == BAKLAVA_F32 && G > 8)) return false;
  if (d->dtype == BAKLAVA_BF16 && G > 8 && d->D != 128) return false;
  if (d->sink < 0 || d->recent < 0) return false;
  if (d->policy != BAKLAVA_POLICY_SCORE && d->policy != BAKLAVA_POLICY_STREAMING) return false;
  if ((int64_t)d->L * d->batch * d->Hkv > INT32_MAX) return false;
  return true;
}

// Segments of the eviction move: the destination range [0, budget) of every cache in runs of
// kMoveSegRows rows; a segment that has a successor owns a halo slot of cap - budget rows.
void count_segments(const baklava_desc* d, const int32_t* cap, const int32_t* budget, int64_t* n_segs,
                    int64_t* halo_rows) {
  const int64_t cpl = (int64_t)d->batch * d->Hkv;
  const int64_t n_caches = (int64_t)d->L * cpl;
  *n_segs = 0;
  *halo_rows = 0;
  for (int64_t c = 0; c < n_caches; ++c) {
    const int64_t b = budget[(c / cpl) * d->Hkv + c % d->Hkv];
    const int64_t ns = std::max<int64_t>(1, (b + kMoveSegRows - 1) / kMoveSegRows);
    *n_segs += ns;
    *halo_rows += (ns - 1) * std::max<int64_t>(0, cap[c] - b);
  }
}

WorkspacePlan plan_workspace(const baklava_desc* d, const int32_t* cap, const int32_t* budget) {
  WorkspacePlan w{};
  const int64_t n_caches = (int64_t)d->L * d->batch * d->Hkv;
  const int G = d->Hq / d->Hkv;
  const size_t row_bytes = (size_t)d->D * (d->dtype == BAKLAVA_BF16 ? 2 : 4);
  int64_t total_tokens = 0;
  for (int64_t c = 0; c < n_caches; ++c) total_tokens += cap[c];
  count_segments(d, cap, budget, &w.n_segs, &w.halo_rows);
  w.max_items = count_items(cap, n_caches, kSizingChunk);
  size_t o = 0;
  for (int k = 0; k < 2; ++k) {
    w.items[k] = o;   o = align256(o + (size_t)w.max_items * sizeof(Item));
    w.multi[k] = o;   o = align256(o + (size_t)n_caches * sizeof(MultiCache));
  }
  w.part_o = o;       o = align256(o + (size_t)w.max_items * G * d->D * 4);
  w.part_ml = o;      o = align256(o + (size_t)w.max_items * G * 2 * 4);
  w.final_ml = o;     o = align256(o + (size_t)n_caches * G * 2 * 4);
  // the record of the pending calls of every cache (score tracking): 32 packed query rows, their
  // (max, 1/sum), the rows each call saw, the count of pending calls per head
  const bool track = d->track_scores != 0;
  w.lag_q = o;        o = align256(o + (track ? (size_t)n_caches * kLagRows * row_bytes : 0));
  w.lag_ml = o;       o = align256(o + (track ? (size_t)n_caches * kLagRows * 2 * 4 : 0));
  w.lag_n = o;        o = align256(o + (size_t)n_caches * kLagCalls * 4);
  w.lag_cnt = o;      o = align256(o + (size_t)n_caches * G * 4);
  w.status = o;       o = align256(o + 256);
  w.kept = o;         o = align256(o + (size_t)total_tokens * 4);
  w.info = o;         o = align256(o + (size_t)n_caches * sizeof(CompactInfo));
  w.order_all = o;    o = align256(o + (size_t)n_caches * 4);
  w.order_layer = o;  o = align256(o + (size_t)n_caches * 4);
  w.segs = o;         o = align256(o + (size_t)w.n_segs * sizeof(MoveSeg));
  w.seg_split = o;    o = align256(o + (size_t)w.n_segs * 4);
  w.halo_k = o;       o = align256(o + (size_t)w.halo_rows * row_bytes);
  w.halo_v = o;       o = align256(o + (size_t)w.halo_rows * row_bytes);
  w.halo_score = o;   o = align256(o + (size_t)w.halo_rows * 4);
  w.halo_pos = o;     o = align256(o + (size_t)w.halo_rows * 4);
  // selection of the caches too long for one workgroup: tile table and per-tile digit counters
  w.n_tiles = 0;
  w.n_long = 0;
  for (int64_t c = 0; c < n_caches; ++c)
    if (cap[c] > kMinLongRows) {  // room for every threshold BAKLAVA_OPT_TILED_SELECT_ROWS may set
      w.n_tiles += ((int64_t)cap[c] + kTileRows - 1) / kTileRows;
      w.n_long += 1;
    }
  w.tiles = o;        o = align256(o + (size_t)w.n_tiles * sizeof(SelTile));
  w.tile_hist = o;    o = align256(o + (size_t)w.n_tiles * 4 * 256 * 4);
  w.sel_state = o;    o = align256(o + (size_t)w.n_long * 4 * sizeof(SelState));
  w.total = o;
  return w;
}

}  // namespace

struct baklava_ctx {
  baklava_desc d;
  int64_t n_caches;
  int32_t cpl;  // caches per layer
  int32_t G;
  int32_t row_bytes;
  std::vector<int64_t> off;
  std::vector<int32_t> cap, len, budget;
  std::vector<int32_t> order_all, order_layer;  // caches, longest first (whole model / inside each layer)
  std::vector<int32_t> seg_begin;               // cache -> first segment of the eviction move
  std::vector<int32_t> tile_begin;              // cache -> first tile of the tiled selection (long caches only have any)
  int32_t kernel_pref;
  bool layer_one_wave;   // default schedule of layer-range launches: one workgroup per compute unit
  int32_t target_items;  // > 0: layer-range launches lengthen their runs until a layer has at most this many items
  int32_t target_items_whole;  // > 0: the same for launches over the whole model
  int32_t n_cus;               // compute units of the device
  int32_t select_long_rows;    // caches with more capacity than this are ranked tile by tile at eviction
  int32_t lag_gp_log2;         // score tracking: log2 of G rounded up to 4, 8 or 16 (rows a call takes in a record)
  struct Schedule {
    int32_t chunk = 0;
    std::vector<int32_t> max_count;    // layer -> longest work item of the layer, rows
    std::vector<int32_t> cib;          // cache -> first item
    std::vector<int32_t> multi_begin;  // layer -> first entry of the list of multi-item caches
  } sched[2];                          // 0: layer sub-range launches, 1: whole-model launches
  WorkspacePlan plan;
  char* ws;
  int32_t time_kernel;         // 0 off, 1 events recorded around the attention kernel, 2 events carried by its dispatch
  bool track_on;               // score tracking in force (BAKLAVA_OPT_TRACK_SCORES pauses it)
  std::vector<hipEvent_t> ev;  // pairs (before, after); the first 2 * ev_used are recorded
  size_t ev_used;
};

namespace {

// Builds one of the two split-K schedules with the host planner and uploads it.  Schedule 0
// serves launches over a layer sub-range (launch order inside each layer, so a layer range is a
// contiguous slice), schedule 1 launches over the whole model.  The table depends on capacities
// only, so it is uploaded once; the kernels clamp each run to the live length.
int build_schedule(baklava_ctx* ctx, int which, int chunk) {
  int64_t n_items = 0;
  std::vector<baklava_work_item> items((size_t)ctx->plan.max_items);
  const int st = baklava_plan_schedule(ctx->off.data(), ctx->cap.data(), ctx->d.L, ctx->cpl, chunk,
                                       which == 0 ? ctx->target_items : ctx->target_items_whole, which,
                                       ctx->plan.max_items,
                                       items.data(), &n_items);
  if (st != BAKLAVA_OK) return st;
  static_assert(sizeof(baklava_work_item) == sizeof(Item), "work item layouts must match");
  // cache -> first partial slot, and the caches that need the combine kernel (in launch order)
  std::vector<int32_t> cib(ctx->n_caches + 1, 0), multi_begin(ctx->d.L + 1, 0);
  std::vector<MultiCache> multi;
  std::vector<int32_t> max_count(ctx->d.L, 0);
  for (int64_t i = 0; i < n_items; ++i) {
    const baklava_work_item& it = items[i];
    max_count[it.cache / ctx->cpl] = std::max(max_count[it.cache / ctx->cpl], it.count);
    if (it.start == 0) {
      cib[it.cache] = it.slot;
      if (it.nsplit > 1) {
        multi.push_back(MultiCache{it.cache, it.slot, it.slot + it.nsplit, 0});
        multi_begin[it.cache / ctx->cpl + 1] += 1;
      }
    }
  }
  cib[ctx->n_caches] = (int32_t)n_items;
  for (int32_t l = 0; l < ctx->d.L; ++l) multi_begin[l + 1] += multi_begin[l];
  if (!hip_ok(hipDeviceSynchronize())) return BAKLAVA_EHIP;  // no launch may still read the old table
  if (!hip_ok(hipMemcpy(ctx->ws + ctx->plan.items[which], items.data(), (size_t)n_items * sizeof(Item),
                        hipMemcpyHostToDevice)) ||
      (!multi.empty() &&
       !hip_ok(hipMemcpy(ctx->ws + ctx->plan.multi[which], multi.data(), multi.size() * sizeof(MultiCache), hipMemcpyHostToDevice))))
    return BAKLAVA_EHIP;
  ctx->sched[which].cib.swap(cib);
  ctx->sched[which].multi_begin.swap(multi_begin);
  ctx->sched[which].chunk = chunk;
  ctx->sched[which].max_count.swap(max_count);
  return BAKLAVA_OK;
}

// Tile table of the eviction's selection for long caches (depends on capacities and the threshold
// only), in cache order, so that the tiles of a layer range are a contiguous slice.
int build_tiles(baklava_ctx* ctx) {
  std::vector<SelTile> tiles;
  const int64_t n_caches = ctx->n_caches;
  std::vector<int32_t> tile_begin(n_caches + 1, 0);
  int32_t n_long = 0;
  for (int64_t c = 0; c < n_caches; ++c) {
    tile_begin[c] = (int32_t)tiles.size();
    if (ctx->cap[c] <= ctx->select_long_rows) continue;
    const int32_t nt = (int32_t)(((int64_t)ctx->cap[c] + kTileRows - 1) / kTileRows);
    const int32_t first = (int32_t)tiles.size();
    for (int32_t t = 0; t < nt; ++t) tiles.push_back(SelTile{(int32_t)c, t, first, nt, n_long, 0});
    n_long += 1;
  }
  tile_begin[n_caches] = (int32_t)tiles.size();
  if ((int64_t)tiles.size() > ctx->plan.n_tiles || n_long > ctx->plan.n_long) return BAKLAVA_ECAPACITY;
  if (!hip_ok(hipDeviceSynchronize())) return BAKLAVA_EHIP;  // no launch may still read the old table
  if (!tiles.empty() &&
      !hip_ok(hipMemcpy(ctx->ws + ctx->plan.tiles, tiles.data(), tiles.size() * sizeof(SelTile), hipMemcpyHostToDevice)))
    return BAKLAVA_EHIP;
  ctx->tile_begin.swap(tile_begin);
  return BAKLAVA_OK;
}

bool range_ok(const baklava_ctx* ctx, int32_t lb, int32_t lc) {
  return lb >= 0 && lc > 0 && (int64_t)lb + lc <= ctx->d.L;
}

// The weights of the calls on record go to the score plane now (see DecodeParams): a pass over the
// K rows of the layer range, after which the records are empty.  Only the MFMA attention kernel
// (bf16, D = 128) leaves calls on record.
int flush_records(baklava_ctx* ctx, int32_t layer_begin, int32_t layer_count, hipStream_t s) {
  if (!ctx->d.track_scores || !(ctx->d.dtype == BAKLAVA_BF16 && ctx->d.D == 128)) return BAKLAVA_OK;
  const int64_t c0 = (int64_t)layer_begin * ctx->cpl;
  const int64_t c1 = c0 + (int64_t)layer_count * ctx->cpl;
  const int which = (layer_begin == 0 && layer_count == ctx->d.L) ? 1 : 0;
  const baklava_ctx::Schedule& sc = ctx->sched[which];
  const int32_t i0 = sc.cib[c0], i1 = sc.cib[c1];
  DecodeParams p{};
  p.k = ctx->d.k; p.score = ctx->d.score;
  p.items = reinterpret_cast<const Item*>(ctx->ws + ctx->plan.items[which]) + i0;
  p.lag_q = ctx->ws + ctx->plan.lag_q;
  p.lag_ml = reinterpret_cast<float*>(ctx->ws + ctx->plan.lag_ml);
  p.lag_n = reinterpret_cast<int32_t*>(ctx->ws + ctx->plan.lag_n);
  p.lag_cnt = reinterpret_cast<int32_t*>(ctx->ws + ctx->plan.lag_cnt);
  p.G = ctx->G; p.lag_gp_log2 = ctx->lag_gp_log2;
  p.scale_log2e = (float)(1.4426950408889634 / std::sqrt((double)ctx->d.D));
  const int32_t longest = *std::max_element(sc.max_count.begin() + layer_begin,
                                            sc.max_count.begin() + layer_begin + layer_count);
  if (!hip_ok(launch_score_flush_mfma(p, i1 - i0, longest, s))) return BAKLAVA_EHIP;
  if (!hip_ok(launch_fill_i32(p.lag_cnt + c0 * ctx->G, 0, (c1 - c0) * ctx->G, s))) return BAKLAVA_EHIP;
  return BAKLAVA_OK;
}

// The vector-ALU path's score update for the call that has just been enqueued with query `q`.
int score_pass(baklava_ctx* ctx, int32_t layer_begin, int32_t layer_count, const void* q, hipStream_t s) {
  const int64_t c0 = (int64_t)layer_begin * ctx->cpl;
  const int64_t c1 = c0 + (int64_t)layer_count * ctx->cpl;
  const int which = (layer_begin == 0 && layer_count == ctx->d.L) ? 1 : 0;
  const baklava_ctx::Schedule& sc = ctx->sched[which];
  const int32_t i0 = sc.cib[c0], i1 = sc.cib[c1];
  ScoreParams p;
  p.k = ctx->d.k; p.q = q;
  p.ml = reinterpret_cast<const float*>(ctx->ws + ctx->plan.final_ml);
  p.len = ctx->d.len;
  p.items = reinterpret_cast<const Item*>(ctx->ws + ctx->plan.items[which]) + i0;
  p.score = ctx->d.score;
  p.G = ctx->G; p.Hq = ctx->d.Hq; p.Hkv = ctx->d.Hkv;
  p.cache_begin = (int32_t)c0;
  p.scale_log2e = (float)(1.4426950408889634 / std::sqrt((double)ctx->d.D));
  const int32_t longest = *std::max_element(sc.max_count.begin() + layer_begin,
                                            sc.max_count.begin() + layer_begin + layer_count);
  if (!hip_ok(launch_score_pass(p, ctx->d.dtype, ctx->d.D, i1 - i0, longest, s))) return BAKLAVA_EHIP;
  return BAKLAVA_OK;
}

// host_lengths: the host mirror of the lengths is checked and advanced (the calls that take the token
// position by value); otherwise the device tables alone decide and evolve.
int decode_impl(baklava_ctx* ctx, int32_t layer_begin, int32_t layer_count, const void* k_new,
                const void* v_new, int32_t token_pos, const int32_t* token_pos_dev, bool host_lengths,
                const void* q, float* out, void* stream) {
  const bool fused = k_new != nullptr;
  const int64_t c0 = (int64_t)layer_begin * ctx->cpl;
  const int64_t c1 = c0 + (int64_t)layer_count * ctx->cpl;
  if (host_lengths) {
    for (int64_t c = c0; c < c1; ++c) {
      if (fused && ctx->len[c] >= ctx->cap[c]) return BAKLAVA_ECAPACITY;
      if (!fused && ctx->len[c] <= 0) return BAKLAVA_ESTATE;
    }
  }
  const bool whole = layer_begin == 0 && layer_count == ctx->d.L;
  const int which = whole ? 1 : 0;
  const baklava_ctx::Schedule& sc = ctx->sched[which];
  const int32_t i0 = sc.cib[c0], i1 = sc.cib[c1];
  hipStream_t s = (hipStream_t)stream;
  const bool mfma_able = ctx->d.dtype == BAKLAVA_BF16 && ctx->d.D == 128;
  const bool use_mfma = ctx->kernel_pref == 2 || (ctx->kernel_pref == 0 && mfma_able);
  const bool track = ctx->track_on;
  // The vector-ALU kernel adds its weights right after the call; weights an earlier MFMA call left
  // pending come first, so that the scores grow in the order of the calls.
  if (track && !use_mfma) {
    const int st = flush_records(ctx, layer_begin, layer_count, s);
    if (st != BAKLAVA_OK) return st;
  }
  DecodeParams p;
  p.k = ctx->d.k; p.v = ctx->d.v; p.q = q; p.out = out;
  p.off = ctx->d.off; p.len = ctx->d.len;
  // Slots are numbered cache by cache and the launch order only permutes caches inside a layer
  // (schedule 0), so the launch-ordered table of a layer range is the slice [i0, i1).
  p.items = reinterpret_cast<const Item*>(ctx->ws + ctx->plan.items[which]) + i0;
  p.part_o = reinterpret_cast<float*>(ctx->ws + ctx->plan.part_o);
  p.part_ml = reinterpret_cast<float*>(ctx->ws + ctx->plan.part_ml);
  p.final_ml = reinterpret_cast<float*>(ctx->ws + ctx->plan.final_ml);
  p.lag_q = ctx->ws + ctx->plan.lag_q;
  p.lag_ml = reinterpret_cast<float*>(ctx->ws + ctx->plan.lag_ml);
  p.lag_n = reinterpret_cast<int32_t*>(ctx->ws + ctx->plan.lag_n);
  p.lag_cnt = reinterpret_cast<int32_t*>(ctx->ws + ctx->plan.lag_cnt);
  p.cap = ctx->d.cap;
  p.score = ctx->d.score;
  p.pos = ctx->d.pos;
  const int32_t m0 = sc.multi_begin[layer_begin], m1 = sc.multi_begin[layer_begin + layer_count];
  p.multi = reinterpret_cast<const MultiCache*>(ctx->ws + ctx->plan.multi[which]) + m0;
  p.k_new = k_new; p.v_new = v_new;
  p.token_pos_dev = token_pos_dev;
  p.status = reinterpret_cast<int32_t*>(ctx->ws + ctx->plan.status);
  p.G = ctx->G; p.Hq = ctx->d.Hq; p.Hkv = ctx->d.Hkv; p.batch = ctx->d.batch;
  p.cache_begin = (int32_t)c0;
  p.lag = (track && use_mfma) ? 1 : 0;
  p.lag_batch = kLagRows >> ctx->lag_gp_log2;
  p.lag_gp_log2 = ctx->lag_gp_log2;
  p.ring_slots = 0;
  p.fused_append = fused ? 1 : 0;
  p.token_pos = token_pos;
  p.row_bytes = ctx->row_bytes;
  p.scale_log2e = (float)(1.4426950408889634 / std::sqrt((double)ctx->d.D));
  hipEvent_t ev0 = nullptr, ev1 = nullptr;
  if (ctx->time_kernel) {
    while (ctx->ev.size() < 2 * (ctx->ev_used + 1)) {
      hipEvent_t e;
      if (!hip_ok(hipEventCreate(&e))) return BAKLAVA_EHIP;
      ctx->ev.push_back(e);
    }
    ev0 = ctx->ev[2 * ctx->ev_used];
    ev1 = ctx->ev[2 * ctx->ev_used + 1];
    if (!(ctx->time_kernel == 2 && use_mfma) && !hip_ok(hipEventRecord(ev0, s))) return BAKLAVA_EHIP;
  }
  const bool on_dispatch = ctx->time_kernel == 2 && use_mfma;
  const int32_t longest = *std::max_element(sc.max_count.begin() + layer_begin,
                                            sc.max_count.begin() + layer_begin + layer_count);
  hipError_t e = use_mfma ? launch_decode_mfma(p, i1 - i0, longest, i1 - i0 <= ctx->n_cus, s,
                                               on_dispatch ? ev0 : nullptr, on_dispatch ? ev1 : nullptr)
                          : launch_decode_valu(p, ctx->d.dtype, ctx->d.D, i1 - i0, s);
  if (!hip_ok(e)) return BAKLAVA_EHIP;
  if (ctx->time_kernel) {
    if (!on_dispatch && !hip_ok(hipEventRecord(ev1, s))) return BAKLAVA_EHIP;
    ctx->ev_used += 1;
  }
  if (!hip_ok(launch_combine(p, ctx->d.D, m1 - m0, s))) return BAKLAVA_EHIP;
  if (fused && host_lengths)
    for (int64_t c = c0; c < c1; ++c) ctx->len[c] += 1;
  if (track && !use_mfma) return score_pass(ctx, layer_begin, layer_count, q, s);
  return BAKLAVA_OK;
}

}  // namespace

void baklava::note_hip_error(hipError_t e) { g_last_hip_error = (int)e; }

extern "C" int baklava_last_hip_error(void) { return g_last_hip_error; }

extern "C" size_t baklava_workspace_bytes(const baklava_desc* desc, const int32_t* cap_host,
                                          const int32_t* budget_host) {
  if (!shape_ok(desc) || !cap_host || !budget_host) return 0;
  const int64_t n_caches = (int64_t)desc->L * desc->batch * desc->Hkv;
  for (int64_t c = 0; c < n_caches; ++c)
    if (cap_host[c] < 0) return 0;
  for (int64_t i = 0; i < (int64_t)desc->L * desc->Hkv; ++i)
    if (budget_host[i] < 0) return 0;
  return plan_workspace(desc, cap_host, budget_host).total;
}

extern "C" int baklava_create(const baklava_desc* desc, const int64_t* off_host, const int32_t* cap_host,
                              const int32_t* len_host, const int32_t* budget_host, baklava_ctx** out) {
  if (!out) return BAKLAVA_EINVAL;
  *out = nullptr;
  if (!shape_ok(desc) || !off_host || !cap_host || !budget_host) return BAKLAVA_EINVAL;
  if (!desc->k || !desc->v || !desc->score || !desc->pos || !desc->off || !desc->cap || !desc->len ||
      !desc->budget || !desc->workspace)
    return BAKLAVA_EINVAL;
  if (((uintptr_t)desc->k | (uintptr_t)desc->v) & 15) return BAKLAVA_EINVAL;
  if ((uintptr_t)desc->workspace & 255) return BAKLAVA_EINVAL;
  const int64_t n_caches = (int64_t)desc->L * desc->batch * desc->Hkv;
  const int64_t m = (int64_t)desc->L * desc->Hkv;
  for (int64_t i = 0; i < m; ++i) {
    if (budget_host[i] < 0) return BAKLAVA_EINVAL;
    const int need = desc->policy == BAKLAVA_POLICY_SCORE ? desc->sink + desc->recent : desc->sink;
    if (budget_host[i] < need) return BAKLAVA_EINFEASIBLE;
  }
  // The arena must be packed as baklava_layout lays it out (off[c] = capacities before c): the
  // workspace planes that run parallel to the arena (kept lists) are indexed by the same offsets.
  int64_t packed = 0;
  for (int64_t c = 0; c < n_caches; ++c) {
    if (cap_host[c] < 0 || off_host[c] != packed) return BAKLAVA_EINVAL;
    packed += cap_host[c];
    if (len_host && (len_host[c] < 0 || len_host[c] > cap_host[c])) return BAKLAVA_ECAPACITY;
  }
  baklava_ctx* ctx = new (std::nothrow) baklava_ctx();
  if (!ctx) return BAKLAVA_ENOMEM;
  ctx->d = *desc;
  ctx->n_caches = n_caches;
  ctx->cpl = desc->batch * desc->Hkv;
  ctx->G = desc->Hq / desc->Hkv;
  ctx->row_bytes = desc->D * (desc->dtype == BAKLAVA_BF16 ? 2 : 4);
  ctx->lag_gp_log2 = ctx->G <= 4 ? 2 : ctx->G <= 8 ? 3 : 4;
  ctx->off.assign(off_host, off_host + n_caches);
  ctx->cap.assign(cap_host, cap_host + n_caches);
  if (len_host) ctx->len.assign(len_host, len_host + n_caches);
  else ctx->len.assign(n_caches, 0);
  ctx->budget.assign(budget_host, budget_host + m);
  ctx->kernel_pref = 0;
  // A launch over part of the layers is one wave of workgroups: at most one per compute unit.
  {
    int dev = 0, cus = 0;
    if (!hip_ok(hipGetDevice(&dev)) ||
        !hip_ok(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev))) {
      delete ctx;
      return BAKLAVA_EHIP;
    }
    // One wave only pays while every cache can still be cut into about four work items; with more
    // caches per layer the runs differ too much in length and several waves of shorter items
    // balance better (measured on llama32-shaped layers: 64 caches per layer, one wave +6%;
    // 128 caches, five items per compute unit +4%; 256 caches, +48%).
    ctx->layer_one_wave = (int64_t)ctx->cpl * 4 <= cus;
    ctx->target_items = ctx->layer_one_wave ? cus : kWholeItemsPerCu * cus;
    ctx->n_cus = cus;
    // Whole-model launches: runs long enough to amortise the per-item costs, yet enough items for
    // the dispatcher to even out the load over several waves of workgroups.
    ctx->target_items_whole = kWholeItemsPerCu * cus;
  }
  ctx->time_kernel = 0;
  ctx->track_on = desc->track_scores != 0;
  ctx->ev_used = 0;
  ctx->plan = plan_workspace(desc, cap_host, budget_host);
  ctx->ws = reinterpret_cast<char*>(desc->workspace);
  if (desc->workspace_bytes < ctx->plan.total) { delete ctx; return BAKLAVA_ECAPACITY; }

  // Launch orders: longest caches first, over the whole model and within each layer.
  auto longer = [&](int32_t a, int32_t b) { return ctx->cap[a] > ctx->cap[b]; };
  ctx->order_all.resize(n_caches);
  std::iota(ctx->order_all.begin(), ctx->order_all.end(), 0);
  ctx->order_layer = ctx->order_all;
  std::stable_sort(ctx->order_all.begin(), ctx->order_all.end(), longer);
  for (int32_t l = 0; l < desc->L; ++l)
    std::stable_sort(ctx->order_layer.begin() + (int64_t)l * ctx->cpl,
                     ctx->order_layer.begin() + (int64_t)(l + 1) * ctx->cpl, longer);
  if (!hip_ok(hipMemcpy(ctx->ws + ctx->plan.order_all, ctx->order_all.data(), n_caches * 4, hipMemcpyHostToDevice)) ||
      !hip_ok(hipMemcpy(ctx->ws + ctx->plan.order_layer, ctx->order_layer.data(), n_caches * 4, hipMemcpyHostToDevice))) {
    delete ctx;
    return BAKLAVA_EHIP;
  }
  // No call is pending for the score pass, and the status word is clear.
  if (!hip_ok(hipMemset(ctx->ws + ctx->plan.lag_cnt, 0, (size_t)n_caches * ctx->G * 4)) ||
      !hip_ok(hipMemset(ctx->ws + ctx->plan.status, 0, 256))) {
    delete ctx;
    return BAKLAVA_EHIP;
  }
  // Segment table of the eviction move (depends on budgets and capacities only).
  {
    std::vector<MoveSeg> segs;
    segs.reserve((size_t)ctx->plan.n_segs);
    ctx->seg_begin.assign(n_caches + 1, 0);
    int64_t halo = 0;
    for (int64_t c = 0; c < n_caches; ++c) {
      ctx->seg_begin[c] = (int32_t)segs.size();
      const int64_t b = ctx->budget[(c / ctx->cpl) * desc->Hkv + c % desc->Hkv];
      const int64_t hs = std::max<int64_t>(0, ctx->cap[c] - b);
      const int64_t ns = std::max<int64_t>(1, (b + kMoveSegRows - 1) / kMoveSegRows);
      for (int64_t k = 0; k < ns; ++k) {
        MoveSeg sg;
        sg.c = (int32_t)c;
        sg.a = (int32_t)(k * kMoveSegRows);
        sg.halo_row = (k + 1 < ns && hs > 0) ? (int32_t)halo : -1;
        sg.pad = 0;
        if (k + 1 < ns) halo += hs;
        segs.push_back(sg);
      }
    }
    ctx->seg_begin[n_caches] = (int32_t)segs.size();
    if ((int64_t)segs.size() != ctx->plan.n_segs || halo != ctx->plan.halo_rows || halo > INT32_MAX ||
        !hip_ok(hipMemcpy(ctx->ws + ctx->plan.segs, segs.data(), segs.size() * sizeof(MoveSeg), hipMemcpyHostToDevice))) {
      delete ctx;
      return BAKLAVA_EHIP;
    }
  }
  ctx->select_long_rows = n_caches < kFewCaches ? kMinLongRows : kDefaultLongRows;
  {
    const int st = build_tiles(ctx);
    if (st != BAKLAVA_OK) { delete ctx; return st; }
  }
  if (!hip_ok(prepare_decode_mfma())) { delete ctx; return BAKLAVA_EHIP; }
  int st = build_schedule(ctx, 0, ctx->layer_one_wave ? kDefaultChunk : kDefaultChunkWhole);
  if (st == BAKLAVA_OK) st = build_schedule(ctx, 1, kDefaultChunkWhole);
  if (st != BAKLAVA_OK) { delete ctx; return st; }
  *out = ctx;
  return BAKLAVA_OK;
}

extern "C" int baklava_destroy(baklava_ctx* ctx) {
  if (!ctx) return BAKLAVA_EINVAL;
  for (hipEvent_t e : ctx->ev) (void)hipEventDestroy(e);
  delete ctx;
  return BAKLAVA_OK;
}

extern "C" int baklava_set_option(baklava_ctx* ctx, int32_t option, int64_t value) {
  if (!ctx) return BAKLAVA_EINVAL;
  switch (option) {
    case BAKLAVA_OPT_CHUNK_TOKENS:
    case BAKLAVA_OPT_CHUNK_TOKENS_WHOLE: {
      if (value < kMinChunk || value % 64 || value > kMaxChunk) return BAKLAVA_EINVAL;
      const int which = option == BAKLAVA_OPT_CHUNK_TOKENS ? 0 : 1;
      if ((int32_t)value == ctx->sched[which].chunk) return BAKLAVA_OK;
      return build_schedule(ctx, which, (int32_t)value);
    }
    case BAKLAVA_OPT_TARGET_ITEMS:
    case BAKLAVA_OPT_TARGET_ITEMS_WHOLE: {
      if (value < 0 || value > (1 << 20)) return BAKLAVA_EINVAL;
      const int which = option == BAKLAVA_OPT_TARGET_ITEMS ? 0 : 1;
      int32_t& target = which == 0 ? ctx->target_items : ctx->target_items_whole;
      if ((int32_t)value == target) return BAKLAVA_OK;
      target = (int32_t)value;
      return build_schedule(ctx, which, ctx->sched[which].chunk);
    }
    case BAKLAVA_OPT_KERNEL:
      if (value < 0 || value > 2) return BAKLAVA_EINVAL;
      if (value == 2 && !(ctx->d.dtype == BAKLAVA_BF16 && ctx->d.D == 128)) return BAKLAVA_EINVAL;
      if (value == 1 && ctx->G > 8) return BAKLAVA_EINVAL;
      ctx->kernel_pref = (int32_t)value;
      return BAKLAVA_OK;
    case BAKLAVA_OPT_TILED_SELECT_ROWS: {
      if (value < kMinLongRows || value > INT32_MAX) return BAKLAVA_EINVAL;
      if ((int32_t)value == ctx->select_long_rows) return BAKLAVA_OK;
      const int32_t old = ctx->select_long_rows;
      ctx->select_long_rows = (int32_t)value;
      const int st = build_tiles(ctx);
      if (st != BAKLAVA_OK) ctx->select_long_rows = old;
      return st;
    }
    case BAKLAVA_OPT_TRACK_SCORES:
      if (value != 0 && value != 1) return BAKLAVA_EINVAL;
      if (value == 1 && !ctx->d.track_scores) return BAKLAVA_EINVAL;  // the workspace holds no records
      ctx->track_on = value == 1;
      return BAKLAVA_OK;
    case BAKLAVA_OPT_TIME_KERNEL:
      if (value < 0 || value > 2) return BAKLAVA_EINVAL;
      if (ctx->ev_used && value != ctx->time_kernel) return BAKLAVA_ESTATE;  // read the pending record first
      ctx->time_kernel = (int32_t)value;
      return BAKLAVA_OK;
    default:
      return BAKLAVA_EINVAL;
  }
}

extern "C" int baklava_profile_read(baklava_ctx* ctx, double* total_ms_out, int64_t* launches_out) {
  if (!ctx || !total_ms_out || !launches_out) return BAKLAVA_EINVAL;
  double total = 0.0;
  for (size_t i = 0; i < ctx->ev_used; ++i) {
    if (!hip_ok(hipEventSynchronize(ctx->ev[2 * i + 1]))) return BAKLAVA_EHIP;
    float ms = 0.f;
    if (!hip_ok(hipEventElapsedTime(&ms, ctx->ev[2 * i], ctx->ev[2 * i + 1]))) return BAKLAVA_EHIP;
    total += ms;
  }
  *total_ms_out = total;
  *launches_out = (int64_t)ctx->ev_used;
  ctx->ev_used = 0;
  return BAKLAVA_OK;
}

extern "C" int baklava_reset(baklava_ctx* ctx, void* stream) {
  if (!ctx) return BAKLAVA_EINVAL;
  if (!hip_ok(launch_fill_i32(ctx->d.len, 0, ctx->n_caches, (hipStream_t)stream))) return BAKLAVA_EHIP;
  if (!hip_ok(launch_fill_i32(reinterpret_cast<int32_t*>(ctx->ws + ctx->plan.lag_cnt), 0, ctx->n_caches * ctx->G,
                              (hipStream_t)stream)))
    return BAKLAVA_EHIP;
  std::fill(ctx->len.begin(), ctx->len.end(), 0);
  return BAKLAVA_OK;
}

extern "C" int baklava_set_lengths(baklava_ctx* ctx, const int32_t* len_host, void* stream) {
  if (!ctx || !len_host) return BAKLAVA_EINVAL;
  for (int64_t c = 0; c < ctx->n_caches; ++c) {
    if (len_host[c] < 0) return BAKLAVA_EINVAL;
    if (len_host[c] > ctx->cap[c]) return BAKLAVA_ECAPACITY;
  }
  ctx->len.assign(len_host, len_host + ctx->n_caches);
  // Weights of a call over the old contents are not owed to the new ones.
  if (!hip_ok(launch_fill_i32(reinterpret_cast<int32_t*>(ctx->ws + ctx->plan.lag_cnt), 0, ctx->n_caches * ctx->G,
                              (hipStream_t)stream)))
    return BAKLAVA_EHIP;
  // The mirror is the staging buffer: wait for the copy so that later appends may change it.
  if (!hip_ok(hipMemcpyAsync(ctx->d.len, ctx->len.data(), ctx->n_caches * 4, hipMemcpyHostToDevice,
                             (hipStream_t)stream)))
    return BAKLAVA_EHIP;
  if (!hip_ok(hipStreamSynchronize((hipStream_t)stream))) return BAKLAVA_EHIP;
  return BAKLAVA_OK;
}

extern "C" int baklava_append(baklava_ctx* ctx, int32_t layer_begin, int32_t layer_count,
                              const void* k_new, const void* v_new, int32_t token_pos, void* stream) {
  if (!ctx || !k_new || !v_new || !range_ok(ctx, layer_begin, layer_count)) return BAKLAVA_EINVAL;
  if (((uintptr_t)k_new | (uintptr_t)v_new) & 15) return BAKLAVA_EINVAL;
  const int64_t c0 = (int64_t)layer_begin * ctx->cpl;
  const int64_t c1 = c0 + (int64_t)layer_count * ctx->cpl;
  for (int64_t c = c0; c < c1; ++c)
    if (ctx->len[c] >= ctx->cap[c]) return BAKLAVA_ECAPACITY;
  AppendParams p;
  p.k = ctx->d.k; p.v = ctx->d.v; p.score = ctx->d.score; p.pos = ctx->d.pos;
  p.off = ctx->d.off; p.cap = ctx->d.cap; p.len = ctx->d.len;
  p.k_new = k_new; p.v_new = v_new;
  p.token_pos_dev = nullptr;
  p.cache_begin = (int32_t)c0; p.token_pos = token_pos; p.row_bytes = ctx->row_bytes;
  if (!hip_ok(launch_append(p, (int)(c1 - c0), (hipStream_t)stream))) return BAKLAVA_EHIP;
  for (int64_t c = c0; c < c1; ++c) ctx->len[c] += 1;
  return BAKLAVA_OK;
}

extern "C" int baklava_decode_attn(baklava_ctx* ctx, int32_t layer_begin, int32_t layer_count,
                                   const void* q, float* out, void* stream) {
  if (!ctx || !q || !out || !range_ok(ctx, layer_begin, layer_count)) return BAKLAVA_EINVAL;
  if (((uintptr_t)q & 15) || ((uintptr_t)out & 15)) return BAKLAVA_EINVAL;
  return decode_impl(ctx, layer_begin, layer_count, nullptr, nullptr, 0, nullptr, true, q, out, stream);
}

extern "C" int baklava_append_decode_attn(baklava_ctx* ctx, int32_t layer_begin, int32_t layer_count,
                                          const void* k_new, const void* v_new, int32_t token_pos,
                                          const void* q, float* out, void* stream) {
  if (!ctx || !q || !out || !k_new || !v_new || !range_ok(ctx, layer_begin, layer_count)) return BAKLAVA_EINVAL;
  if (((uintptr_t)q | (uintptr_t)out | (uintptr_t)k_new | (uintptr_t)v_new) & 15) return BAKLAVA_EINVAL;
  return decode_impl(ctx, layer_begin, layer_count, k_new, v_new, token_pos, nullptr, true, q, out, stream);
}

extern "C" int baklava_append_decode_attn_replay(baklava_ctx* ctx, int32_t layer_begin, int32_t layer_count,
                                                 const void* k_new, const void* v_new,
                                                 const int32_t* token_pos_dev, const void* q, float* out,
                                                 void* stream) {
  if (!ctx || !q || !out || !k_new || !v_new || !token_pos_dev || !range_ok(ctx, layer_begin, layer_count))
    return BAKLAVA_EINVAL;
  if (((uintptr_t)q | (uintptr_t)out | (uintptr_t)k_new | (uintptr_t)v_new) & 15) return BAKLAVA_EINVAL;
  if ((uintptr_t)token_pos_dev & 3) return BAKLAVA_EINVAL;
  return decode_impl(ctx, layer_begin, layer_count, k_new, v_new, 0, token_pos_dev, false, q, out, stream);
}

extern "C" int baklava_sync_lengths(baklava_ctx* ctx, void* stream) {
  if (!ctx) return BAKLAVA_EINVAL;
  hipStream_t s = (hipStream_t)stream;
  int32_t status = 0;
  int32_t* status_dev = reinterpret_cast<int32_t*>(ctx->ws + ctx->plan.status);
  if (!hip_ok(hipMemcpyAsync(ctx->len.data(), ctx->d.len, ctx->n_caches * 4, hipMemcpyDeviceToHost, s)) ||
      !hip_ok(hipMemcpyAsync(&status, status_dev, 4, hipMemcpyDeviceToHost, s)) ||
      !hip_ok(hipStreamSynchronize(s)))
    return BAKLAVA_EHIP;
  if (status == 0) return BAKLAVA_OK;
  if (!hip_ok(launch_fill_i32(status_dev, 0, 1, s))) return BAKLAVA_EHIP;
  return BAKLAVA_ECAPACITY;
}

extern "C" int baklava_flush_scores(baklava_ctx* ctx, int32_t layer_begin, int32_t layer_count, void* stream) {
  if (!ctx || !range_ok(ctx, layer_begin, layer_count)) return BAKLAVA_EINVAL;
  return flush_records(ctx, layer_begin, layer_count, (hipStream_t)stream);
}

extern "C" int baklava_compact(baklava_ctx* ctx, int32_t layer_begin, int32_t layer_count,
                               int32_t* kept_idx_out, void* stream) {
  if (!ctx || !range_ok(ctx, layer_begin, layer_count)) return BAKLAVA_EINVAL;
  const int64_t c0 = (int64_t)layer_begin * ctx->cpl;
  const int64_t c1 = c0 + (int64_t)layer_count * ctx->cpl;
  CompactParams p;
  p.k = ctx->d.k; p.v = ctx->d.v; p.score = ctx->d.score; p.pos = ctx->d.pos;
  p.off = ctx->d.off; p.len = ctx->d.len; p.budget = ctx->d.budget;
  const bool whole = layer_begin == 0 && layer_count == ctx->d.L;
  p.order = whole ? reinterpret_cast<const int32_t*>(ctx->ws + ctx->plan.order_all)
                  : reinterpret_cast<const int32_t*>(ctx->ws + ctx->plan.order_layer) + c0;
  p.kept = kept_idx_out ? kept_idx_out : reinterpret_cast<int32_t*>(ctx->ws + ctx->plan.kept);
  p.info = reinterpret_cast<CompactInfo*>(ctx->ws + ctx->plan.info);
  p.Hkv = ctx->d.Hkv; p.batch = ctx->d.batch;
  p.sink = ctx->d.sink; p.recent = ctx->d.recent; p.policy = ctx->d.policy;
  p.row_bytes = ctx->row_bytes;
  p.write_identity = kept_idx_out ? 1 : 0;
  const int32_t s0 = ctx->seg_begin[c0], s1 = ctx->seg_begin[c1];
  p.segs = reinterpret_cast<const MoveSeg*>(ctx->ws + ctx->plan.segs) + s0;
  p.seg_split = reinterpret_cast<int32_t*>(ctx->ws + ctx->plan.seg_split);
  p.seg_base = s0;
  p.halo_k = ctx->ws + ctx->plan.halo_k;
  p.halo_v = ctx->ws + ctx->plan.halo_v;
  p.halo_score = reinterpret_cast<float*>(ctx->ws + ctx->plan.halo_score);
  p.halo_pos = reinterpret_cast<int32_t*>(ctx->ws + ctx->plan.halo_pos);
  hipStream_t s = (hipStream_t)stream;
  // The selection ranks rows by their scores: weights still owed to them are added first.
  {
    const int st = flush_records(ctx, layer_begin, layer_count, s);
    if (st != BAKLAVA_OK) return st;
  }
  p.cap = ctx->d.cap;
  const int32_t t0 = ctx->tile_begin[c0], t1 = ctx->tile_begin[c1];
  p.tiles = reinterpret_cast<const SelTile*>(ctx->ws + ctx->plan.tiles) + t0;
  p.tile_hist = reinterpret_cast<int32_t*>(ctx->ws + ctx->plan.tile_hist);
  p.sel_state = reinterpret_cast<SelState*>(ctx->ws + ctx->plan.sel_state);
  p.long_rows = ctx->select_long_rows;
  if (!hip_ok(launch_compact_select(p, (int)(c1 - c0), t1 - t0, s))) return BAKLAVA_EHIP;
  if (!hip_ok(launch_compact_move(p, s1 - s0, s))) return BAKLAVA_EHIP;
  for (int64_t c = c0; c < c1; ++c) {
    const int32_t b = ctx->budget[(c / ctx->cpl) * ctx->d.Hkv + c % ctx->d.Hkv];
    ctx->len[c] = std::min(ctx->len[c], b);
  }
  return BAKLAVA_OK;
}

extern "C" size_t baklava_profile_workspace_bytes(int32_t batch, int32_t Hq, int32_t T) {
  if (batch <= 0 || Hq <= 0 || T <= 0) return 0;
  const int64_t n_tiles = ((int64_t)T + 127) / 128;  // 128 tokens per workgroup
  return align256((size_t)batch * Hq * n_tiles * sizeof(float));
}

extern "C" int baklava_profile_similarity(const void* q, const void* k, const void* v, int32_t batch,
                                          int32_t Hq, int32_t Hkv, int32_t T, int32_t D, int32_t dtype,
                                          float* cos_out, float* sim_out, float* lse_out, void* workspace,
                                          size_t workspace_bytes, void* stream) {
  if (!q || !k || !v || !sim_out || !workspace) return BAKLAVA_EINVAL;
  if (batch <= 0 || Hq <= 0 || Hkv <= 0 || T <= 0 || Hq % Hkv) return BAKLAVA_EINVAL;
  if (D != 128 || dtype != BAKLAVA_BF16) return BAKLAVA_EINVAL;
  if (((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)workspace) & 15) return BAKLAVA_EINVAL;
  if (((uintptr_t)sim_out | (uintptr_t)cos_out | (uintptr_t)lse_out) & 3) return BAKLAVA_EINVAL;
  if ((int64_t)batch * Hq * (((int64_t)T + 127) / 128) > INT32_MAX) return BAKLAVA_EINVAL;
  if (workspace_bytes < baklava_profile_workspace_bytes(batch, Hq, T)) return BAKLAVA_ECAPACITY;
  if (!hip_ok(launch_profile_similarity(q, k, v, batch, Hq, Hkv, T, cos_out, sim_out, lse_out,
                                        reinterpret_cast<float*>(workspace), (hipStream_t)stream)))
    return BAKLAVA_EHIP;
  return BAKLAVA_OK;
}

extern "C" size_t baklava_layer_workspace_bytes(int32_t n_seq, int32_t T) {
  if (n_seq <= 0 || T <= 0) return 0;
  return align256((size_t)n_seq * (((size_t)T + 15) / 16) * sizeof(float));  // 16 rows per workgroup
}

extern "C" int baklava_layer_similarity(const void* x_in, const void* x_out, int32_t n_seq, int32_t T,
                                        int32_t hidden, int32_t dtype, float* cos_out, float* sim_out,
                                        void* workspace, size_t workspace_bytes, void* stream) {
  if (!x_in || !x_out || !sim_out || !workspace) return BAKLAVA_EINVAL;
  if (n_seq <= 0 || T <= 0 || hidden <= 0 || hidden % 8 || dtype != BAKLAVA_BF16) return BAKLAVA_EINVAL;
  if (((uintptr_t)x_in | (uintptr_t)x_out | (uintptr_t)workspace) & 15) return BAKLAVA_EINVAL;
  if (((uintptr_t)sim_out | (uintptr_t)cos_out) & 3) return BAKLAVA_EINVAL;
  if ((int64_t)n_seq * (((int64_t)T + 15) / 16) > INT32_MAX) return BAKLAVA_EINVAL;
  if (workspace_bytes < baklava_layer_workspace_bytes(n_seq, T)) return BAKLAVA_ECAPACITY;
  if (!hip_ok(launch_layer_similarity(x_in, x_out, n_seq, T, hidden, cos_out, sim_out,
                                      reinterpret_cast<float*>(workspace), (hipStream_t)stream)))
    return BAKLAVA_EHIP;
  return BAKLAVA_OK;
}

extern "C" int baklava_prefill_scores(const void* q, const void* k, const float* lse, const int64_t* row_off,
                                      int32_t batch, int32_t Hq, int32_t Hkv, int32_t T, int32_t D,
                                      int32_t dtype, float* score_out, void* stream) {
  if (!q || !k || !lse || !score_out) return BAKLAVA_EINVAL;
  if (batch <= 0 || Hq <= 0 || Hkv <= 0 || T <= 0 || Hq % Hkv) return BAKLAVA_EINVAL;
  if (D != 128 || dtype != BAKLAVA_BF16) return BAKLAVA_EINVAL;
  if (((uintptr_t)q | (uintptr_t)k) & 15) return BAKLAVA_EINVAL;
  if (((uintptr_t)lse | (uintptr_t)score_out) & 3 || ((uintptr_t)row_off & 7)) return BAKLAVA_EINVAL;
  if ((int64_t)batch * Hkv * (((int64_t)T + 127) / 128) > INT32_MAX) return BAKLAVA_EINVAL;
  if (!hip_ok(launch_prefill_scores(q, k, lse, row_off, batch, Hq, Hkv, T, score_out, (hipStream_t)stream)))
    return BAKLAVA_EHIP;
  return BAKLAVA_OK;
}

extern "C" int baklava_lengths(baklava_ctx* ctx, int32_t* len_host_out) {
  if (!ctx || !len_host_out) return BAKLAVA_EINVAL;
  std::memcpy(len_host_out, ctx->len.data(), ctx->n_caches * sizeof(int32_t));
  return BAKLAVA_OK;
}

extern "C" int baklava_stream_probe(void* dst, const void* src, int64_t bytes, int32_t mode, void* stream) {
  if (!dst || !src || bytes <= 0 || (bytes & 15) || (mode < 0 || mode > 3)) return BAKLAVA_EINVAL;
  if (((uintptr_t)dst | (uintptr_t)src) & 15) return BAKLAVA_EINVAL;
  if (!hip_ok(launch_stream_probe(dst, src, bytes, mode, (hipStream_t)stream))) return BAKLAVA_EHIP;
  return BAKLAVA_OK;
}
