// Internal declarations shared by the library's own translation units.
#ifndef BAKLAVA_COMMON_H
#define BAKLAVA_COMMON_H

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace baklava {

// 16-byte load with the non-temporal hint, for data a kernel reads exactly once.
#ifdef __HIPCC__
typedef uint32_t nt_u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load_nt16(const void* ptr) {
  const nt_u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const nt_u32x4_t*>(ptr));
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void store_nt16(void* ptr, uint4 v) {
  const nt_u32x4_t x = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(x, reinterpret_cast<nt_u32x4_t*>(ptr));
}
#endif

constexpr int kLagRows = 32;   // packed query rows of a cache's record of pending calls (score tracking)
constexpr int kLagCalls = 8;   // most calls such a record holds
constexpr int kMoveSegRows = 4096;  // destination rows per workgroup of the eviction move
constexpr int kTileRows = 8192;     // rows per tile of a cache that is ranked tile by tile (one workgroup per tile and pass)
constexpr int kMinLongRows = kTileRows;  // smallest capacity from which a cache may be ranked that way

// One split-K work item (same layout as baklava_work_item of the public header): rows
// [start, start + count) of cache c; its partial result goes to partial slot `slot`.  Rows at or
// beyond the cache's live length are skipped by the kernel.
struct Item {
  int32_t c, start, count, slot;
  int32_t nsplit;  // work items of this cache
  int32_t pad;
  int64_t row0;    // arena row of `start`: off[c] + start
};

// Result of the selection pass for one cache.
struct CompactInfo {
  int32_t new_len;      // rows that survive
  int32_t first_moved;  // smallest evicted row index (== old length when nothing is evicted)
  int32_t old_len;
  int32_t pad;
};

// One tile of a cache that is too long for one workgroup's selection.
struct SelTile {
  int32_t c, tile;
  int32_t first_tile;  // index of the cache's tile 0 in the tile table
  int32_t n_tiles;     // tiles of the cache
  int32_t long_idx;    // index of the cache among the caches that are ranked this way
  int32_t pad;
};

// State of the radix select of a long cache after a pass.
struct SelState {
  uint32_t prefix;   // digits found so far, in place
  int32_t need;      // rank of the wanted key among the keys that match the prefix
  int32_t digit[4];
};

// A cache that the combine kernel serves, with its partial slots [slot_begin, slot_end): one
// 16-byte record, so that the kernel needs a single load before it can fetch the partials.
struct MultiCache {
  int32_t c, slot_begin, slot_end, pad;
};

struct DecodeParams {
  void* k;
  void* v;
  const void* q;
  float* out;
  const int64_t* off;
  int32_t* len;
  const Item* items;               // work items of the launched range, in launch order
  float* part_o;                   // [n_items, G, D] un-normalised partial outputs
  float* part_ml;                  // [n_items, G, 2]  (running max in log2 units, sum)
  float* final_ml;                 // [n_caches, G, 2] (global max, 1 / global sum) of the latest call
  // Score tracking, MFMA kernel: the weights of a call are added to the score plane by a later
  // call over the same caches (or by the score pass that baklava_flush_scores launches), because
  // only then are the softmax normalisers known to every work item.  Each cache keeps a record of
  // up to lag_batch pending calls; their query rows are packed into two 16-row operands (call s,
  // head g -> packed row s * Gp + g, Gp = G rounded up to 4, 8 or 16), so that two extra matrix
  // products per slab serve all of them.  A call that finds lag_batch calls pending adds their
  // weights and starts the record again with itself.
  void* lag_q;                     // [n_caches, kLagRows, D] packed query rows of the pending calls
  float* lag_ml;                   // [n_caches, kLagRows, 2] their (max, 1 / sum), same row numbering
  int32_t* lag_n;                  // [n_caches, kLagCalls] rows that were live at pending call s
  int32_t* lag_cnt;                // [n_caches, G] pending calls (one counter per head, all equal:
                                   // each block of the combine kernel reads and writes its own)
  const int32_t* cap;
  float* score;
  int32_t* pos;
  const MultiCache* multi;         // caches of the launched range that have more than one work item
  const void* k_new;               // fused append: [caches of the range, D] rows to add first
  const void* v_new;
  const int32_t* token_pos_dev;    // fused append: the new row's position, read on the device (or null)
  int32_t* status;                 // device status word: bit 0 = a fused append found its cache full
  int32_t G, Hq, Hkv, batch;
  int32_t cache_begin;             // first cache id of the launched range
  int32_t lag;                     // 1: record this call, apply the pending ones when due (MFMA kernel)
  int32_t lag_batch;               // calls a record holds: kLagRows / Gp
  int32_t lag_gp_log2;             // log2(Gp)
  int32_t ring_slots;              // MFMA kernel, lag: slabs per wavefront whose new scores wait in LDS
  int32_t fused_append;            // 1: every cache of the range first receives its new row
  int32_t token_pos;
  int32_t row_bytes;
  float scale_log2e;               // log2(e) / sqrt(D)
};

// Score pass of the vector-ALU path over the K rows alone, right after its attention call:
// score_j += sum_g 2^(q_g . k_j scale - M_g) / L_g over the live rows of every cache of the range.
struct ScoreParams {
  const void* k;
  const void* q;                   // [layer_count, batch, Hq, D], the call's query rows
  const float* ml;                 // final_ml of the call
  const int32_t* len;
  const Item* items;
  float* score;
  int32_t G, Hq, Hkv;
  int32_t cache_begin;
  float scale_log2e;
};

struct AppendParams {
  void* k;
  void* v;
  float* score;
  int32_t* pos;
  const int64_t* off;
  const int32_t* cap;
  int32_t* len;
  const void* k_new;
  const void* v_new;
  const int32_t* token_pos_dev;  // the row's position, read on the device (or null: token_pos)
  int32_t cache_begin;
  int32_t token_pos;
  int32_t row_bytes;
};

// One destination segment of the eviction move: rows [a, a + seg_rows) of cache c.  Segments that
// have a successor own a halo slot (room for cap - budget rows) in the workspace.
struct MoveSeg {
  int32_t c, a;
  int32_t halo_row;  // first row of this segment's halo slot, or -1
  int32_t pad;
};

struct CompactParams {
  void* k;
  void* v;
  float* score;
  int32_t* pos;
  const int64_t* off;
  int32_t* len;
  const int32_t* budget;
  const int32_t* order;  // launch order: blockIdx.x -> cache id
  int32_t* kept;         // [total_tokens], packed by off
  CompactInfo* info;     // [n_caches]
  int32_t Hkv, batch;
  int32_t sink, recent, policy;
  int32_t row_bytes;
  int32_t write_identity;  // 1: also write 0..n-1 for caches that evict nothing
  const MoveSeg* segs;     // segments of the launched cache range
  int32_t* seg_split;      // [n_segs] first destination row of a segment whose source lies past its end
  void* halo_k;            // halo copies of the rows a segment needs from beyond its end
  void* halo_v;
  float* halo_score;
  int32_t* halo_pos;
  int32_t seg_base;        // index of segs[0] in seg_split
  const int32_t* cap;
  const SelTile* tiles;    // tiles of the long caches of the launched range
  int32_t* tile_hist;      // [all tiles][4 passes][256] digit counters, indexed by first_tile + tile
  SelState* sel_state;     // [long caches][4] state after pass 0..3
  int32_t long_rows;       // caches with more capacity than this are ranked tile by tile
};

// Records a failed HIP call for baklava_last_hip_error() (per host thread).
void note_hip_error(hipError_t e);

// Launchers (defined next to their kernels).  All return hipError_t of the launch.
hipError_t launch_decode_valu(const DecodeParams& p, int dtype, int D, int n_items, hipStream_t s);
// max_count: longest work item of the launch (rows); one_wave: the launch has at most one workgroup per
// compute unit, so a workgroup may take the whole LDS (score tracking keeps its new scores there)
hipError_t launch_decode_mfma(const DecodeParams& p, int n_items, int max_count, bool one_wave, hipStream_t s,
                              hipEvent_t ev0 = nullptr, hipEvent_t ev1 = nullptr);
hipError_t prepare_decode_mfma();
// the weights of the calls on record, from the K rows alone (bf16, D = 128; needs only the lag_*,
// k, score, items, G and scale fields)
hipError_t launch_score_flush_mfma(const DecodeParams& p, int n_items, int max_count, hipStream_t s);
hipError_t launch_profile_similarity(const void* q, const void* k, const void* v, int batch, int Hq, int Hkv,
                                     int T, float* cos_out, float* sim_out, float* lse_out, float* tile_sum,
                                     hipStream_t s);
hipError_t launch_layer_similarity(const void* x_in, const void* x_out, int n_seq, int T, int hidden,
                                   float* cos_out, float* sim_out, float* tile_sum, hipStream_t s);
hipError_t launch_prefill_scores(const void* q, const void* k, const float* lse, const int64_t* row_off,
                                 int batch, int Hq, int Hkv, int T, float* score, hipStream_t s);
hipError_t launch_combine(const DecodeParams& p, int D, int n_multi, hipStream_t s);
// max_count: the largest row count of a work item in the launched range (or a bound on it)
hipError_t launch_score_pass(const ScoreParams& p, int dtype, int D, int n_items, int max_count, hipStream_t s);
hipError_t launch_append(const AppendParams& p, int n_caches, hipStream_t s);
hipError_t launch_fill_i32(int32_t* dst, int32_t value, int64_t n, hipStream_t s);
hipError_t launch_compact_select(const CompactParams& p, int n_caches, int n_tiles, hipStream_t s);
hipError_t launch_compact_move(const CompactParams& p, int n_segs, hipStream_t s);
hipError_t launch_stream_probe(void* dst, const void* src, int64_t bytes, int mode, hipStream_t s);

}  // namespace baklava
#endif
