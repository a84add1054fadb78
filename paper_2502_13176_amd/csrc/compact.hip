// Budget-enforcing eviction (f_evict, Eqs. 5-6): selection of the surviving rows (one workgroup
// per cache, long caches first; caches beyond what one workgroup sweeps quickly are cut into tiles
// and go through one kernel per radix pass), then a stable in-place move (one workgroup per segment).
#include "common.h"

namespace baklava {

namespace {

constexpr int kSelThreads = 512;
constexpr int kSelWaves = kSelThreads / 64;
constexpr int kSelUnroll = 8;  // score loads in flight per thread in the counting passes
constexpr int kSelRows = 16;   // consecutive rows per thread in the emit pass (four 16-byte loads)
constexpr int kEmitTile = kSelThreads * kSelRows;

// Order-preserving map from fp32 to uint32 (larger float -> larger key); -0 is folded onto +0 so
// that it ties with it, as a floating-point comparison would.
__device__ __forceinline__ uint32_t score_key(float f) {
  const uint32_t u = __float_as_uint(f + 0.0f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Exclusive prefix sum of `v` over the workgroup; `total` receives the sum.  `sm` holds one
// word per wavefront.  Ends with a barrier, so `sm` can be reused right away.
__device__ __forceinline__ int block_exclusive_scan(int v, int* sm, int& total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int incl = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int t = __shfl_up(incl, o);
    if (lane >= o) incl += t;
  }
  if (lane == 63) sm[wave] = incl;
  __syncthreads();
  int base = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < kSelWaves; ++w) {
    const int x = sm[w];
    if (w < wave) base += x;
    tot += x;
  }
  __syncthreads();
  total = tot;
  return base + incl - v;
}

// What the selection of one cache is after: the middle rows [mid_lo, mid_hi) compete for k places.
struct SelGoal {
  int n, b, k, mid_lo, mid_hi;
};

__device__ __forceinline__ SelGoal sel_goal(const CompactParams& p, int c) {
  SelGoal g;
  g.n = p.len[c];
  const int cpl = p.batch * p.Hkv;
  g.b = p.budget[(c / cpl) * p.Hkv + c % p.Hkv];
  const int s = p.sink;
  const int r = (p.policy == 1) ? (g.b - s) : p.recent;
  g.k = g.b - s - r;  // middle rows that survive, >= 0 (checked at context creation)
  g.mid_lo = s;
  g.mid_hi = g.n - r;
  return g;
}

// One counting pass of the radix select over rows [j_begin, j_end) of the middle: keys whose digits
// above `shift` equal `prefix` are counted by their digit at `shift` into the LDS histogram.
// A thread adds up runs of equal digits among its own keys before it touches the histogram: in
// the first pass most scores share their leading bits, and one atomic per key on the same few
// counters would serialise the whole workgroup.
template <int UNROLL>
__device__ __forceinline__ void count_digits(const float* score, int j_begin, int j_end, uint32_t prefix,
                                             uint32_t mask, int shift, int* hist) {
  const int tid = threadIdx.x;
  for (int j0 = j_begin + tid; j0 < j_end; j0 += kSelThreads * UNROLL) {
    uint32_t key[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      const int j = j0 + u * kSelThreads;
      key[u] = score_key(j < j_end ? score[j] : 0.f);
    }
    int run_digit = -1, run = 0;
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      const int j = j0 + u * kSelThreads;
      const bool live = j < j_end && (key[u] & mask) == prefix;
      const int digit = (key[u] >> shift) & 255;
      if (live && digit == run_digit) {
        run += 1;
      } else if (live) {
        if (run) atomicAdd(&hist[run_digit], run);
        run_digit = digit;
        run = 1;
      }
    }
    if (run) atomicAdd(&hist[run_digit], run);
  }
}

// The digit of the need-th largest key given the 256 counters of a pass: thread t looks at digit
// 255 - t; `above` = keys with a larger digit.  Exactly one digit has above < need <= above + its own
// count.  Results through the shared words; ends with a barrier.
__device__ __forceinline__ void find_digit(const int* hist, int need, int* sm_scan, int* sh_digit, int* sh_need) {
  const int tid = threadIdx.x;
  const int mine = tid < 256 ? hist[255 - tid] : 0;
  int all;
  const int above = block_exclusive_scan(mine, sm_scan, all);
  if (tid < 256 && above < need && above + mine >= need) {
    *sh_digit = 255 - tid;
    *sh_need = need - above;
  }
  __syncthreads();
}

// LDS an emit needs: the keys of a tile, padded by one word per 16 so that a thread's 16 consecutive
// keys and its neighbours' fall into different banks; once every thread has read its keys (the
// workgroup scan in between has barriers) the same words collect the tile's part of the kept list.
constexpr int kEmitKeyWords = kEmitTile + kEmitTile / 16;

// Stable emit of the rows [j_begin, j_end) of a cache.  A row survives if it is a sink or recent
// row, if its key exceeds the threshold, or if it is among the first need_eq rows (of the whole
// cache) whose key equals it; its place in the list is the number of survivors before it, i.e.
// (rows of the first two kinds before it) + min(rows with an equal key before it, need_eq).  Both
// counts come from one workgroup scan of a packed pair per tile of kEmitTile rows (at most
// kSelRows * kSelThreads = 2^13 each).  sure_base / eq_base: the two counts over the rows before
// j_begin.  Global memory is touched in whole lines only: the tile's scores are loaded row t,
// t + 512, ... per thread (all loads in flight at once) and handed to the thread that owns 16
// consecutive rows through LDS; the tile's survivors, which occupy consecutive places of the list,
// are collected in LDS and written out together.  The smallest evicted row index of the range goes
// to *sh_first (shared, initialised by the caller to the cache's length).
__device__ __forceinline__ void emit_rows(const float* score, int32_t* kept, const SelGoal& g, uint32_t thr,
                                          int need_eq, int j_begin, int j_end, int sure_base, int eq_base,
                                          int* sm_scan, int* sh_first, uint32_t* lds_key) {
  const int tid = threadIdx.x;
  const int n = g.n;
  int32_t* lds_out = reinterpret_cast<int32_t*>(lds_key);
  for (int j0 = j_begin; j0 < j_end; j0 += kEmitTile) {
    const int live = j_end - j0;  // rows of this tile (a short cache fills only the front of it)
    if (g.k > 0) {
      float sc[kSelRows];
#pragma unroll
      for (int u = 0; u < kSelRows; ++u) {
        const int j = j0 + tid + u * kSelThreads;
        sc[u] = 0.f;
        if (u * kSelThreads < live) sc[u] = (j >= g.mid_lo && j < g.mid_hi && j < j_end) ? score[j] : 0.f;
      }
#pragma unroll
      for (int u = 0; u < kSelRows; ++u) {
        const int r = tid + u * kSelThreads;
        if (u * kSelThreads < live) lds_key[r + (r >> 4)] = score_key(sc[u]);
      }
      __syncthreads();
    }
    const int jt = j0 + tid * kSelRows;
    bool sure[kSelRows], eq[kSelRows];
    int n_sure = 0, n_eq = 0;
#pragma unroll
    for (int i = 0; i < kSelRows; ++i) {
      const int j = jt + i;
      const bool in = j < j_end;
      const bool middle = in && j >= g.mid_lo && j < g.mid_hi;
      const uint32_t key = (middle && g.k > 0) ? lds_key[tid * (kSelRows + 1) + i] : 0u;
      sure[i] = (in && !middle) || (middle && g.k > 0 && key > thr);
      eq[i] = middle && g.k > 0 && key == thr;
      n_sure += sure[i] ? 1 : 0;
      n_eq += eq[i] ? 1 : 0;
    }
    int total;
    const int excl = block_exclusive_scan(n_sure | (n_eq << 16), sm_scan, total);
    const int place0 = sure_base + min(eq_base, need_eq);  // place of the tile's first survivor
    int sure_before = sure_base + (excl & 0xffff);
    int eq_before = eq_base + ((uint32_t)excl >> 16);
    int first_out = n;
#pragma unroll
    for (int i = 0; i < kSelRows; ++i) {
      const int j = jt + i;
      const bool keep = sure[i] || (eq[i] && eq_before < need_eq);
      if (keep) lds_out[sure_before + min(eq_before, need_eq) - place0] = j;
      else if (j < j_end) first_out = min(first_out, j);
      sure_before += sure[i] ? 1 : 0;
      eq_before += eq[i] ? 1 : 0;
    }
    // rows leave in ascending order of the tiles, so only the first tile that evicts has to report
    if (first_out < n && first_out < *(volatile int*)sh_first) atomicMin(sh_first, first_out);
    sure_base += total & 0xffff;
    eq_base += (uint32_t)total >> 16;
    const int survivors = sure_base + min(eq_base, need_eq) - place0;
    __syncthreads();
    for (int i = tid; i < survivors; i += kSelThreads) kept[place0 + i] = lds_out[i];
    __syncthreads();  // the LDS areas are free again
  }
}

// Selection for the caches one workgroup sweeps alone (capacity up to p.long_rows), long caches
// first; longer caches are left to the tile kernels below.
__global__ __launch_bounds__(kSelThreads) void compact_select_kernel(CompactParams p) {
  const int c = p.order[blockIdx.x];
  if (p.cap[c] > p.long_rows) return;
  const int tid = threadIdx.x;
  const SelGoal g = sel_goal(p, c);
  const int n = g.n;
  const int64_t off = p.off[c];
  int32_t* kept = p.kept + off;
  const float* score = p.score + off;

  if (n <= g.b) {
    if (p.write_identity)
      for (int j = tid; j < n; j += kSelThreads) kept[j] = j;
    if (tid == 0) p.info[c] = CompactInfo{n, n, n, 0};
    return;
  }

  __shared__ int hist[256];
  __shared__ int sm_scan[kSelWaves];
  __shared__ int sh_digit, sh_need, sh_first;
  __shared__ uint32_t lds_key[kEmitKeyWords];

  uint32_t thr = 0;
  int need_eq = 0;
  if (g.k > 0) {
    // Radix select of the k-th largest key of the middle, 8 bits per pass, high digits first.
    uint32_t prefix = 0, mask = 0;
    int need = g.k;
    for (int shift = 24; shift >= 0; shift -= 8) {
      for (int i = tid; i < 256; i += kSelThreads) hist[i] = 0;
      __syncthreads();
      count_digits<kSelUnroll>(score, g.mid_lo, g.mid_hi, prefix, mask, shift, hist);
      __syncthreads();
      find_digit(hist, need, sm_scan, &sh_digit, &sh_need);
      prefix |= (uint32_t)sh_digit << shift;
      need = sh_need;
      mask |= 0xffu << shift;
      __syncthreads();
    }
    thr = prefix;
    need_eq = need;  // rows whose key equals thr that still survive (oldest first)
  }

  if (tid == 0) sh_first = n;
  __syncthreads();
  emit_rows(score, kept, g, thr, need_eq, 0, n, 0, 0, sm_scan, &sh_first, lds_key);
  __syncthreads();
  if (tid == 0) p.info[c] = CompactInfo{g.b, sh_first, n, 0};
}

// ---- caches too long for one workgroup -------------------------------------------------------
// A long cache is cut into tiles of kTileRows rows (over its capacity), one workgroup per tile and
// pass.  Pass P (one kernel each, P = 0..3) leaves the 256 counters of every tile in the workspace;
// the counters of a cache are the sums over its tiles, which every workgroup of the next kernel forms
// for itself (a few thousand additions) before it searches the digit: no atomics between workgroups,
// no counters to clear, no waiting on another workgroup, and one kernel per pass.  The last kernel
// knows the threshold, derives from the stored counters how many survivors the tiles before its own
// hold, and emits its tile.

// State of a long cache's selection after pass P - 1, formed by every workgroup of the kernel that
// follows that pass: the state after pass P - 2 (stored by that kernel's predecessor) advanced by
// the digit search on the summed tile counters of pass P - 1.  Tile 0's workgroup stores it for the
// next kernel.  Ends with a barrier; `hist` is free again.
template <int P>
__device__ __forceinline__ SelState state_before_pass(const CompactParams& p, const SelTile& tl, int k, int* hist,
                                                      int* sm_scan, int* sh_digit, int* sh_need) {
  SelState st = SelState{0u, k, {0, 0, 0, 0}};
  if (P == 0) return st;
  if (P >= 2) st = p.sel_state[(int64_t)tl.long_idx * 4 + (P - 2)];
  const int tid = threadIdx.x;
  if (tid < 256) {
    int sum = 0;
    for (int j = 0; j < tl.n_tiles; ++j) sum += p.tile_hist[((int64_t)(tl.first_tile + j) * 4 + (P - 1)) * 256 + tid];
    hist[tid] = sum;
  }
  __syncthreads();
  find_digit(hist, st.need, sm_scan, sh_digit, sh_need);
  st.prefix |= (uint32_t)*sh_digit << (24 - 8 * (P - 1));
  st.need = *sh_need;
  st.digit[P - 1] = *sh_digit;
  __syncthreads();
  if (tl.tile == 0 && tid == 0) p.sel_state[(int64_t)tl.long_idx * 4 + (P - 1)] = st;
  return st;
}

template <int PASS>
__global__ __launch_bounds__(kSelThreads) void compact_tile_count_kernel(CompactParams p) {
  const SelTile tl = p.tiles[blockIdx.x];
  const int c = tl.c;
  const int tid = threadIdx.x;
  const SelGoal g = sel_goal(p, c);
  if (PASS == 0 && tl.tile == 0 && tid == 0) {
    // the selection's result record; the emit kernel lowers first_moved with atomicMin
    p.info[c] = g.n <= g.b ? CompactInfo{g.n, g.n, g.n, 0} : CompactInfo{g.b, g.n, g.n, 0};
  }
  if (g.n <= g.b || g.k <= 0) return;  // nothing to rank (uniform over the cache's workgroups)
  __shared__ int hist[256];
  __shared__ int sm_scan[kSelWaves];
  __shared__ int sh_digit, sh_need;
  const SelState st = state_before_pass<PASS>(p, tl, g.k, hist, sm_scan, &sh_digit, &sh_need);
  for (int i = tid; i < 256; i += kSelThreads) hist[i] = 0;
  __syncthreads();
  const int shift = 24 - 8 * PASS;
  const uint32_t mask = PASS == 0 ? 0u : (0xffffffffu << (shift + 8));
  const int j_begin = max(g.mid_lo, tl.tile * kTileRows), j_end = min(g.mid_hi, (tl.tile + 1) * kTileRows);
  count_digits<kTileRows / kSelThreads>(p.score + p.off[c], j_begin, j_end, st.prefix, mask, shift, hist);
  __syncthreads();
  if (tid < 256) p.tile_hist[((int64_t)(tl.first_tile + tl.tile) * 4 + PASS) * 256 + tid] = hist[tid];
}

__global__ __launch_bounds__(kSelThreads) void compact_tile_emit_kernel(CompactParams p) {
  const SelTile tl = p.tiles[blockIdx.x];
  const int c = tl.c;
  const int tid = threadIdx.x;
  const SelGoal g = sel_goal(p, c);
  const int n = g.n;
  const int64_t off = p.off[c];
  int32_t* kept = p.kept + off;
  const int j_begin = tl.tile * kTileRows, j_end = min(n, (tl.tile + 1) * kTileRows);
  if (n <= g.b) {
    if (p.write_identity)
      for (int j = j_begin + tid; j < j_end; j += kSelThreads) kept[j] = j;
    return;
  }
  __shared__ int hist[256];
  __shared__ int sm_scan[kSelWaves];
  __shared__ int sh_digit, sh_need, sh_first;
  __shared__ uint32_t lds_key[kEmitKeyWords];
  uint32_t thr = 0;
  int need_eq = 0, sure_base = 0, eq_base = 0;
  if (g.k > 0) {
    const SelState st = state_before_pass<4>(p, tl, g.k, hist, sm_scan, &sh_digit, &sh_need);
    thr = st.prefix;
    need_eq = st.need;
    // Survivors in the tiles before this one, from their counters: keys that some pass ranked above the
    // threshold's digit, and keys equal to the threshold (capped by need_eq where they are used).
    // One wavefront per earlier tile in turn, its 64 lanes over the 256 counters of each pass.
    const int lane = tid & 63, wave = tid >> 6;
    int sure = 0, eq = 0;
    for (int j = wave; j < tl.tile; j += kSelWaves) {
      const int32_t* th = p.tile_hist + (int64_t)(tl.first_tile + j) * 4 * 256;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int d = lane + 64 * q;
#pragma unroll
        for (int ps = 0; ps < 4; ++ps) sure += d > st.digit[ps] ? th[ps * 256 + d] : 0;
        eq += d == st.digit[3] ? th[3 * 256 + d] : 0;
      }
    }
    (void)block_exclusive_scan(sure, sm_scan, sure_base);
    (void)block_exclusive_scan(eq, sm_scan, eq_base);
  }
  const int before = min(j_begin, n);  // rows in front of this tile
  sure_base += min(before, g.mid_lo) + max(0, before - g.mid_hi);
  if (tid == 0) sh_first = n;
  __syncthreads();
  if (j_begin < j_end)
    emit_rows(p.score + off, kept, g, thr, need_eq, j_begin, j_end, sure_base, eq_base, sm_scan, &sh_first, lds_key);
  __syncthreads();
  if (tid == 0 && sh_first < n) atomicMin(&p.info[c].first_moved, sh_first);
}

constexpr int kMoveThreads = 512;
constexpr int kMoveRows = 128;  // rows per tile

// The move is stable and in place: row p <- row kept[p], with kept[p] >= p and
// kept[p] - p <= (rows evicted) <= capacity - budget.  A cache's destination range is cut into
// segments of kMoveSegRows rows, one workgroup each.  Inside a segment tiles go in ascending
// order and every load of a tile finishes (barrier) before any store, so a tile's sources are
// never rows an earlier tile wrote.  The only rows a segment reads that another segment writes
// are the few at its end whose source lies past the segment: those are copied to a halo slot
// by a first kernel, before anything is overwritten.

// Phase 1: save the halo of every segment that has a successor.
template <int PIECES>
__global__ __launch_bounds__(256) void compact_halo_kernel(CompactParams p) {
  const MoveSeg sg = p.segs[blockIdx.x];
  const CompactInfo info = p.info[sg.c];
  if (info.first_moved >= info.old_len) return;  // nothing evicted
  const int b = info.new_len;
  const int e = sg.a + kMoveSegRows;
  if (e >= b || sg.halo_row < 0) return;         // last segment: its far sources are overwritten by nobody
  const int tid = threadIdx.x;
  const int64_t off = p.off[sg.c];
  const int32_t* kept = p.kept + off;
  // first destination row whose source is at or past the segment end (kept is ascending)
  int lo = sg.a, hi = e;
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if (kept[mid] >= e) hi = mid; else lo = mid + 1;
  }
  const int split = lo, n_halo = e - split;
  if (tid == 0) p.seg_split[p.seg_base + blockIdx.x] = split;
  const uint4* K = reinterpret_cast<const uint4*>(p.k) + off * PIECES;
  const uint4* V = reinterpret_cast<const uint4*>(p.v) + off * PIECES;
  uint4* HK = reinterpret_cast<uint4*>(p.halo_k) + (int64_t)sg.halo_row * PIECES;
  uint4* HV = reinterpret_cast<uint4*>(p.halo_v) + (int64_t)sg.halo_row * PIECES;
  for (int idx = tid; idx < n_halo * PIECES; idx += 256) {
    const int r = idx / PIECES, piece = idx % PIECES;
    const int64_t src = kept[split + r];
    HK[(int64_t)r * PIECES + piece] = K[src * PIECES + piece];
    HV[(int64_t)r * PIECES + piece] = V[src * PIECES + piece];
  }
  for (int r = tid; r < n_halo; r += 256) {
    const int src = kept[split + r];
    p.halo_score[sg.halo_row + r] = p.score[off + src];
    p.halo_pos[sg.halo_row + r] = p.pos[off + src];
  }
}

// Phase 2: the move itself.
// K/V rows are read once and written once here: non-temporal loads and stores (measured: the move
// of a full eviction is 14% faster with them).
#define BAKLAVA_MOVE_LD(ptr) load_nt16(ptr)
#define BAKLAVA_MOVE_ST(ptr, v) store_nt16(ptr, v)
template <int PIECES>  // 16-byte pieces per row
__global__ __launch_bounds__(kMoveThreads) void compact_move_kernel(CompactParams p) {
  const MoveSeg sg = p.segs[blockIdx.x];
  const int c = sg.c;
  const CompactInfo info = p.info[c];
  if (info.first_moved >= info.old_len) return;  // nothing evicted
  const int tid = threadIdx.x;
  const int b = info.new_len;
  if (sg.a == 0 && tid == 0) p.len[c] = b;
  const int e = min(sg.a + kMoveSegRows, b);
  if (e <= info.first_moved) return;             // every row of this segment stays where it is
  // rows [split, e) take their source from the halo slot
  const bool has_halo = (sg.a + kMoveSegRows < b) && sg.halo_row >= 0;
  const int split = has_halo ? p.seg_split[p.seg_base + blockIdx.x] : e;
  const int64_t off = p.off[c];
  const int32_t* kept = p.kept + off;
  constexpr int PER_PLANE = kMoveRows * PIECES / kMoveThreads;  // pieces per thread per plane
  uint4* K = reinterpret_cast<uint4*>(p.k) + off * PIECES;
  uint4* V = reinterpret_cast<uint4*>(p.v) + off * PIECES;
  const uint4* HK = reinterpret_cast<const uint4*>(p.halo_k) + (int64_t)sg.halo_row * PIECES;
  const uint4* HV = reinterpret_cast<const uint4*>(p.halo_v) + (int64_t)sg.halo_row * PIECES;
  float* score = p.score + off;
  int32_t* pos = p.pos + off;

  const int first = max(sg.a, (info.first_moved / kMoveRows) * kMoveRows);
  for (int p0 = first; p0 < e; p0 += kMoveRows) {
    uint4 kb[PER_PLANE], vb[PER_PLANE];
    float sc = 0.f;
    int ps = 0;
#pragma unroll
    for (int i = 0; i < PER_PLANE; ++i) {
      const int idx = tid + i * kMoveThreads;
      const int row = min(p0 + idx / PIECES, e - 1), piece = idx % PIECES;  // clamped: a row of this segment
      if (row >= split) {
        kb[i] = HK[(int64_t)(row - split) * PIECES + piece];
        vb[i] = HV[(int64_t)(row - split) * PIECES + piece];
      } else {
        const int64_t src = kept[row];
        kb[i] = BAKLAVA_MOVE_LD(K + src * PIECES + piece);
        vb[i] = BAKLAVA_MOVE_LD(V + src * PIECES + piece);
      }
    }
    if (tid < kMoveRows && p0 + tid < e) {
      const int row = p0 + tid;
      if (row >= split) {
        sc = p.halo_score[sg.halo_row + row - split];
        ps = p.halo_pos[sg.halo_row + row - split];
      } else {
        const int src = kept[row];
        sc = score[src];
        ps = pos[src];
      }
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < PER_PLANE; ++i) {
      const int idx = tid + i * kMoveThreads;
      const int row = p0 + idx / PIECES, piece = idx % PIECES;
      if (row < e) {
        BAKLAVA_MOVE_ST(K + (int64_t)row * PIECES + piece, kb[i]);
        BAKLAVA_MOVE_ST(V + (int64_t)row * PIECES + piece, vb[i]);
      }
    }
    if (tid < kMoveRows && p0 + tid < e) {
      score[p0 + tid] = sc;
      pos[p0 + tid] = ps;
    }
  }
}

}  // namespace

hipError_t launch_compact_select(const CompactParams& p, int n_caches, int n_tiles, hipStream_t s) {
  if (n_caches <= 0) return hipSuccess;
  compact_select_kernel<<<dim3(n_caches), dim3(kSelThreads), 0, s>>>(p);
  if (n_tiles > 0) {
    const dim3 grid(n_tiles), block(kSelThreads);
    compact_tile_count_kernel<0><<<grid, block, 0, s>>>(p);
    compact_tile_count_kernel<1><<<grid, block, 0, s>>>(p);
    compact_tile_count_kernel<2><<<grid, block, 0, s>>>(p);
    compact_tile_count_kernel<3><<<grid, block, 0, s>>>(p);
    compact_tile_emit_kernel<<<grid, block, 0, s>>>(p);
  }
  return hipGetLastError();
}

hipError_t launch_compact_move(const CompactParams& p, int n_segs, hipStream_t s) {
  if (n_segs <= 0) return hipSuccess;
  const dim3 grid(n_segs);
  switch (p.row_bytes / 16) {
    case 8:
      compact_halo_kernel<8><<<grid, dim3(256), 0, s>>>(p);
      compact_move_kernel<8><<<grid, dim3(kMoveThreads), 0, s>>>(p);
      break;
    case 16:
      compact_halo_kernel<16><<<grid, dim3(256), 0, s>>>(p);
      compact_move_kernel<16><<<grid, dim3(kMoveThreads), 0, s>>>(p);
      break;
    case 32:
      compact_halo_kernel<32><<<grid, dim3(256), 0, s>>>(p);
      compact_move_kernel<32><<<grid, dim3(kMoveThreads), 0, s>>>(p);
      break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace baklava
