// Budget-enforcing eviction (f_evict, Eqs. 5-6): selection of the surviving rows (one workgroup
// per cache, long caches first), then a stable in-place move (one workgroup per segment).
#include "common.h"

namespace baklava {

namespace {

constexpr int kSelThreads = 512;
constexpr int kSelWaves = kSelThreads / 64;
constexpr int kSelUnroll = 8;  // score loads in flight per thread in the counting passes
constexpr int kSelRows = 4;    // consecutive rows per thread in the emit pass

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

__global__ __launch_bounds__(kSelThreads) void compact_select_kernel(CompactParams p) {
  const int c = p.order[blockIdx.x];
  const int tid = threadIdx.x;
  const int n = p.len[c];
  const int cpl = p.batch * p.Hkv;
  const int b = p.budget[(c / cpl) * p.Hkv + c % p.Hkv];
  const int64_t off = p.off[c];
  int32_t* kept = p.kept + off;
  const float* score = p.score + off;

  if (n <= b) {
    if (p.write_identity)
      for (int j = tid; j < n; j += kSelThreads) kept[j] = j;
    if (tid == 0) p.info[c] = CompactInfo{n, n, n, 0};
    return;
  }
  const int s = p.sink;
  const int r = (p.policy == 1) ? (b - s) : p.recent;
  const int k = b - s - r;  // middle rows that survive, >= 0 (checked at context creation)
  const int mid_lo = s, mid_hi = n - r;

  __shared__ int hist[256];
  __shared__ int sm_scan[kSelWaves];
  __shared__ uint32_t sh_prefix;
  __shared__ int sh_need, sh_first;

  uint32_t thr = 0;
  int need_eq = 0;
  if (k > 0) {
    // Radix select of the k-th largest key of the middle, 8 bits per pass, high digits first.
    uint32_t prefix = 0, mask = 0;
    int need = k;
    for (int shift = 24; shift >= 0; shift -= 8) {
      for (int i = tid; i < 256; i += kSelThreads) hist[i] = 0;
      __syncthreads();
      // kSelUnroll independent loads per thread before the first use
      for (int j0 = mid_lo + tid; j0 < mid_hi; j0 += kSelThreads * kSelUnroll) {
        uint32_t key[kSelUnroll];
#pragma unroll
        for (int u = 0; u < kSelUnroll; ++u) {
          const int j = j0 + u * kSelThreads;
          key[u] = score_key(j < mid_hi ? score[j] : 0.f);
        }
#pragma unroll
        for (int u = 0; u < kSelUnroll; ++u) {
          const int j = j0 + u * kSelThreads;
          const bool live = j < mid_hi && (key[u] & mask) == prefix;
          const uint32_t digit = (key[u] >> shift) & 255;
          if (live) atomicAdd(&hist[digit], 1);
        }
      }
      __syncthreads();
      // The digit of the need-th largest key: thread t looks at digit 255 - t; `above` = keys with a
      // larger digit.  Exactly one digit has above < need <= above + its own count.
      {
        const int mine = tid < 256 ? hist[255 - tid] : 0;
        int all;
        const int above = block_exclusive_scan(mine, sm_scan, all);
        if (tid < 256 && above < need && above + mine >= need) {
          sh_prefix = prefix | ((uint32_t)(255 - tid) << shift);
          sh_need = need - above;
        }
      }
      __syncthreads();
      prefix = sh_prefix;
      need = sh_need;
      mask |= 0xffu << shift;
      __syncthreads();
    }
    thr = prefix;
    need_eq = need;  // rows whose key equals thr that still survive (oldest first)
  }

  // Stable emit, kSelRows consecutive rows per thread and tile.  A row survives if it is a sink or
  // recent row, if its key exceeds the threshold, or if it is among the first need_eq rows whose key
  // equals it; its place in the list is the number of survivors before it, i.e. (rows of the first
  // two kinds before it) + min(rows with an equal key before it, need_eq).  Both counts come from
  // one workgroup scan of a packed pair (at most kSelRows * kSelThreads < 2^16 per tile).
  if (tid == 0) sh_first = n;
  __syncthreads();
  int sure_base = 0, eq_base = 0;
  for (int j0 = 0; j0 < n; j0 += kSelThreads * kSelRows) {
    const int jt = j0 + tid * kSelRows;
    uint32_t key[kSelRows];
    bool sure[kSelRows], eq[kSelRows];
    int n_sure = 0, n_eq = 0;
#pragma unroll
    for (int i = 0; i < kSelRows; ++i) {
      const int j = jt + i;
      const bool in = j < n;
      const bool middle = in && j >= mid_lo && j < mid_hi;
      key[i] = (middle && k > 0) ? score_key(score[j]) : 0u;
      sure[i] = (in && !middle) || (middle && k > 0 && key[i] > thr);
      eq[i] = middle && k > 0 && key[i] == thr;
      n_sure += sure[i] ? 1 : 0;
      n_eq += eq[i] ? 1 : 0;
    }
    int total;
    const int excl = block_exclusive_scan(n_sure | (n_eq << 16), sm_scan, total);
    int sure_before = sure_base + (excl & 0xffff);
    int eq_before = eq_base + (excl >> 16);
    int first_out = n;
#pragma unroll
    for (int i = 0; i < kSelRows; ++i) {
      const int j = jt + i;
      const bool keep = sure[i] || (eq[i] && eq_before < need_eq);
      if (keep) kept[sure_before + min(eq_before, need_eq)] = j;
      else if (j < n) first_out = min(first_out, j);
      sure_before += sure[i] ? 1 : 0;
      eq_before += eq[i] ? 1 : 0;
    }
    // rows leave in ascending order of the tiles, so only the first tile that evicts has to report
    if (first_out < n && first_out < *(volatile int*)&sh_first) atomicMin(&sh_first, first_out);
    sure_base += total & 0xffff;
    eq_base += total >> 16;
  }
  __syncthreads();
  if (tid == 0) p.info[c] = CompactInfo{b, sh_first, n, 0};
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

hipError_t launch_compact_select(const CompactParams& p, int n_caches, hipStream_t s) {
  if (n_caches <= 0) return hipSuccess;
  compact_select_kernel<<<dim3(n_caches), dim3(kSelThreads), 0, s>>>(p);
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
