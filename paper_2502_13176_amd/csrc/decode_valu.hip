// Decode attention over ragged caches, vector-ALU version, plus the kernels every decode call
// shares: split combine, score update, append, fill.
//
// Each work item (a run of rows of one cache) is one workgroup of four wavefronts.  A 256-byte
// row is spread over 16 lanes as 16-byte pieces, so one wavefront load instruction fetches four
// whole rows, fully coalesced.  Each lane group keeps its own running (max, sum, output) for
// every query head of the group (online softmax, Eq. 1 re-associated) and the groups are merged
// once at the end: no barrier and no cross-group traffic inside the streaming loop.
#include "common.h"
#include "decode_tail.h"

namespace baklava {

namespace {

struct bf16x8 { uint4 raw; };

template <typename T> struct Row;
template <> struct Row<float> {
  static constexpr int EPL = 4;  // elements per 16-byte piece
  __device__ static void widen(const uint4& r, float* f) {
    f[0] = __uint_as_float(r.x); f[1] = __uint_as_float(r.y);
    f[2] = __uint_as_float(r.z); f[3] = __uint_as_float(r.w);
  }
};
template <> struct Row<uint16_t> {  // bf16 storage
  static constexpr int EPL = 8;
  __device__ static void widen(const uint4& r, float* f) {
    f[0] = __uint_as_float(r.x << 16); f[1] = __uint_as_float(r.x & 0xffff0000u);
    f[2] = __uint_as_float(r.y << 16); f[3] = __uint_as_float(r.y & 0xffff0000u);
    f[4] = __uint_as_float(r.z << 16); f[5] = __uint_as_float(r.z & 0xffff0000u);
    f[6] = __uint_as_float(r.w << 16); f[7] = __uint_as_float(r.w & 0xffff0000u);
  }
};

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

constexpr float kNegInf = -__builtin_huge_valf();

// Merge two online-softmax states that share a query head.
__device__ __forceinline__ void merge_state(float& m, float& l, float* acc, int n_acc, float mo,
                                            float lo, const float* acco) {
  const float mn = fmaxf(m, mo);
  const float ms = (mn == kNegInf) ? 0.f : mn;
  const float a = fast_exp2(m - ms), b = fast_exp2(mo - ms);
  l = l * a + lo * b;
  for (int e = 0; e < n_acc; ++e) acc[e] = acc[e] * a + acco[e] * b;
  m = mn;
}

template <typename T, int D, int GT>
__global__ __launch_bounds__(256) void decode_partial_valu(DecodeParams p) {
  constexpr int EPL = Row<T>::EPL;
  constexpr int LPR = D / EPL;   // lanes per row
  constexpr int RPW = 64 / LPR;  // rows per wavefront load
  constexpr int U = 4;           // rows in flight per lane
  constexpr int TILE = RPW * U;
  constexpr int NW = 4;

  const Item it = p.items[blockIdx.x];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int sub = lane % LPR, rg = lane / LPR;
  const int G = p.G;
  const int n_old = p.len[it.c];
  const int64_t off_c = it.row0 - it.start;
  // a fused append only happens while the cache has room (a full cache sets the status word)
  const int add = (p.fused_append && n_old < p.cap[it.c]) ? 1 : 0;
  const int n = n_old + add;
  const int token_pos = p.token_pos_dev ? *p.token_pos_dev : p.token_pos;
  if (p.fused_append) {
    if (add) append_new_row(p, it, n_old, off_c, token_pos);
    else if (it.start == 0 && threadIdx.x == 0) *p.status = 1;
  }
  int cnt = min(it.start + it.count, n) - it.start;
  if (cnt < 0) cnt = 0;
  const int64_t row0 = off_c + it.start;
  const T* Kb = reinterpret_cast<const T*>(p.k) + row0 * D + sub * EPL;
  const T* Vb = reinterpret_cast<const T*>(p.v) + row0 * D + sub * EPL;

  const int c_rel = it.c - p.cache_begin;
  const int64_t qrow0 = (int64_t)(c_rel / p.Hkv) * p.Hq + (int64_t)(c_rel % p.Hkv) * G;
  float qr[GT][EPL];
#pragma unroll
  for (int g = 0; g < GT; ++g) {
    if (g < G) {
      const uint4 raw = *reinterpret_cast<const uint4*>(reinterpret_cast<const T*>(p.q) +
                                                        (qrow0 + g) * D + sub * EPL);
      Row<T>::widen(raw, qr[g]);
#pragma unroll
      for (int e = 0; e < EPL; ++e) qr[g][e] *= p.scale_log2e;
    } else {
#pragma unroll
      for (int e = 0; e < EPL; ++e) qr[g][e] = 0.f;
    }
  }

  float m[GT], l[GT], acc[GT][EPL];
#pragma unroll
  for (int g = 0; g < GT; ++g) {
    m[g] = kNegInf; l[g] = 0.f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[g][e] = 0.f;
  }

  for (int t0 = wave * TILE; t0 < cnt; t0 += NW * TILE) {
    uint4 kraw[U], vraw[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int r = min(t0 + u * RPW + rg, cnt - 1);  // clamped: always a live row of this item
      // read once per step: non-temporal, so that the stream does not displace other cached data
      kraw[u] = load_nt16(Kb + (int64_t)r * D);
      vraw[u] = load_nt16(Vb + (int64_t)r * D);
    }
    float s[U][GT];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float kf[EPL];
      Row<T>::widen(kraw[u], kf);
      const int r = t0 + u * RPW + rg;
      const bool live = r < cnt;
#pragma unroll
      for (int g = 0; g < GT; ++g) {
        float d = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) d = fmaf(qr[g][e], kf[e], d);
#pragma unroll
        for (int o = LPR / 2; o > 0; o >>= 1) d += __shfl_xor(d, o);
        s[u][g] = live ? d : kNegInf;
      }
    }
#pragma unroll
    for (int g = 0; g < GT; ++g) {
      float mx = s[0][g];
#pragma unroll
      for (int u = 1; u < U; ++u) mx = fmaxf(mx, s[u][g]);
      const float mn = fmaxf(m[g], mx);
      const float ms = (mn == kNegInf) ? 0.f : mn;
      const float alpha = fast_exp2(m[g] - ms);
      m[g] = mn;
      l[g] *= alpha;
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc[g][e] *= alpha;
#pragma unroll
      for (int u = 0; u < U; ++u) s[u][g] = fast_exp2(s[u][g] - ms);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float vf[EPL];
      Row<T>::widen(vraw[u], vf);
#pragma unroll
      for (int g = 0; g < GT; ++g) {
        l[g] += s[u][g];
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[g][e] = fmaf(s[u][g], vf[e], acc[g][e]);
      }
    }
  }

  // Merge the lane groups of a wavefront (lanes with equal `sub`).
#pragma unroll
  for (int o = LPR; o < 64; o <<= 1) {
#pragma unroll
    for (int g = 0; g < GT; ++g) {
      float acco[EPL];
      const float mo = __shfl_xor(m[g], o), lo = __shfl_xor(l[g], o);
#pragma unroll
      for (int e = 0; e < EPL; ++e) acco[e] = __shfl_xor(acc[g][e], o);
      merge_state(m[g], l[g], acc[g], EPL, mo, lo, acco);
    }
  }

  // Hand the four wavefronts' results over through LDS.
  __shared__ float sm[NW * GT * D + 2 * NW * GT];
  float* sm_o = sm;                  // [NW][GT][D]
  float* sm_m = sm + NW * GT * D;    // [NW][GT]
  float* sm_l = sm_m + NW * GT;      // [NW][GT]
  if (rg == 0) {
#pragma unroll
    for (int g = 0; g < GT; ++g) {
      if (sub == 0) { sm_m[wave * GT + g] = m[g]; sm_l[wave * GT + g] = l[g]; }
#pragma unroll
      for (int e = 0; e < EPL; ++e) sm_o[(wave * GT + g) * D + sub * EPL + e] = acc[g][e];
    }
  }
  __syncthreads();
  finish_item<D, GT>(p, it, G, n, sm_o, sm_m, sm_l);
}

// Merge of the split partials of one (cache, query head):
//   out = sum_s o_s 2^(m_s - M) / sum_s l_s 2^(m_s - M)
// which is the softmax of Eq. 7 with the sum over rows regrouped by split.  One workgroup per
// (cache with several work items, query head); 256 / D thread groups share the splits.
template <int D>
__global__ __launch_bounds__(256) void combine_kernel(DecodeParams p) {
  constexpr int GROUPS = 256 / D;
  const int G = p.G;
  const MultiCache mc = p.multi[blockIdx.x / G];
  const int c = mc.c;
  const int g = blockIdx.x % G;
  const int tid = threadIdx.x;
  const int d = tid % D, grp = tid / D;
  const int ib = mc.slot_begin, ie = mc.slot_end;
  // where this call's record goes; read by every thread before the barrier below, written after it
  const int slot = p.lag ? lag_slot(p, p.lag_cnt[(int64_t)c * G + g]) : 0;
  float m = kNegInf, l = 0.f, o = 0.f;
#pragma unroll 8
  for (int s = ib + grp; s < ie; s += GROUPS) {
    const float ms = p.part_ml[((int64_t)s * G + g) * 2];
    const float ls = p.part_ml[((int64_t)s * G + g) * 2 + 1];
    const float os = p.part_o[((int64_t)s * G + g) * D + d];
    const float mn = fmaxf(m, ms);
    const float msafe = (mn == kNegInf) ? 0.f : mn;
    const float a = fast_exp2(m - msafe), b = fast_exp2(ms - msafe);
    l = l * a + ls * b;
    o = o * a + os * b;
    m = mn;
  }
  __shared__ float red_o[GROUPS][D], red_m[GROUPS], red_l[GROUPS];
  red_o[grp][d] = o;
  if (d == 0) { red_m[grp] = m; red_l[grp] = l; }
  __syncthreads();
  if (grp == 0) {
    float mm = red_m[0];
#pragma unroll
    for (int w = 1; w < GROUPS; ++w) mm = fmaxf(mm, red_m[w]);
    const float ms = (mm == kNegInf) ? 0.f : mm;
    float ll = 0.f, oo = 0.f;
#pragma unroll
    for (int w = 0; w < GROUPS; ++w) {
      const float a = fast_exp2(red_m[w] - ms);
      ll += red_l[w] * a;
      oo += red_o[w][d] * a;
    }
    const float inv = 1.f / ll;
    const int c_rel = c - p.cache_begin;
    const int64_t orow = (int64_t)(c_rel / p.Hkv) * p.Hq + (int64_t)(c_rel % p.Hkv) * G + g;
    int n_now = 0;  // live rows after this call (thread 0 of head 0's block)
    p.out[orow * D + d] = oo * inv;
    if (d == 0) {
      p.final_ml[((int64_t)c * G + g) * 2 + 0] = ms;
      p.final_ml[((int64_t)c * G + g) * 2 + 1] = inv;
      if (g == 0) {
        int n = p.len[c];
        if (p.fused_append && n < p.cap[c]) p.len[c] = ++n;  // the fused append's row is now counted
        n_now = n;
      }
    }
    // This head's part of the record a later score pass over the cache needs (see DecodeParams).
    // Each block reads and writes the pending-call counter of its own head only.
    if (p.lag) {
      const int64_t m = (int64_t)c * kLagRows + (slot << p.lag_gp_log2) + g;
      if (tid * 16 < p.row_bytes) {
        const uint4* src = reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(p.q) + orow * p.row_bytes);
        reinterpret_cast<uint4*>(reinterpret_cast<char*>(p.lag_q) + m * p.row_bytes)[tid] = src[tid];
      }
      if (d == 0) {
        p.lag_ml[m * 2 + 0] = ms;
        p.lag_ml[m * 2 + 1] = inv;
        if (g == 0) p.lag_n[(int64_t)c * kLagCalls + slot] = n_now;
        p.lag_cnt[(int64_t)c * G + g] = slot + 1;
      }
    }
  }
}

// score_j += sum_g 2^(q_g . k_j scale - M_g) / L_g  (cumulative attention per cached token, summed
// over the query heads that share the cache), from the K rows alone once the normalisers of the
// call are final: the vector-ALU path's score update, launched right after its attention call.
// Workgroup (x, y) updates rows [y * kScoreTile, +kScoreTile) of work item x, so that long work
// items still spread over many workgroups.  Row layout as in the attention kernel above: a row
// over D / EPL lanes, 64 / (D / EPL) rows per wavefront load.
constexpr int kScoreTile = 1024;
template <typename T, int D, int GT>
__global__ __launch_bounds__(256) void score_pass_kernel(ScoreParams p) {
  constexpr int EPL = Row<T>::EPL;
  constexpr int LPR = D / EPL;
  constexpr int RPW = 64 / LPR;
  const Item it = p.items[blockIdx.x];
  const int G = p.G;
  const int cnt = min(it.start + it.count, p.len[it.c]) - it.start;
  const int r_begin = blockIdx.y * kScoreTile;
  if (r_begin >= cnt) return;
  const int r_end = min(cnt, r_begin + kScoreTile);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int sub = lane % LPR, rg = lane / LPR;
  const int c_rel = it.c - p.cache_begin;
  const T* qrows = reinterpret_cast<const T*>(p.q) +
                   ((int64_t)(c_rel / p.Hkv) * p.Hq + (int64_t)(c_rel % p.Hkv) * G) * D;
  float qr[GT][EPL], M[GT], inv[GT];
#pragma unroll
  for (int g = 0; g < GT; ++g) {
    M[g] = 0.f;
    inv[g] = 0.f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) qr[g][e] = 0.f;
    if (g < G) {
      Row<T>::widen(*reinterpret_cast<const uint4*>(qrows + g * D + sub * EPL), qr[g]);
#pragma unroll
      for (int e = 0; e < EPL; ++e) qr[g][e] *= p.scale_log2e;
      M[g] = p.ml[((int64_t)it.c * G + g) * 2];
      inv[g] = p.ml[((int64_t)it.c * G + g) * 2 + 1];
    }
  }
  const T* Kb = reinterpret_cast<const T*>(p.k) + it.row0 * D + sub * EPL;
  float* sc = p.score + it.row0;
  for (int r0 = r_begin + wave * RPW; r0 < r_end; r0 += 4 * RPW) {
    const int r = r0 + rg;
    float kf[EPL];
    Row<T>::widen(load_nt16(Kb + (int64_t)min(r, r_end - 1) * D), kf);
    float w = 0.f;
#pragma unroll
    for (int g = 0; g < GT; ++g) {
      float d = 0.f;
#pragma unroll
      for (int e = 0; e < EPL; ++e) d = fmaf(qr[g][e], kf[e], d);
#pragma unroll
      for (int o = LPR / 2; o > 0; o >>= 1) d += __shfl_xor(d, o);
      w += fast_exp2(d - M[g]) * inv[g];  // heads beyond G: 2^0 * 0
    }
    if (r < r_end && sub == 0) sc[r] += w;
  }
}

// [K'; K_t], [V'; V_t] of Eq. 7: the new row goes to slot len, then len += 1.
__global__ __launch_bounds__(64) void append_kernel(AppendParams p) {
  const int c = p.cache_begin + blockIdx.x;
  const int n = p.len[c];
  if (n >= p.cap[c]) return;  // the host has already refused this case
  const int64_t row = p.off[c] + n;
  const int pieces = p.row_bytes / 16;
  const int lane = threadIdx.x;
  const int plane = lane / 32, piece = lane % 32;
  if (piece < pieces) {
    const char* src = reinterpret_cast<const char*>(plane ? p.v_new : p.k_new) +
                      (int64_t)blockIdx.x * p.row_bytes + piece * 16;
    char* dst = reinterpret_cast<char*>(plane ? p.v : p.k) + row * p.row_bytes + piece * 16;
    *reinterpret_cast<uint4*>(dst) = *reinterpret_cast<const uint4*>(src);
  }
  if (lane == 63) {
    p.score[row] = 0.f;
    p.pos[row] = p.token_pos_dev ? *p.token_pos_dev : p.token_pos;
  }
  __syncthreads();
  if (lane == 0) p.len[c] = n + 1;
}

__global__ void fill_i32_kernel(int32_t* dst, int32_t value, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = value;
}

template <typename T, int D>
hipError_t launch_valu_g(const DecodeParams& p, int n_items, hipStream_t s) {
  const dim3 grid(n_items), block(256);
  if (p.G <= 2) decode_partial_valu<T, D, 2><<<grid, block, 0, s>>>(p);
  else if (p.G <= 4) decode_partial_valu<T, D, 4><<<grid, block, 0, s>>>(p);
  else if (p.G <= 8) decode_partial_valu<T, D, 8><<<grid, block, 0, s>>>(p);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace

hipError_t launch_decode_valu(const DecodeParams& p, int dtype, int D, int n_items, hipStream_t s) {
  if (n_items <= 0) return hipSuccess;
  if (dtype == 0 && D == 128) return launch_valu_g<uint16_t, 128>(p, n_items, s);
  if (dtype == 0 && D == 64) return launch_valu_g<uint16_t, 64>(p, n_items, s);
  if (dtype == 1 && D == 128) return launch_valu_g<float, 128>(p, n_items, s);
  if (dtype == 1 && D == 64) return launch_valu_g<float, 64>(p, n_items, s);
  return hipErrorInvalidValue;
}

hipError_t launch_combine(const DecodeParams& p, int D, int n_multi, hipStream_t s) {
  if (n_multi <= 0) return hipSuccess;
  const dim3 grid(n_multi * p.G), block(256);
  if (D == 128) combine_kernel<128><<<grid, block, 0, s>>>(p);
  else if (D == 64) combine_kernel<64><<<grid, block, 0, s>>>(p);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

template <typename T, int D>
hipError_t launch_score_g(const ScoreParams& p, const dim3& grid, hipStream_t s) {
  if (p.G <= 4) score_pass_kernel<T, D, 4><<<grid, dim3(256), 0, s>>>(p);
  else if (p.G <= 8) score_pass_kernel<T, D, 8><<<grid, dim3(256), 0, s>>>(p);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t launch_score_pass(const ScoreParams& p, int dtype, int D, int n_items, int max_count, hipStream_t s) {
  if (n_items <= 0 || max_count <= 0) return hipSuccess;
  const dim3 grid(n_items, (max_count + kScoreTile - 1) / kScoreTile);
  if (dtype == 0 && D == 128) return launch_score_g<uint16_t, 128>(p, grid, s);
  if (dtype == 0 && D == 64) return launch_score_g<uint16_t, 64>(p, grid, s);
  if (dtype == 1 && D == 128) return launch_score_g<float, 128>(p, grid, s);
  if (dtype == 1 && D == 64) return launch_score_g<float, 64>(p, grid, s);
  return hipErrorInvalidValue;
}

hipError_t launch_append(const AppendParams& p, int n_caches, hipStream_t s) {
  if (n_caches <= 0) return hipSuccess;
  append_kernel<<<dim3(n_caches), dim3(64), 0, s>>>(p);
  return hipGetLastError();
}

hipError_t launch_fill_i32(int32_t* dst, int32_t value, int64_t n, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  fill_i32_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s>>>(dst, value, n);
  return hipGetLastError();
}

}  // namespace baklava
