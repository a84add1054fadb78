// Decode attention over ragged caches, MFMA version (bf16, D = 128, up to 16 query heads per
// KV head).
//
// The G query heads that share a KV head form the N side (padded to 16) of two matrix products
// per 32-row slab, both issued as v_mfma_f32_16x16x32_bf16:
//
//   S^T[row, g]  = K[row, :] . Q[g, :]          A = K rows (staged through LDS: whole rows are
//                                               loaded, lane (row%16, j) then reads its 8
//                                               consecutive head-dim elements), B = Q
//   O^T[d, g]   += V^T[d, rows] . P^T[rows, g]  A = V^T (staged through LDS, read back
//                                               transposed), B = P^T
//
// The accumulator layout of S^T (lane (g, j) holds rows 4j..4j+3 of each 16-row tile) is
// already a valid B-operand layout for the second product once the slab's 32 rows are numbered
// k = 8j + 4*tile + i, so the softmax weights never leave their lane; V^T is read from LDS
// with the same numbering.  Each query head's statistics (running max, sum) live in the 4 lanes
// g, g+16, g+32, g+48.  Softmax weights are split into two bf16 terms (high part and residual)
// so that the second product keeps ~16 bits of each weight.
//
// Both K and V are fetched as whole 256-byte rows, four rows per load instruction.  Reading K
// straight into the A-operand layout would save its trip through LDS, but touches only 64 bytes
// of each of 16 rows per instruction, and that access shape streams about 10% slower from HBM
// than whole rows do.
//
// Each wavefront of a workgroup streams its own 32-row slabs and owns a private LDS region: there
// is no barrier inside the loop.
//
// Score tracking (cumulative attention per cached row) rides on the same stream, a few calls late:
// a row's weight needs the softmax normaliser of the whole cache, which no work item knows before
// the call is over.  So each call records its query rows and final (max, 1/sum) per cache, and a
// later call -- whose K rows pass through LDS anyway -- forms the recorded calls' logits with one
// more product that reuses the K operands (the matrix pipe is < 10% busy), turns them into
// normalised weights and adds them to the scores.  The G query heads fill only G of the 16 rows of
// a matrix operand, so the rows of up to 32 / G recorded calls are packed into two operands and
// the scores are touched only on every (32 / G)-th call (every 8th at G <= 4).  On such a call the
// scores of a slab are read with the slab and the new values wait in LDS until the work item is
// done, so the extra HBM writes (4 bytes per row) fall at the end of a launch instead of between
// the K/V reads.
#include <hip/hip_ext.h>

#include "common.h"
#include "decode_tail.h"

#include <algorithm>
#include <type_traits>

namespace baklava {

namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float floatx4_t __attribute__((ext_vector_type(4)));

#ifndef BAKLAVA_MFMA_NW
#define BAKLAVA_MFMA_NW 4
#endif
constexpr int kWaves = BAKLAVA_MFMA_NW;
constexpr int kSlab = 32;       // rows per wavefront iteration
constexpr int kVStride = 288;   // bytes between staged V rows: 256 + 32, so the 16 rows touched by one
                                // transposed read spread evenly over the LDS banks
constexpr int kKStride = 272;   // bytes between staged K rows: 256 + 16, so 16 lanes that read the same
                                // 16 bytes of 16 consecutive rows hit 16 different bank groups
constexpr int kD = 128;
constexpr float kNegInf = -__builtin_huge_valf();

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
typedef short s16x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ bf16x8_t as_bf16x8(u32x4_t x) { return __builtin_bit_cast(bf16x8_t, x); }

// The recorded calls of one cache as a lane sees them.  The packed query rows fill kSets operands
// of 16 rows (packed row R = call * G' + head sits in operand R / 16, row R % 16); each is the A
// operand of a product S' = Q' K^T (lane (m, j), chunk c holds row m, elements 32c + 8j .. +8) that
// leaves lane (row, jg) with the logits of the operand's rows 4*jg .. 4*jg+3, which all belong to
// one call, so the lane keeps their (max, 1/sum) and the number of rows that call saw.
constexpr int kSets = 2;
constexpr int kRecRows = 16 * kSets;  // packed rows of a record
constexpr int kRecCalls = 8;          // most calls a record holds (G <= 4)
struct Record {
  bf16x8_t q[kSets][4];
  float m[kSets][4], inv[kSets][4];
  int n_slot[kSets];
};

__device__ __forceinline__ void load_record(const DecodeParams& p, int c, int G, int pending, int n16, int jg,
                                            Record& r) {
  const int gp_mask = (1 << p.lag_gp_log2) - 1;
  const unsigned char* lq = reinterpret_cast<const unsigned char*>(p.lag_q) + (int64_t)c * kRecRows * (kD * 2);
#pragma unroll
  for (int e = 0; e < kSets; ++e) {
    const int R = 16 * e + n16;  // the packed row this lane holds a part of
#pragma unroll
    for (int ch = 0; ch < 4; ++ch) {
      u32x4_t raw = {0u, 0u, 0u, 0u};  // rows beyond the G heads of a call, calls not on record: zero
      if ((R & gp_mask) < G && (R >> p.lag_gp_log2) < pending)
        raw = *reinterpret_cast<const u32x4_t*>(lq + R * (kD * 2) + ch * 64 + jg * 16);
      r.q[e][ch] = as_bf16x8(raw);
    }
    const int slot = (16 * e + 4 * jg) >> p.lag_gp_log2;
    r.n_slot[e] = 0;
    if (slot < pending) r.n_slot[e] = p.lag_n[(int64_t)c * kRecCalls + slot];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int m = 16 * e + 4 * jg + i;
      r.m[e][i] = 0.f;
      r.inv[e][i] = 0.f;
      if ((m & gp_mask) < G && slot < pending) {
        r.m[e][i] = p.lag_ml[((int64_t)c * kRecRows + m) * 2];
        r.inv[e][i] = p.lag_ml[((int64_t)c * kRecRows + m) * 2 + 1];
      }
    }
  }
}

// Weights the recorded calls give to the 32 rows of a slab whose first row has cache index `row_first`:
// sum over calls and heads of 2^(s' - M') / L' for the rows a call saw.  sp[e][T] holds the logits of
// operand e and tile T as the product left them.  On return lane l < 32 holds the weight of row l of
// the slab.
__device__ __forceinline__ float record_weights(const floatx4_t (&sp)[kSets][2], const Record& r, float cs,
                                                int row_first, int lane) {
  const int n16 = lane & 15;
  float w[2];
#pragma unroll
  for (int T = 0; T < 2; ++T) {
    w[T] = 0.f;
#pragma unroll
    for (int e = 0; e < kSets; ++e) {
      float acc = 0.f;
#pragma unroll
      for (int i = 0; i < 4; ++i) acc += fast_exp2(sp[e][T][i] * cs - r.m[e][i]) * r.inv[e][i];
      // a row the call did not see is left out by a select: its logit may be anything
      w[T] += (row_first + T * 16 + n16 < r.n_slot[e]) ? acc : 0.f;
    }
    w[T] += __shfl_xor(w[T], 16);  // an operand's rows 4*jg .. 4*jg+3 sit in lane group jg
    w[T] += __shfl_xor(w[T], 32);
  }
  return (lane & 16) ? w[1] : w[0];
}

#ifndef BAKLAVA_MFMA_WAVES_PER_EU
#define BAKLAVA_MFMA_WAVES_PER_EU 2
#endif
template <bool LAG>
__global__ __launch_bounds__(64 * kWaves, BAKLAVA_MFMA_WAVES_PER_EU) void decode_partial_mfma(DecodeParams p) {
  __shared__ __attribute__((aligned(16))) unsigned char lds[kWaves * kSlab * kVStride];
  __shared__ __attribute__((aligned(16))) unsigned char lds_k[kWaves * kSlab * kKStride];  // K staging
  // LAG: the new scores of the slabs a wavefront has processed ([32] floats per slab, p.ring_slots
  // slabs per wavefront) wait here until the work item is done (or the area is full), so that the
  // score writes of a launch fall together at its end instead of being interleaved with the K/V
  // reads, which the memory system handles badly.
  extern __shared__ __attribute__((aligned(16))) float lds_ring[];

  const Item it = p.items[blockIdx.x];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n16 = lane & 15, jg = lane >> 4;
  const int G = p.G;
  // Table entries are read before the fused append stores anything, so that they stay scalar loads.
  const int n_old = p.len[it.c];
  const int64_t off_c = it.row0 - it.start;
  // A fused append only happens while the cache has room; a full cache is attended as it is and
  // reported through the status word.
  const int add = (p.fused_append && n_old < p.cap[it.c]) ? 1 : 0;
  const int n = n_old + add;
  const int token_pos = p.token_pos_dev ? *p.token_pos_dev : p.token_pos;
  // Recorded calls (LAG).  When the record is full this call adds their weights to the scores.
  const int pending = LAG ? p.lag_cnt[(int64_t)it.c * G] : 0;
  const bool apply = LAG && pending >= p.lag_batch;
  Record rec;
  if (LAG && apply) load_record(p, it.c, G, pending, n16, jg, rec);
  if (p.fused_append) {
    if (add) append_new_row(p, it, n_old, off_c, token_pos);
    else if (it.start == 0 && threadIdx.x == 0) *p.status = 1;
  }
  int cnt = min(it.start + it.count, n) - it.start;
  if (cnt < 0) cnt = 0;
  const int64_t row0 = off_c + it.start;
  const unsigned char* Kb = reinterpret_cast<const unsigned char*>(p.k) + row0 * (kD * 2);
  const unsigned char* Vb = reinterpret_cast<const unsigned char*>(p.v) + row0 * (kD * 2);
  unsigned char* myl = lds + wave * (kSlab * kVStride);
  unsigned char* myk = lds_k + wave * (kSlab * kKStride);

  const int c_rel = it.c - p.cache_begin;
  const int64_t qrow0 = (int64_t)(c_rel / p.Hkv) * p.Hq + (int64_t)(c_rel % p.Hkv) * G;

  floatx4_t o[8];
#pragma unroll
  for (int b = 0; b < 8; ++b) o[b] = floatx4_t{0.f, 0.f, 0.f, 0.f};
  float m_run = kNegInf;  // running max of head n16, log2 units, equal in the 4 lanes of a head
  float l_part = 0.f;     // this lane's share of the running sum
  const float cs = p.scale_log2e;

  // Row indices are clamped to the last live row of the work item, so nothing outside the live
  // rows is ever read; a clamped row's softmax weight is forced to zero below.  Offsets from the
  // item's first row fit 32 bits (a work item spans < 2^23 rows).
  const int last = cnt - 1;
  const uint32_t v_lane = n16 * 16;
  u32x4_t kr[8];
  u32x4_t vr[8];

  // K and V rows are read once per step: non-temporal loads keep them from displacing the rest of
  // the cache hierarchy's contents (measured: +4.6% on the attention kernel).
#define BAKLAVA_LD(ptr) __builtin_nontemporal_load(ptr)
#define BAKLAVA_LOAD_K(T0)                                                                        \
  _Pragma("unroll") for (int i = 0; i < 8; ++i) {                                                 \
    const uint32_t off = (uint32_t)min((T0) + jg + 4 * i, last) * (kD * 2) + v_lane;              \
    kr[i] = BAKLAVA_LD(reinterpret_cast<const u32x4_t*>(Kb + off));                               \
  }
#define BAKLAVA_LOAD_V(T0)                                                                        \
  _Pragma("unroll") for (int i = 0; i < 8; ++i) {                                                 \
    const uint32_t off = (uint32_t)min((T0) + jg + 4 * i, last) * (kD * 2) + v_lane;              \
    vr[i] = BAKLAVA_LD(reinterpret_cast<const u32x4_t*>(Vb + off));                               \
  }

  // LAG: lane l < 32 owns row l of each slab.  The row's score is fetched with the slab's K rows;
  // the new value goes to this wavefront's part of the LDS area and from there to HBM when the work
  // item is done.
  float* const sc_base = p.score + row0;
  float sc_cur = 0.f;
#define BAKLAVA_LOAD_SC(T0) \
  if (APPLY && lane < kSlab) sc_cur = sc_base[min((T0) + lane, last)];
  float* ring = lds_ring + wave * p.ring_slots * kSlab;
  int ring_n = 0;         // slabs held in the LDS area
  int ring_t0 = 0;        // first row of the oldest one; the others follow at kWaves * kSlab rows each
  auto flush_ring = [&]() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    // two slabs per store instruction: lanes 0..31 take an even slot, lanes 32..63 the next one
    for (int sidx = lane >> 5; sidx < ring_n; sidx += 2) {
      const int r = ring_t0 + sidx * (kWaves * kSlab) + (lane & 31);
      if (r < cnt) sc_base[r] = ring[sidx * kSlab + (lane & 31)];
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();  // the area may be written again
    ring_n = 0;
  };

  // The stream over the work item's rows, compiled twice: with the score update of the recorded
  // calls (APPLY) and without it, so that calls that only record run the plain loop.
  auto stream_rows = [&](auto apply_tag) {
  constexpr bool APPLY = decltype(apply_tag)::value;
  // Order of the first loads: K of the first slab, then the query, then V.  The loop's first wait
  // (for K and, on the first pass, the query) then leaves the V loads in flight, and the stream
  // starts one memory round trip earlier than with the query fetched first.
  int t0 = wave * kSlab;
  if (t0 < cnt) {
    BAKLAVA_LOAD_K(t0)
    BAKLAVA_LOAD_SC(t0)
  }
  // B operand of the first product: lane (g, j), chunk c holds Q[g][32c + 8j .. +8).
  bf16x8_t qb[4];
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    u32x4_t raw = {0u, 0u, 0u, 0u};
    if (n16 < G)
      raw = *reinterpret_cast<const u32x4_t*>(reinterpret_cast<const unsigned char*>(p.q) +
                                              (qrow0 + n16) * (kD * 2) + c * 64 + jg * 16);
    qb[c] = as_bf16x8(raw);
  }
  if (t0 < cnt) {
    BAKLAVA_LOAD_V(t0)
  }

  for (; t0 < cnt; t0 += kWaves * kSlab) {
    const int tn = t0 + kWaves * kSlab;

    // ---- stage K rows in LDS; the next slab's K loads reuse the registers ----------------------
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      *reinterpret_cast<u32x4_t*>(myk + (jg + 4 * i) * kKStride + n16 * 16) = kr[i];
    }
    BAKLAVA_LOAD_K(tn)  // past the end every row clamps to the last live row: harmless re-reads
    const float sc_old = sc_cur;
    BAKLAVA_LOAD_SC(tn)
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    // ---- S^T = K Q^T: lane (row%16, j) reads elements 32c + 8j .. +8 of its row ----------------
    floatx4_t s[2], sp[kSets][2];
#pragma unroll
    for (int T = 0; T < 2; ++T) {
      s[T] = floatx4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int e = 0; e < kSets; ++e) sp[e][T] = floatx4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const u32x4_t a = *reinterpret_cast<const u32x4_t*>(myk + (T * 16 + n16) * kKStride + c * 64 + jg * 16);
        s[T] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(a), qb[c], s[T], 0, 0, 0);
        // The same K registers are a valid B operand (lane (row, j): elements 32c + 8j .. +8 of its
        // row), so S' = Q' K^T costs no further LDS read: lane (row, jg) receives the pending
        // call's logits of heads 4*jg .. 4*jg+3 for row 16T + row of the slab.
        if (APPLY) {
#pragma unroll
          for (int e = 0; e < kSets; ++e)
            sp[e][T] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(rec.q[e][c], as_bf16x8(a), sp[e][T], 0, 0, 0);
        }
      }
    }

    // ---- stage V rows in LDS, then the next slab's V loads reuse the registers ----------------
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      *reinterpret_cast<u32x4_t*>(myl + (jg + 4 * i) * kVStride + n16 * 16) = vr[i];
    }
    BAKLAVA_LOAD_V(tn)

    // ---- online softmax on the accumulator layout --------------------------------------------
    float x[8];
#pragma unroll
    for (int T = 0; T < 2; ++T)
#pragma unroll
      for (int i = 0; i < 4; ++i) x[T * 4 + i] = s[T][i] * cs;
    if (t0 + kSlab > cnt) {
#pragma unroll
      for (int T = 0; T < 2; ++T)
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (t0 + T * 16 + jg * 4 + i >= cnt) x[T * 4 + i] = kNegInf;
    }
    if (APPLY) {
      const float wr = record_weights(sp, rec, cs, it.start + t0, lane);
      if (ring_n == 0) ring_t0 = t0;
      if (lane < kSlab) ring[ring_n * kSlab + lane] = sc_old + wr;  // lane l: row l of the slab
      if (++ring_n == p.ring_slots) flush_ring();
    }
    float mx = x[0];
#pragma unroll
    for (int e = 1; e < 8; ++e) mx = fmaxf(mx, x[e]);
    if (__any(mx > m_run)) {
      mx = fmaxf(mx, __shfl_xor(mx, 16));
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float mn = fmaxf(m_run, mx);  // finite: row t0 is live and belongs to this slab
      const float alpha = fast_exp2(m_run - mn);
      m_run = mn;
      l_part *= alpha;
#pragma unroll
      for (int b = 0; b < 8; ++b) o[b] *= alpha;
    }
    u32x4_t ph;
    bf16x8_t pl;
#pragma unroll
    for (int e = 0; e < 8; e += 2) {
      const float p0 = fast_exp2(x[e] - m_run), p1 = fast_exp2(x[e + 1] - m_run);
      l_part += p0 + p1;
      const uint32_t u0 = __float_as_uint(p0), u1 = __float_as_uint(p1);
      ph[e / 2] = (u0 >> 16) | (u1 & 0xffff0000u);  // truncated high parts
      pl[e] = (__bf16)(p0 - __uint_as_float(u0 & 0xffff0000u));
      pl[e + 1] = (__bf16)(p1 - __uint_as_float(u1 & 0xffff0000u));
    }

    // ---- O^T += V^T P^T -----------------------------------------------------------------------
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    // ds_read_b64_tr_b16 hands lane 4a+j of a 16-lane group the j-th 16-bit element of the four
    // lanes 4k+a (k = 0..3).  Lane 4k+a points at row 4*jg+k of the tile, head-dim elements
    // 16b+4a .. +3, so lane m receives V[row 4*jg+k][16b+m] for k = 0..3: one half of the A operand.
    const unsigned char* tr0 = myl + (jg * 4 + (n16 >> 2)) * kVStride + (n16 & 3) * 8;
#pragma unroll
    for (int b = 0; b < 8; ++b) {
      typedef __attribute__((address_space(3))) s16x4_t* lds_ptr_t;
      const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(tr0 + b * 32));
      const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(tr0 + 16 * kVStride + b * 32));
      const bf16x8_t a = __builtin_bit_cast(bf16x8_t, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
      o[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, as_bf16x8(ph), o[b], 0, 0, 0);
      o[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, pl, o[b], 0, 0, 0);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
  }
  if (APPLY && ring_n > 0) flush_ring();
  };  // stream_rows
  if (LAG && apply) stream_rows(std::true_type{});
  else stream_rows(std::false_type{});
#undef BAKLAVA_LD
#undef BAKLAVA_LOAD_K
#undef BAKLAVA_LOAD_V
#undef BAKLAVA_LOAD_SC

  // Sum of the four lanes of a head.
  float l_tot = l_part;
  l_tot += __shfl_xor(l_tot, 16);
  l_tot += __shfl_xor(l_tot, 32);

  // Hand the four wavefronts' results over through LDS (reusing the staging area).
  __syncthreads();
  float* sm_o = reinterpret_cast<float*>(lds);                    // [kWaves][16][kD]
  float* sm_m = sm_o + kWaves * 16 * kD;                          // [kWaves][16]
  float* sm_l = sm_m + kWaves * 16;                               // [kWaves][16]
  static_assert((kWaves * 16 * kD + 2 * kWaves * 16) * 4 <= kWaves * kSlab * kVStride, "LDS reuse");
  if (n16 < G) {
#pragma unroll
    for (int b = 0; b < 8; ++b)
#pragma unroll
      for (int i = 0; i < 4; ++i) sm_o[(wave * 16 + n16) * kD + b * 16 + jg * 4 + i] = o[b][i];
    if (jg == 0) {
      sm_m[wave * 16 + n16] = m_run;
      sm_l[wave * 16 + n16] = l_tot;
    }
  }
  __syncthreads();
  finish_item<kD, 16, kWaves>(p, it, G, n, sm_o, sm_m, sm_l);
}

// The recorded calls' weights without an attention call to ride on (baklava_flush_scores, and
// baklava_compact before it ranks rows): a pass over the K rows alone.  Same work items, same
// product and the same weights as in the attention kernel, and the same route for K (whole rows
// from HBM, staged in a wave-private LDS region, one slab ahead) and for the scores (read with the
// slab, new values kept in LDS until the work item is done).
__global__ __launch_bounds__(64 * kWaves) void score_flush_mfma(DecodeParams p) {
  __shared__ __attribute__((aligned(16))) unsigned char lds_k[kWaves * kSlab * kKStride];
  extern __shared__ __attribute__((aligned(16))) float lds_ring[];
  const Item it = p.items[blockIdx.x];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n16 = lane & 15, jg = lane >> 4;
  const int G = p.G;
  const int pending = p.lag_cnt[(int64_t)it.c * G];
  if (pending == 0) return;
  int n_seen = 0;  // rows the latest recorded call saw: no earlier one saw more
  for (int s = 0; s < kRecCalls; ++s)
    if (s < pending) n_seen = max(n_seen, p.lag_n[(int64_t)it.c * kRecCalls + s]);
  const int cnt = min(it.start + it.count, n_seen) - it.start;
  if (cnt <= 0) return;
  Record rec;
  load_record(p, it.c, G, pending, n16, jg, rec);
  const int last = cnt - 1;
  const unsigned char* Kb = reinterpret_cast<const unsigned char*>(p.k) + it.row0 * (kD * 2);
  float* const sc_base = p.score + it.row0;
  unsigned char* myk = lds_k + wave * (kSlab * kKStride);
  float* ring = lds_ring + wave * p.ring_slots * kSlab;
  const float cs = p.scale_log2e;
  const uint32_t v_lane = n16 * 16;
  u32x4_t kr[8];
  float sc_cur = 0.f;
  int ring_n = 0, ring_t0 = 0;
  auto flush_ring = [&]() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    for (int sidx = lane >> 5; sidx < ring_n; sidx += 2) {
      const int r = ring_t0 + sidx * (kWaves * kSlab) + (lane & 31);
      if (r < cnt) sc_base[r] = ring[sidx * kSlab + (lane & 31)];
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    ring_n = 0;
  };
#define BAKLAVA_LOAD_SLAB(T0)                                                                       \
  _Pragma("unroll") for (int i = 0; i < 8; ++i) {                                                   \
    const uint32_t off = (uint32_t)min((T0) + jg + 4 * i, last) * (kD * 2) + v_lane;                \
    kr[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(Kb + off));                 \
  }                                                                                                 \
  if (lane < kSlab) sc_cur = sc_base[min((T0) + lane, last)];
  int t0 = wave * kSlab;
  if (t0 < cnt) {
    BAKLAVA_LOAD_SLAB(t0)
  }
  for (; t0 < cnt; t0 += kWaves * kSlab) {
#pragma unroll
    for (int i = 0; i < 8; ++i) *reinterpret_cast<u32x4_t*>(myk + (jg + 4 * i) * kKStride + n16 * 16) = kr[i];
    const float sc_old = sc_cur;
    BAKLAVA_LOAD_SLAB(t0 + kWaves * kSlab)  // past the end every row clamps to the last one: harmless re-reads
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    floatx4_t sp[kSets][2];
#pragma unroll
    for (int T = 0; T < 2; ++T) {
#pragma unroll
      for (int e = 0; e < kSets; ++e) sp[e][T] = floatx4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const u32x4_t a = *reinterpret_cast<const u32x4_t*>(myk + (T * 16 + n16) * kKStride + c * 64 + jg * 16);
#pragma unroll
        for (int e = 0; e < kSets; ++e)
          sp[e][T] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(rec.q[e][c], as_bf16x8(a), sp[e][T], 0, 0, 0);
      }
    }
    const float wr = record_weights(sp, rec, cs, it.start + t0, lane);
    if (ring_n == 0) ring_t0 = t0;
    if (lane < kSlab) ring[ring_n * kSlab + lane] = sc_old + wr;
    if (++ring_n == p.ring_slots) flush_ring();
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();  // the staging area may be written again
  }
#undef BAKLAVA_LOAD_SLAB
  if (ring_n > 0) flush_ring();
}

}  // namespace

// Dynamic LDS the attention kernel may ask for: the whole LDS of a CU minus the static staging areas
// when a workgroup has the CU to itself, half of what two workgroups leave otherwise.
constexpr int kLdsTotal = 160 * 1024;
constexpr int kStatic = kWaves * kSlab * (kVStride + kKStride);
constexpr int kDynMax = kLdsTotal - kStatic - 512;
constexpr int kDynShared = (kLdsTotal - 2 * kStatic - 1024) / 2;
static_assert(kDynShared >= kWaves * kSlab * 4, "room for one slab of scores per wavefront");

// Called when a context is created on the current device, i.e. outside any stream capture: raises
// the kernel's dynamic-LDS limit once, so that launches (captured or not) only launch.
constexpr int kFlushDynMax = 48 * 1024;  // the flush kernel's share for waiting scores, beside its K staging area
hipError_t prepare_decode_mfma() {
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(decode_partial_mfma<true>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, kDynMax);
  if (e != hipSuccess) return e;
  return hipFuncSetAttribute(reinterpret_cast<const void*>(score_flush_mfma),
                             hipFuncAttributeMaxDynamicSharedMemorySize, kFlushDynMax);
}

// With a pair of events the kernel's own dispatch carries them: they take the time stamps of its
// first and last wavefront, not those of commands placed around it on the stream.
hipError_t launch_decode_mfma(const DecodeParams& p_in, int n_items, int max_count, bool one_wave, hipStream_t s,
                              hipEvent_t ev0, hipEvent_t ev1) {
  if (n_items <= 0) return hipSuccess;
  if (p_in.G > 16) return hipErrorInvalidValue;
  DecodeParams p = p_in;
  p.ring_slots = 0;
  const dim3 grid(n_items), block(64 * kWaves);
  const bool timed = ev0 && ev1;
  if (!p.lag) {
    if (timed) hipExtLaunchKernelGGL(decode_partial_mfma<false>, grid, block, 0, s, ev0, ev1, 0, p);
    else decode_partial_mfma<false><<<grid, block, 0, s>>>(p);
    return hipGetLastError();
  }
  // the LDS left beside the staging areas, split over the wavefronts; a launch of several waves of
  // workgroups keeps room for two workgroups per compute unit
  const int slot_bytes = kSlab * 4;
  const int fit = (one_wave ? kDynMax : kDynShared) / (kWaves * slot_bytes);
  const int need = ((max_count + kSlab - 1) / kSlab + kWaves - 1) / kWaves;  // slabs of the longest item per wavefront
  p.ring_slots = std::max(1, std::min(fit, need));
  const size_t dyn = (size_t)p.ring_slots * kWaves * slot_bytes;
  if (timed) hipExtLaunchKernelGGL(decode_partial_mfma<true>, grid, block, dyn, s, ev0, ev1, 0, p);
  else decode_partial_mfma<true><<<grid, block, dyn, s>>>(p);
  return hipGetLastError();
}

hipError_t launch_score_flush_mfma(const DecodeParams& p_in, int n_items, int max_count, hipStream_t s) {
  if (n_items <= 0) return hipSuccess;
  if (p_in.G > 16) return hipErrorInvalidValue;
  DecodeParams p = p_in;
  const int slot_bytes = kSlab * 4;
  const int fit = kFlushDynMax / (kWaves * slot_bytes);
  const int need = ((max_count + kSlab - 1) / kSlab + kWaves - 1) / kWaves;
  p.ring_slots = std::max(1, std::min(fit, need));
  score_flush_mfma<<<dim3(n_items), dim3(64 * kWaves), (size_t)p.ring_slots * kWaves * slot_bytes, s>>>(p);
  return hipGetLastError();
}

}  // namespace baklava
