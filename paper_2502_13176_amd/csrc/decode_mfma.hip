// Decode attention over ragged caches, MFMA version (bf16, D = 128, up to 16 query heads per
// KV head).
//
// The G query heads that share a KV head form the N side (padded to 16) of two matrix products
// per 32-row slab, both issued as v_mfma_f32_16x16x32_bf16:
//
//   S^T[row, g]  = K[row, :] . Q[g, :]          A = K rows (read straight from HBM into the
//                                               A-operand layout: lane (row%16, j) holds 8
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
// Each of the 4 wavefronts of a workgroup streams its own 32-row slabs and owns a private LDS
// region: there is no barrier inside the loop.
#include "common.h"

namespace baklava {

namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float floatx4_t __attribute__((ext_vector_type(4)));

constexpr int kWaves = 4;
constexpr int kSlab = 32;       // rows per wavefront iteration
constexpr int kVStride = 264;   // bytes between staged V rows: 66 dwords, so the 4 row groups of a
                                // transposed read fall into disjoint LDS banks
constexpr int kD = 128;
constexpr float kNegInf = -__builtin_huge_valf();

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

union Frag {
  uint4 u;
  bf16x8_t v;
  uint32_t w[4];
  uint16_t h[8];
};

__global__ __launch_bounds__(256) void decode_partial_mfma(DecodeParams p) {
  __shared__ __attribute__((aligned(16))) unsigned char lds[kWaves * kSlab * kVStride];

  const Item it = p.items[blockIdx.x];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n16 = lane & 15, jg = lane >> 4;
  const int G = p.G;
  const int n = p.len[it.c];
  int cnt = min(it.start + it.count, n) - it.start;
  if (cnt < 0) cnt = 0;
  const int64_t row0 = p.off[it.c] + it.start;
  const unsigned char* Kb = reinterpret_cast<const unsigned char*>(p.k) + row0 * (kD * 2);
  const unsigned char* Vb = reinterpret_cast<const unsigned char*>(p.v) + row0 * (kD * 2);
  unsigned char* myl = lds + wave * (kSlab * kVStride);

  const int c_rel = it.c - p.cache_begin;
  const int64_t qrow0 = (int64_t)(c_rel / p.Hkv) * p.Hq + (int64_t)(c_rel % p.Hkv) * G;

  // B operand of the first product: lane (g, j), chunk c holds Q[g][32c + 8j .. +8).
  Frag qb[4];
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    if (n16 < G)
      qb[c].u = *reinterpret_cast<const uint4*>(reinterpret_cast<const unsigned char*>(p.q) +
                                                (qrow0 + n16) * (kD * 2) + c * 64 + jg * 16);
    else
      qb[c].u = make_uint4(0, 0, 0, 0);
  }

  floatx4_t o[8];
#pragma unroll
  for (int b = 0; b < 8; ++b) o[b] = floatx4_t{0.f, 0.f, 0.f, 0.f};
  float m_run = kNegInf;  // running max of head n16, log2 units, equal in the 4 lanes of a head
  float l_part = 0.f;     // this lane's share of the running sum
  const float cs = p.scale_log2e;

  for (int t0 = wave * kSlab; t0 < cnt; t0 += kWaves * kSlab) {
    // ---- loads: K straight into the A layout, V in whole rows (fully coalesced) -------------
    Frag kr[2][4];
#pragma unroll
    for (int T = 0; T < 2; ++T) {
      const int r = min(t0 + T * 16 + n16, cnt - 1);
#pragma unroll
      for (int c = 0; c < 4; ++c)
        kr[T][c].u = *reinterpret_cast<const uint4*>(Kb + (int64_t)r * (kD * 2) + c * 64 + jg * 16);
    }
    uint4 vr[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int r = min(t0 + jg + 4 * i, cnt - 1);
      vr[i] = *reinterpret_cast<const uint4*>(Vb + (int64_t)r * (kD * 2) + n16 * 16);
    }

    // ---- S^T = K Q^T --------------------------------------------------------------------------
    floatx4_t s[2];
#pragma unroll
    for (int T = 0; T < 2; ++T) {
      s[T] = floatx4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int c = 0; c < 4; ++c)
        s[T] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kr[T][c].v, qb[c].v, s[T], 0, 0, 0);
    }

    // ---- stage V rows in LDS ------------------------------------------------------------------
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      unsigned char* dst = myl + (jg + 4 * i) * kVStride + n16 * 16;
      *reinterpret_cast<uint2*>(dst) = make_uint2(vr[i].x, vr[i].y);
      *reinterpret_cast<uint2*>(dst + 8) = make_uint2(vr[i].z, vr[i].w);
    }

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
    if (p.track && n16 < G) {
#pragma unroll
      for (int T = 0; T < 2; ++T)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int r = t0 + T * 16 + jg * 4 + i;
          if (r < cnt) p.logits[(row0 + r) * G + n16] = x[T * 4 + i];
        }
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
    Frag ph, pl;
#pragma unroll
    for (int e = 0; e < 8; e += 2) {
      const float p0 = fast_exp2(x[e] - m_run), p1 = fast_exp2(x[e + 1] - m_run);
      l_part += p0 + p1;
      const uint32_t u0 = __float_as_uint(p0), u1 = __float_as_uint(p1);
      ph.w[e / 2] = (u0 >> 16) | (u1 & 0xffff0000u);  // truncated high parts
      const float r0 = p0 - __uint_as_float(u0 & 0xffff0000u);
      const float r1 = p1 - __uint_as_float(u1 & 0xffff0000u);
      pl.v[e] = (__bf16)r0;
      pl.v[e + 1] = (__bf16)r1;
    }

    // ---- O^T += V^T P^T -----------------------------------------------------------------------
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
    for (int b = 0; b < 8; ++b) {
      Frag a;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int row = (e / 4) * 16 + jg * 4 + (e % 4);
        a.h[e] = *reinterpret_cast<const uint16_t*>(myl + row * kVStride + (b * 16 + n16) * 2);
      }
      o[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.v, ph.v, o[b], 0, 0, 0);
      o[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.v, pl.v, o[b], 0, 0, 0);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
  }

  // Sum of the four lanes of a head.
  float l_tot = l_part;
  l_tot += __shfl_xor(l_tot, 16);
  l_tot += __shfl_xor(l_tot, 32);

  // Merge the four wavefronts through LDS (reusing the staging area) and write the partial.
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
  for (int idx = threadIdx.x; idx < G * kD; idx += 256) {
    const int g = idx / kD, d = idx % kD;
    float mm = sm_m[g];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) mm = fmaxf(mm, sm_m[w * 16 + g]);
    const float ms = (mm == kNegInf) ? 0.f : mm;
    float ll = 0.f, oo = 0.f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      const float a = fast_exp2(sm_m[w * 16 + g] - ms);
      ll += sm_l[w * 16 + g] * a;
      oo += sm_o[(w * 16 + g) * kD + d] * a;
    }
    p.part_o[((int64_t)it.slot * G + g) * kD + d] = oo;
    if (d == 0) {
      p.part_ml[((int64_t)it.slot * G + g) * 2 + 0] = mm;
      p.part_ml[((int64_t)it.slot * G + g) * 2 + 1] = ll;
    }
  }
}

}  // namespace

hipError_t launch_decode_mfma(const DecodeParams& p, int n_items, hipStream_t s) {
  if (n_items <= 0) return hipSuccess;
  if (p.G > 16) return hipErrorInvalidValue;
  decode_partial_mfma<<<dim3(n_items), dim3(256), 0, s>>>(p);
  return hipGetLastError();
}

}  // namespace baklava
