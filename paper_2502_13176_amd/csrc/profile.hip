// One-time profiling (Algorithm 1, step 1): for every attention head of a prompt, causal attention
// over the prompt fused with the token-wise cosine between the head's input row v_t and its output
// row softmax(q_t K^T / sqrt(D)) V, and the mean of those cosines.
//
// A dense contraction (2 D T (T + 1) flops per head), so it runs on the matrix cores.  The tiling
// is the decode kernel's, with 16 prompt tokens where that kernel has the query heads of a group:
//
//   S^T[key, token]  = K[key, :] . Q[token, :]          A = K rows from LDS, B = Q (registers)
//   O^T[d, token]   += V^T[d, keys] . P^T[keys, token]   A = V^T (LDS, transposed read), B = P^T
//
// A workgroup of 4 wavefronts owns 128 consecutive tokens of one head, 32 per wavefront (two
// 16-token column tiles that share every A operand read from LDS).  Keys and values arrive in
// tiles of 64 rows, loaded by the whole workgroup and double-buffered in LDS; a wavefront skips
// the key tiles that lie entirely above its tokens (causal mask) and masks the others
// element-wise.  The softmax normaliser cancels in the cosine, so the output is never divided.
#include "common.h"

namespace baklava {

namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float floatx4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
typedef short s16x4_t __attribute__((ext_vector_type(4)));

constexpr int kD = 128;
constexpr int kWaves = 4;
constexpr int kTokPerWave = 32;                    // two column tiles of 16
constexpr int kTokPerWg = kWaves * kTokPerWave;    // 128
constexpr int kKeyTile = 64;                       // rows per LDS stage
constexpr int kKStride = 272;                      // as in the decode kernel: conflict-free operand reads
constexpr int kVStride = 288;
constexpr float kNegInf = -__builtin_huge_valf();
constexpr float kMaxSlack = 8.f;                   // a logit may exceed its token's reference maximum by this much
constexpr float kCosEps = 1e-8f;                   // lower clamp of the product of the two norms

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ bf16x8_t as_bf16x8(u32x4_t x) { return __builtin_bit_cast(bf16x8_t, x); }

struct ProfileParams {
  const unsigned char* q;  // [batch, Hq, T, D] bf16
  const unsigned char* k;  // [batch, Hkv, T, D]
  const unsigned char* v;
  float* cos_out;          // [batch, Hq, T] or null
  float* lse_out;          // [batch, Hq, T] or null: log2 of the sum over visible keys of 2^(scaled logit)
  float* tile_sum;         // [batch * Hq, n_tiles] sum of the cosines of each 128-token tile
  int32_t T, Hq, Hkv, n_tiles;
  float scale_log2e;
};

__global__ __launch_bounds__(256, 2) void profile_attn_kernel(ProfileParams p) {
  __shared__ __attribute__((aligned(16))) unsigned char lds_k[2][kKeyTile * kKStride];
  __shared__ __attribute__((aligned(16))) unsigned char lds_v[2][kKeyTile * kVStride];
  __shared__ float wave_sum[kWaves];

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int n16 = lane & 15, jg = lane >> 4;
  const int T = p.T;
  // heaviest tiles (the last tokens of the prompt) are launched first
  const int bh = blockIdx.x % (gridDim.x / p.n_tiles);
  const int tile = p.n_tiles - 1 - blockIdx.x / (gridDim.x / p.n_tiles);
  const int G = p.Hq / p.Hkv;
  const int b = bh / p.Hq, h = bh % p.Hq;
  const int64_t kv_head = (int64_t)b * p.Hkv + h / G;
  const unsigned char* Qb = p.q + (int64_t)bh * T * (kD * 2);
  const unsigned char* Kb = p.k + kv_head * T * (kD * 2);
  const unsigned char* Vb = p.v + kv_head * T * (kD * 2);

  const int q0 = tile * kTokPerWg;          // first token of the workgroup
  const int qw0 = q0 + wave * kTokPerWave;  // first token of this wavefront
  const int last_tok = min(q0 + kTokPerWg, T) - 1;
  const int n_key_tiles = last_tok / kKeyTile + 1;

  // B operand of the first product: lane (token, j), chunk c holds Q[token][32c + 8j .. +8).
  bf16x8_t qb[2][4];
  int tok[2];
#pragma unroll
  for (int nt = 0; nt < 2; ++nt) {
    tok[nt] = qw0 + nt * 16 + n16;
    const int row = min(tok[nt], T - 1);  // tokens past the prompt repeat the last one and are never written
#pragma unroll
    for (int c = 0; c < 4; ++c)
      qb[nt][c] = as_bf16x8(*reinterpret_cast<const u32x4_t*>(Qb + (int64_t)row * (kD * 2) + c * 64 + jg * 16));
  }

  floatx4_t o[2][8];
#pragma unroll
  for (int nt = 0; nt < 2; ++nt)
#pragma unroll
    for (int bb = 0; bb < 8; ++bb) o[nt][bb] = floatx4_t{0.f, 0.f, 0.f, 0.f};
  float m_ref[2] = {kNegInf, kNegInf};  // reference maximum of the exponent, log2 units
  float l_part[2] = {0.f, 0.f};
  const float cs = p.scale_log2e;

  // Cooperative tile load: 64 rows x 16 pieces of 16 bytes per plane, 4 pieces per thread and plane.
  u32x4_t kreg[4], vreg[4];
  auto load_tile = [&](int kt) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int idx = tid + i * 256;
      const int row = min(kt * kKeyTile + idx / 16, T - 1), piece = idx % 16;
      kreg[i] = *reinterpret_cast<const u32x4_t*>(Kb + (int64_t)row * (kD * 2) + piece * 16);
      vreg[i] = *reinterpret_cast<const u32x4_t*>(Vb + (int64_t)row * (kD * 2) + piece * 16);
    }
  };
  auto store_tile = [&](int buf) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int idx = tid + i * 256;
      const int row = idx / 16, piece = idx % 16;
      *reinterpret_cast<u32x4_t*>(&lds_k[buf][row * kKStride + piece * 16]) = kreg[i];
      *reinterpret_cast<u32x4_t*>(&lds_v[buf][row * kVStride + piece * 16]) = vreg[i];
    }
  };

  load_tile(0);
  store_tile(0);
  __syncthreads();

  for (int kt = 0; kt < n_key_tiles; ++kt) {
    const int buf = kt & 1;
    const bool more = kt + 1 < n_key_tiles;
    if (more) load_tile(kt + 1);

    const int kt0 = kt * kKeyTile;        // first key of the tile
    if (kt0 <= qw0 + kTokPerWave - 1) {   // else wholly above this wavefront's tokens (uniform per wavefront)
      // ---- S^T = K Q^T for the tile's two 32-key slabs and both column tiles; every K operand is
      //      read once.  A slab that is wholly masked for this wavefront (diagonal tile only) is
      //      computed and masked like any other.
      floatx4_t s[2][2][2];  // [slab][column tile][16-key tile]
      // The 16 K operands of the tile (slab, 16-key tile, 32-element chunk) are read four ahead of
      // their use, so that the matrix instructions do not wait for LDS.
      const unsigned char* kbase = &lds_k[buf][n16 * kKStride + jg * 16];
      u32x4_t ka[4];
#pragma unroll
      for (int i = 0; i < 4; ++i)
        ka[i] = *reinterpret_cast<const u32x4_t*>(kbase + (i / 4) * 16 * kKStride + (i % 4) * 64);
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int sl = i / 8, tt = (i / 4) % 2, c = i % 4;
        if (c == 0) {
          s[sl][0][tt] = floatx4_t{0.f, 0.f, 0.f, 0.f};
          s[sl][1][tt] = floatx4_t{0.f, 0.f, 0.f, 0.f};
        }
        const bf16x8_t a = as_bf16x8(ka[i % 4]);
        s[sl][0][tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, qb[0][c], s[sl][0][tt], 0, 0, 0);
        s[sl][1][tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, qb[1][c], s[sl][1][tt], 0, 0, 0);
        if (i + 4 < 16)
          ka[i % 4] = *reinterpret_cast<const u32x4_t*>(kbase + ((i + 4) / 4) * 16 * kKStride + ((i + 4) % 4) * 64);
      }

      // ---- causal mask (lane (token, j): keys 4j..4j+3 of each 16-key tile), raw maxima ----------
      if (kt0 + kKeyTile - 1 > qw0) {  // some (key, token) pair of the tile is masked
        // (the empty statement keeps this a real, wavefront-uniform branch: turned into selects it
        // would run, and cost a quarter of the vector instructions, on every tile below the diagonal)
        asm volatile("" ::: "memory");
#pragma unroll
        for (int sl = 0; sl < 2; ++sl)
#pragma unroll
          for (int nt = 0; nt < 2; ++nt)
#pragma unroll
            for (int tt = 0; tt < 2; ++tt)
#pragma unroll
              for (int i = 0; i < 4; ++i)
                if (kt0 + sl * 32 + tt * 16 + jg * 4 + i > tok[nt]) s[sl][nt][tt][i] = kNegInf;
      }
      float mx[2];
#pragma unroll
      for (int nt = 0; nt < 2; ++nt) {
        mx[nt] = kNegInf;
#pragma unroll
        for (int sl = 0; sl < 2; ++sl)
#pragma unroll
          for (int tt = 0; tt < 2; ++tt)
#pragma unroll
            for (int i = 0; i < 4; ++i) mx[nt] = fmaxf(mx[nt], s[sl][nt][tt][i]);
        mx[nt] *= cs;
      }
      // Lazy running maximum: the reference m_ref of a token only moves when a logit exceeds it by
      // more than kMaxSlack (log2 units), so weights stay below 2^kMaxSlack and the rescale of the
      // accumulators is rare after the first tile.  (First tile: m_ref = -inf, always taken; key 0
      // is visible to every token, so the new reference is finite.)
      if (__any(mx[0] > m_ref[0] + kMaxSlack) || __any(mx[1] > m_ref[1] + kMaxSlack)) {
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) {
          float m = mx[nt];
          m = fmaxf(m, __shfl_xor(m, 16));
          m = fmaxf(m, __shfl_xor(m, 32));
          const float mn = fmaxf(m_ref[nt], m);
          const float alpha = fast_exp2(m_ref[nt] - mn);
          m_ref[nt] = mn;
          l_part[nt] *= alpha;
#pragma unroll
          for (int bb = 0; bb < 8; ++bb) o[nt][bb] *= alpha;
        }
      }

      // ---- weights and O^T += V^T P^T, slab by slab, in one basic block so that the vector work
      //      of one slab can be scheduled between the matrix instructions of the other -----------
      const float nm0 = -m_ref[0], nm1 = -m_ref[1];
#pragma unroll
      for (int sl = 0; sl < 2; ++sl) {
        // The slab's 16 transposed V operands are fetched before the weights are formed, so that the
        // LDS latency hides behind the exponentials; every operand serves both column tiles.
        const unsigned char* tr0 = &lds_v[buf][(sl * 32 + jg * 4 + (n16 >> 2)) * kVStride + (n16 & 3) * 8];
        bf16x8_t va[8];
#pragma unroll
        for (int bb = 0; bb < 8; ++bb) {
          typedef __attribute__((address_space(3))) s16x4_t* lds_ptr_t;
          const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(tr0 + bb * 32));
          const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(tr0 + 16 * kVStride + bb * 32));
          va[bb] = __builtin_bit_cast(bf16x8_t, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
        }
        // each weight is split into a truncated bf16 high part and a bf16 residual, so the second
        // product keeps ~16 bits of it (one bf16 term alone costs about 1e-3 on a token's cosine)
        u32x4_t ph[2];
        bf16x8_t pl[2];
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) {
          const float nm = nt ? nm1 : nm0;
#pragma unroll
          for (int e = 0; e < 8; e += 2) {
            const float p0 = fast_exp2(fmaf(s[sl][nt][e / 4][e % 4], cs, nm));
            const float p1 = fast_exp2(fmaf(s[sl][nt][e / 4][e % 4 + 1], cs, nm));
            l_part[nt] += p0 + p1;
            const uint32_t u0 = __float_as_uint(p0), u1 = __float_as_uint(p1);
            ph[nt][e / 2] = (u0 >> 16) | (u1 & 0xffff0000u);
            pl[nt][e] = (__bf16)(p0 - __uint_as_float(u0 & 0xffff0000u));
            pl[nt][e + 1] = (__bf16)(p1 - __uint_as_float(u1 & 0xffff0000u));
          }
        }
#pragma unroll
        for (int bb = 0; bb < 8; ++bb) {
          o[0][bb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va[bb], as_bf16x8(ph[0]), o[0][bb], 0, 0, 0);
          o[1][bb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va[bb], as_bf16x8(ph[1]), o[1][bb], 0, 0, 0);
          o[0][bb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va[bb], pl[0], o[0][bb], 0, 0, 0);
          o[1][bb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va[bb], pl[1], o[1][bb], 0, 0, 0);
        }
      }
    }

    if (more) store_tile(buf ^ 1);  // last read in the previous iteration, before its closing barrier
    __syncthreads();
  }

  // ---- cosine between v_t and the (un-normalised) output row, per token --------------------------
  // Lane (token, j) holds O[token][16 bb + 4 j + i].
  float wsum = 0.f;
#pragma unroll
  for (int nt = 0; nt < 2; ++nt) {
    float l_tot = l_part[nt];
    l_tot += __shfl_xor(l_tot, 16);
    l_tot += __shfl_xor(l_tot, 32);
    const int row = min(tok[nt], T - 1);
    float dot = 0.f, no = 0.f, nv = 0.f;
#pragma unroll
    for (int bb = 0; bb < 8; ++bb) {
      const u32x2_t raw = *reinterpret_cast<const u32x2_t*>(Vb + (int64_t)row * (kD * 2) + (bb * 16 + jg * 4) * 2);
      const float v0 = __uint_as_float(raw.x << 16), v1 = __uint_as_float(raw.x & 0xffff0000u);
      const float v2 = __uint_as_float(raw.y << 16), v3 = __uint_as_float(raw.y & 0xffff0000u);
      const floatx4_t ov = o[nt][bb];
      dot += ov[0] * v0 + ov[1] * v1 + ov[2] * v2 + ov[3] * v3;
      no += ov[0] * ov[0] + ov[1] * ov[1] + ov[2] * ov[2] + ov[3] * ov[3];
      nv += v0 * v0 + v1 * v1 + v2 * v2 + v3 * v3;
    }
    dot += __shfl_xor(dot, 16); dot += __shfl_xor(dot, 32);
    no += __shfl_xor(no, 16);   no += __shfl_xor(no, 32);
    nv += __shfl_xor(nv, 16);   nv += __shfl_xor(nv, 32);
    const float inv_l = 1.f / l_tot;
    const float cosv = (dot * inv_l) / fmaxf(sqrtf(no) * inv_l * sqrtf(nv), kCosEps);
    const bool live = tok[nt] < T && jg == 0;
    if (live) {
      if (p.cos_out) p.cos_out[(int64_t)bh * T + tok[nt]] = cosv;
      if (p.lse_out) p.lse_out[(int64_t)bh * T + tok[nt]] = m_ref[nt] + __builtin_log2f(l_tot);
      wsum += cosv;
    }
  }
  // sum over the wavefront's tokens (lanes with j = 0 hold them), then over the workgroup, in a fixed order
#pragma unroll
  for (int off = 8; off > 0; off >>= 1) wsum += __shfl_xor(wsum, off);
  if (lane == 0) wave_sum[wave] = wsum;
  __syncthreads();
  if (tid == 0)
    p.tile_sum[(int64_t)bh * p.n_tiles + tile] = (wave_sum[0] + wave_sum[1]) + (wave_sum[2] + wave_sum[3]);
}

// Mean over the prompt: one wavefront per head adds the tile sums in a fixed order.
__global__ __launch_bounds__(64) void profile_mean_kernel(const float* tile_sum, float* sim_out, int n_tiles, int T) {
  const int bh = blockIdx.x;
  float acc = 0.f;
  for (int i = threadIdx.x; i < n_tiles; i += 64) acc += tile_sum[(int64_t)bh * n_tiles + i];
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off);
  if (threadIdx.x == 0) sim_out[bh] = acc / (float)T;
}

}  // namespace

hipError_t launch_profile_similarity(const void* q, const void* k, const void* v, int batch, int Hq, int Hkv,
                                     int T, float* cos_out, float* sim_out, float* lse_out, float* tile_sum,
                                     hipStream_t s) {
  ProfileParams p;
  p.q = reinterpret_cast<const unsigned char*>(q);
  p.k = reinterpret_cast<const unsigned char*>(k);
  p.v = reinterpret_cast<const unsigned char*>(v);
  p.cos_out = cos_out;
  p.lse_out = lse_out;
  p.tile_sum = tile_sum;
  p.T = T; p.Hq = Hq; p.Hkv = Hkv;
  p.n_tiles = (T + kTokPerWg - 1) / kTokPerWg;
  p.scale_log2e = 1.4426950408889634f / sqrtf((float)kD);
  const int64_t n_wg = (int64_t)batch * Hq * p.n_tiles;
  if (n_wg <= 0 || n_wg > INT32_MAX) return hipErrorInvalidValue;
  profile_attn_kernel<<<dim3((unsigned)n_wg), dim3(256), 0, s>>>(p);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  profile_mean_kernel<<<dim3(batch * Hq), dim3(64), 0, s>>>(tile_sum, sim_out, p.n_tiles, T);
  return hipGetLastError();
}

}  // namespace baklava
