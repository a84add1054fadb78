// Attention scores of a whole prompt at once: score_j = sum over the G query heads of a KV head and
// over the prompt tokens t >= j of softmax_j(q_t . k_j / sqrt(D)), i.e. the column sums of the
// causal attention matrices, the accumulated-attention statistic the eviction ranks by, as it
// stands after a prefill of T tokens (before the first decode step and its eviction, Eqs. 5-6).
//
// The row normalisers come from the attention pass that produced the prompt's outputs (its
// log-sum-exp per token, here in log2 units), so this pass needs the first product only:
//
//   S^T[key, token] = K[key, :] . Q[token, :]     A = K rows (registers, fixed per wavefront),
//                                                 B = Q rows (streamed through LDS)
//   score[key]     += 2^(S^T[key, token] * log2(e)/sqrt(D) - lse2[token])   for key <= token
//
// A workgroup of 4 wavefronts owns 128 consecutive keys of one KV head, 32 per wavefront, and walks
// over the G query heads and, for each, over the tokens from its first key to the end of the
// prompt in tiles of 64, double-buffered in LDS.  Column sums stay in registers (one partial per
// lane and key) and are reduced over the 16 token lanes once, at the end: no atomics, results are
// deterministic.  Key block i streams T - 128 i tokens, so a workgroup takes blocks i and
// n_blocks - 1 - i: equal work for every workgroup of a sequence.
#include "common.h"

namespace baklava {

namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float floatx4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

constexpr int kD = 128;
constexpr int kWaves = 4;
constexpr int kKeysPerWave = 32;
constexpr int kKeysPerWg = kWaves * kKeysPerWave;  // 128
constexpr int kTokTile = 64;                       // tokens per LDS stage
constexpr int kQStride = 272;                      // bytes between staged Q rows (conflict-free operand reads)
constexpr float kNegInf = -__builtin_huge_valf();

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ bf16x8_t as_bf16x8(u32x4_t x) { return __builtin_bit_cast(bf16x8_t, x); }

struct PrefillParams {
  const unsigned char* q;    // [batch, Hq, T, D] bf16
  const unsigned char* k;    // K plane; sequence (b, h) starts at row k_off[b * Hkv + h], or is dense
  const float* lse;          // [batch, Hq, T] log2-sum-exp of the scaled logits, log2 units
  const int64_t* row_off;    // [batch * Hkv] or null
  float* score;              // same row addressing as k
  int32_t T, Hq, Hkv, n_blocks;
  float scale_log2e;
};

__global__ __launch_bounds__(256) void prefill_score_kernel(PrefillParams p) {
  __shared__ __attribute__((aligned(16))) unsigned char lds_q[2][kTokTile * kQStride];
  __shared__ float lds_lse[2][kTokTile];

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int n16 = lane & 15, jg = lane >> 4;
  const int T = p.T;
  const int n_pairs = (p.n_blocks + 1) / 2;
  const int n_seq = gridDim.x / n_pairs;      // batch * Hkv
  const int seq = blockIdx.x % n_seq;         // (b, kv head)
  const int pair = blockIdx.x / n_seq;
  const int G = p.Hq / p.Hkv;
  const int b = seq / p.Hkv, hk = seq % p.Hkv;
  const int64_t row0 = p.row_off ? p.row_off[seq] : (int64_t)seq * T;
  const unsigned char* Kb = p.k + row0 * (kD * 2);

  const float cs = p.scale_log2e;
  // Key block i sees T - 128 i tokens: the workgroup takes blocks i and n_blocks - 1 - i, one after
  // the other, so that every workgroup of a sequence streams (about) the same number of tokens.
  for (int half = 0; half < 2; ++half) {
  const int block = half == 0 ? pair : p.n_blocks - 1 - pair;
  if (half == 1 && block == pair) break;      // odd number of blocks: the middle one is alone
  const int j0 = block * kKeysPerWg;          // first key of the block
  const int jw0 = j0 + wave * kKeysPerWave;   // first key of this wavefront

  // A operand: lane (key % 16, j), 16-key tile tt, chunk c holds K[key][32c + 8j .. +8); loaded once.
  bf16x8_t ka[2][4];
#pragma unroll
  for (int tt = 0; tt < 2; ++tt) {
    const int row = min(jw0 + tt * 16 + n16, T - 1);  // keys past the prompt repeat the last one, never written
#pragma unroll
    for (int c = 0; c < 4; ++c)
      ka[tt][c] = as_bf16x8(*reinterpret_cast<const u32x4_t*>(Kb + (int64_t)row * (kD * 2) + c * 64 + jg * 16));
  }

  float acc[8];  // column-sum partials of keys jw0 + 16 tt + 4 jg + i (e = 4 tt + i), over this lane's tokens
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] = 0.f;

  // Stages: for each query head of the group, the token tiles from the one holding key j0 to the end.
  const int first_tile = j0 / kTokTile;
  const int n_tiles = (T + kTokTile - 1) / kTokTile - first_tile;
  const int n_stages = G * n_tiles;

  u32x4_t qreg[4];
  float lreg = 0.f;
  auto load_stage = [&](int st) {
    const int g = st / n_tiles, t0 = (first_tile + st % n_tiles) * kTokTile;
    const int64_t head = (int64_t)b * p.Hq + (int64_t)hk * G + g;
    const unsigned char* Qh = p.q + head * T * (kD * 2);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int idx = tid + i * 256;
      const int row = min(t0 + idx / 16, T - 1), piece = idx % 16;
      qreg[i] = *reinterpret_cast<const u32x4_t*>(Qh + (int64_t)row * (kD * 2) + piece * 16);
    }
    if (tid < kTokTile) lreg = p.lse[head * T + min(t0 + tid, T - 1)];
  };
  auto store_stage = [&](int buf) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int idx = tid + i * 256;
      *reinterpret_cast<u32x4_t*>(&lds_q[buf][(idx / 16) * kQStride + (idx % 16) * 16]) = qreg[i];
    }
    if (tid < kTokTile) lds_lse[buf][tid] = lreg;
  };

  load_stage(0);
  store_stage(0);
  __syncthreads();

  for (int st = 0; st < n_stages; ++st) {
    const int buf = st & 1;
    const bool more = st + 1 < n_stages;
    if (more) load_stage(st + 1);
    const int t0 = (first_tile + st % n_tiles) * kTokTile;

#pragma unroll
    for (int nt = 0; nt < 4; ++nt) {
      const int tn0 = t0 + nt * 16;         // first token of the column tile
      if (tn0 + 15 < jw0) continue;         // every token precedes every key of this wavefront (uniform)
      floatx4_t s[2];
      s[0] = floatx4_t{0.f, 0.f, 0.f, 0.f};
      s[1] = floatx4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const bf16x8_t qb = as_bf16x8(
            *reinterpret_cast<const u32x4_t*>(&lds_q[buf][(nt * 16 + n16) * kQStride + c * 64 + jg * 16]));
        s[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[0][c], qb, s[0], 0, 0, 0);
        s[1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[1][c], qb, s[1], 0, 0, 0);
      }
      // lane (token, j) holds keys 4j..4j+3 of each 16-key tile
      const int tok = tn0 + n16;
      const float nl = -lds_lse[buf][nt * 16 + n16];
      const bool edge = tn0 < jw0 + kKeysPerWave - 1 || tn0 + 15 >= T;  // some pair is masked, or a token is past the prompt
      if (edge) {
        asm volatile("" ::: "memory");  // keeps this a branch: below the diagonal nothing is masked
#pragma unroll
        for (int tt = 0; tt < 2; ++tt)
#pragma unroll
          for (int i = 0; i < 4; ++i)
            if (jw0 + tt * 16 + jg * 4 + i > tok || tok >= T) s[tt][i] = kNegInf;
      }
#pragma unroll
      for (int tt = 0; tt < 2; ++tt)
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[tt * 4 + i] += fast_exp2(fmaf(s[tt][i], cs, nl));
    }

    if (more) store_stage(buf ^ 1);  // last read in the previous iteration, before its closing barrier
    __syncthreads();
  }

  // sum over the 16 token lanes of each j group, then lanes with token index 0 write their 8 keys
#pragma unroll
  for (int e = 0; e < 8; ++e) {
#pragma unroll
    for (int off = 8; off > 0; off >>= 1) acc[e] += __shfl_xor(acc[e], off);
  }
  if (n16 == 0) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int key = jw0 + (e / 4) * 16 + jg * 4 + (e % 4);
      if (key < T) p.score[row0 + key] = acc[e];
    }
  }
  }
}

}  // namespace

hipError_t launch_prefill_scores(const void* q, const void* k, const float* lse, const int64_t* row_off,
                                 int batch, int Hq, int Hkv, int T, float* score, hipStream_t s) {
  PrefillParams p;
  p.q = reinterpret_cast<const unsigned char*>(q);
  p.k = reinterpret_cast<const unsigned char*>(k);
  p.lse = lse;
  p.row_off = row_off;
  p.score = score;
  p.T = T; p.Hq = Hq; p.Hkv = Hkv;
  p.n_blocks = (T + kKeysPerWg - 1) / kKeysPerWg;
  p.scale_log2e = 1.4426950408889634f / sqrtf((float)kD);
  const int64_t n_wg = (int64_t)batch * Hkv * ((p.n_blocks + 1) / 2);
  if (n_wg <= 0 || n_wg > INT32_MAX) return hipErrorInvalidValue;
  prefill_score_kernel<<<dim3((unsigned)n_wg), dim3(256), 0, s>>>(p);
  return hipGetLastError();
}

}  // namespace baklava
