// Layer importance heuristic ("Layer Importance Heuristic"): the cosine between the input and the
// output hidden state of a layer, token by token, and its mean over the prompt.
//
// HBM-bound: every hidden-state row is read once (2 * hidden * 2 bytes per token for bf16).  One
// wavefront per token row: 64 lanes x 16 bytes per load instruction, all loads of a row pair in
// flight before the first use, non-temporal (read once); three dot products per row reduced over
// the wavefront.  A workgroup takes 16 consecutive rows and writes the sum of their cosines; a
// second small kernel adds the workgroup sums in a fixed order (deterministic, no atomics).
#include <mutex>

#include "baklava.h"
#include "common.h"

namespace baklava {

constexpr int kRowsPerWg = 16;

namespace {

constexpr int kWaves = 4;
constexpr float kCosEps = 1e-8f;

struct LayerParams {
  const unsigned char* x_in;   // [n_seq, T, hidden] bf16
  const unsigned char* x_out;
  float* cos_out;              // [n_seq, T] or null
  float* tile_sum;             // [n_seq, n_tiles]
  int32_t T, hidden, n_tiles;
};

__device__ __forceinline__ void accumulate(uint4 a, uint4 b, float& dot, float& na, float& nb) {
  const uint32_t aw[4] = {a.x, a.y, a.z, a.w}, bw[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const float a0 = __uint_as_float(aw[i] << 16), a1 = __uint_as_float(aw[i] & 0xffff0000u);
    const float b0 = __uint_as_float(bw[i] << 16), b1 = __uint_as_float(bw[i] & 0xffff0000u);
    dot = fmaf(a0, b0, dot); dot = fmaf(a1, b1, dot);
    na = fmaf(a0, a0, na);   na = fmaf(a1, a1, na);
    nb = fmaf(b0, b0, nb);   nb = fmaf(b1, b1, nb);
  }
}

__global__ __launch_bounds__(256) void layer_cosine_kernel(LayerParams p) {
  __shared__ float wave_sum[kWaves];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int seq = blockIdx.x / p.n_tiles, tile = blockIdx.x % p.n_tiles;
  const int64_t row_bytes = (int64_t)p.hidden * 2;
  float wsum = 0.f;
  for (int r = wave; r < kRowsPerWg; r += kWaves) {
    const int t = tile * kRowsPerWg + r;
    if (t >= p.T) break;  // uniform per wavefront
    const unsigned char* a = p.x_in + ((int64_t)seq * p.T + t) * row_bytes;
    const unsigned char* b = p.x_out + ((int64_t)seq * p.T + t) * row_bytes;
    float dot = 0.f, na = 0.f, nb = 0.f;
    // 8 pieces of 1 KiB per tensor in flight per wavefront (a 4096-wide row is one pass)
    for (int64_t h0 = (int64_t)lane * 16; h0 < row_bytes; h0 += 8 * 1024) {
      uint4 av[8], bv[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int64_t o = h0 + u * 1024;
        av[u] = make_uint4(0, 0, 0, 0);
        bv[u] = make_uint4(0, 0, 0, 0);
        if (o < row_bytes) { av[u] = load_nt16(a + o); bv[u] = load_nt16(b + o); }
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) accumulate(av[u], bv[u], dot, na, nb);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
      dot += __shfl_xor(dot, off);
      na += __shfl_xor(na, off);
      nb += __shfl_xor(nb, off);
    }
    const float c = dot / fmaxf(sqrtf(na) * sqrtf(nb), kCosEps);
    if (lane == 0 && p.cos_out) p.cos_out[(int64_t)seq * p.T + t] = c;
    wsum += c;
  }
  if (lane == 0) wave_sum[wave] = wsum;
  __syncthreads();
  if (threadIdx.x == 0)
    p.tile_sum[(int64_t)seq * p.n_tiles + tile] = (wave_sum[0] + wave_sum[1]) + (wave_sum[2] + wave_sum[3]);
}

__global__ __launch_bounds__(64) void layer_mean_kernel(const float* tile_sum, float* sim_out, int n_tiles, int T) {
  const int seq = blockIdx.x;
  float acc = 0.f;
  for (int i = threadIdx.x; i < n_tiles; i += 64) acc += tile_sum[(int64_t)seq * n_tiles + i];
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off);
  if (threadIdx.x == 0) sim_out[seq] = acc / (float)T;
}

}  // namespace

hipError_t launch_layer_similarity(const void* x_in, const void* x_out, int n_seq, int T, int hidden,
                                   float* cos_out, float* sim_out, float* tile_sum, hipStream_t s) {
  LayerParams p;
  p.x_in = reinterpret_cast<const unsigned char*>(x_in);
  p.x_out = reinterpret_cast<const unsigned char*>(x_out);
  p.cos_out = cos_out;
  p.tile_sum = tile_sum;
  p.T = T; p.hidden = hidden;
  p.n_tiles = (T + kRowsPerWg - 1) / kRowsPerWg;
  const int64_t n_wg = (int64_t)n_seq * p.n_tiles;
  if (n_wg <= 0 || n_wg > INT32_MAX) return hipErrorInvalidValue;
  layer_cosine_kernel<<<dim3((unsigned)n_wg), dim3(256), 0, s>>>(p);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  layer_mean_kernel<<<dim3(n_seq), dim3(64), 0, s>>>(tile_sum, sim_out, p.n_tiles, T);
  return hipGetLastError();
}

}  // namespace baklava

// ---------------------------------------------------------------------------------------------
// The same pass for callers that cannot allocate and have no workspace to hand over: the
// per-workgroup partial sums live in a fixed device array instead.
// ---------------------------------------------------------------------------------------------

static __device__ __align__(256) float scratch[BAKLAVA_LAYER_STATIC_MAX_TILES];

namespace {

// In host code the array's name is only a handle for the runtime; the device address has to be
// asked for, once per device (every device holds its own copy of the array).
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
float* g_scratch_ptr[kMaxDevices] = {};

int scratch_for_current_device(float** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) { baklava::note_hip_error(e); return BAKLAVA_EHIP; }
  if (dev < 0 || dev >= kMaxDevices) return BAKLAVA_EINVAL;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    float* ptr = nullptr;
    e = hipGetSymbolAddress(reinterpret_cast<void**>(&ptr), HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr) { baklava::note_hip_error(e); return BAKLAVA_EHIP; }
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return BAKLAVA_OK;
}

}  // namespace

extern "C" int baklava_layer_similarity_static(const void* x_in, const void* x_out, int32_t n_seq, int32_t T,
                                               int32_t hidden, int32_t dtype, float* cos_out, float* sim_out,
                                               void* stream) {
  if (!x_in || !x_out || !sim_out) return BAKLAVA_EINVAL;
  if (n_seq <= 0 || T <= 0 || hidden <= 0 || hidden % 8 || dtype != BAKLAVA_BF16) return BAKLAVA_EINVAL;
  if (((uintptr_t)x_in | (uintptr_t)x_out) & 15) return BAKLAVA_EINVAL;
  if (((uintptr_t)sim_out | (uintptr_t)cos_out) & 3) return BAKLAVA_EINVAL;
  const int64_t tiles = (int64_t)n_seq * (((int64_t)T + baklava::kRowsPerWg - 1) / baklava::kRowsPerWg);
  if (tiles > BAKLAVA_LAYER_STATIC_MAX_TILES) return BAKLAVA_ECAPACITY;
  float* tile_sum = nullptr;
  const int st = scratch_for_current_device(&tile_sum);
  if (st != BAKLAVA_OK) return st;
  // Every partial sum the second kernel reads is written by the first one in this call, so nothing
  // has to be cleared; what earlier calls left in the array is never read.
  const hipError_t e = baklava::launch_layer_similarity(x_in, x_out, n_seq, T, hidden, cos_out, sim_out, tile_sum,
                                                        (hipStream_t)stream);
  if (e != hipSuccess) { baklava::note_hip_error(e); return BAKLAVA_EHIP; }
  return BAKLAVA_OK;
}
