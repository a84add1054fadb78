// Shared head and tail of the two attention kernels: the fused append of the new row, and the
// end of a work item (merge of the workgroup's wavefronts, then either the finished output of a
// cache that has a single work item or the split partial the combine kernel reads).
#ifndef BAKLAVA_DECODE_TAIL_H
#define BAKLAVA_DECODE_TAIL_H

#include "common.h"

namespace baklava {

constexpr float kTailNegInf = -__builtin_huge_valf();

__device__ __forceinline__ float tail_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// [K'; K_t], [V'; V_t] of Eq. 7 inside the attention kernel: the work item whose row range holds
// slot `n_old` copies the new row there before it starts streaming.  The barrier makes the row
// visible to every wavefront of this workgroup; no other workgroup reads that slot.  The caller
// has checked n_old < capacity (uniform over the workgroup).
__device__ __forceinline__ void append_new_row(const DecodeParams& p, const Item& it, int n_old,
                                               int64_t off_c, int token_pos) {
  if (!(n_old >= it.start && n_old < it.start + it.count)) return;  // uniform over the workgroup
  const int tid = threadIdx.x;
  const int pieces = p.row_bytes / 16;
  const int64_t row = off_c + n_old;
  if (tid < 2 * pieces) {
    const int plane = tid / pieces, piece = tid % pieces;
    const char* src = reinterpret_cast<const char*>(plane ? p.v_new : p.k_new) +
                      (int64_t)(it.c - p.cache_begin) * p.row_bytes + piece * 16;
    char* dst = reinterpret_cast<char*>(plane ? p.v : p.k) + row * p.row_bytes + piece * 16;
    *reinterpret_cast<uint4*>(dst) = *reinterpret_cast<const uint4*>(src);
  }
  if (tid == (int)blockDim.x - 1) {
    p.score[row] = 0.f;
    p.pos[row] = token_pos;
  }
  __syncthreads();
}

// Where a call's record goes: behind the pending ones, or to the front when this call has added
// their weights to the scores (the record was full).
__device__ __forceinline__ int lag_slot(const DecodeParams& p, int pending) {
  return pending >= p.lag_batch ? 0 : pending;
}

// End of a work item.  On entry sm_o[w][g][d], sm_m[w][g], sm_l[w][g] (w < NW wavefronts, g-stride
// LDG) hold each wavefront's un-normalised output, running max and sum, and a barrier has been
// passed.  A cache that has a single work item is finished on the spot; otherwise the item's
// partial (max, sum, un-normalised output) is stored for the combine kernel.
template <int D, int LDG, int NW = 4>
__device__ __forceinline__ void finish_item(const DecodeParams& p, const Item& it, int G, int n_new,
                                            const float* sm_o, const float* sm_m, const float* sm_l) {
  const int tid = threadIdx.x;
  const int c = it.c;
  const bool single = it.nsplit == 1;
  const int c_rel = c - p.cache_begin;
  const int64_t orow0 = (int64_t)(c_rel / p.Hkv) * p.Hq + (int64_t)(c_rel % p.Hkv) * G;

  for (int idx = tid; idx < G * D; idx += 64 * NW) {
    const int g = idx / D, d = idx % D;
    float mm = sm_m[g];
#pragma unroll
    for (int w = 1; w < NW; ++w) mm = fmaxf(mm, sm_m[w * LDG + g]);
    const float ms = (mm == kTailNegInf) ? 0.f : mm;
    float ll = 0.f, oo = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      const float a = tail_exp2(sm_m[w * LDG + g] - ms);
      ll += sm_l[w * LDG + g] * a;
      oo += sm_o[(w * LDG + g) * D + d] * a;
    }
    if (single) {
      const float inv = 1.f / ll;
      p.out[(orow0 + g) * D + d] = oo * inv;
      if (d == 0) {
        p.final_ml[((int64_t)c * G + g) * 2 + 0] = ms;
        p.final_ml[((int64_t)c * G + g) * 2 + 1] = inv;
        if (p.lag) {
          const int slot = lag_slot(p, p.lag_cnt[(int64_t)c * G + g]);
          const int64_t m = (int64_t)c * kLagRows + (slot << p.lag_gp_log2) + g;
          p.lag_ml[m * 2 + 0] = ms;
          p.lag_ml[m * 2 + 1] = inv;
        }
      }
    } else {
      p.part_o[((int64_t)it.slot * G + g) * D + d] = oo;
      if (d == 0) {
        p.part_ml[((int64_t)it.slot * G + g) * 2 + 0] = mm;
        p.part_ml[((int64_t)it.slot * G + g) * 2 + 1] = ll;
      }
    }
  }
  if (single && p.fused_append && tid == 0) p.len[c] = n_new;
  if (single && p.lag) {
    // The record a later pass over this cache needs to add this call's weights to the scores: the
    // query rows (the normalisers went to lag_ml above), the number of rows they were taken over,
    // and the new count of pending calls.  Every wavefront of this workgroup, the only one that
    // serves the cache, has read the old record before the barriers that precede this function;
    // the barrier below separates the last read of the old count from its update.
    const int slot = lag_slot(p, p.lag_cnt[(int64_t)c * G]);
    const int ppr = p.row_bytes / 16;  // 16-byte pieces per row
    const uint4* src = reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(p.q) + orow0 * p.row_bytes);
    uint4* dst = reinterpret_cast<uint4*>(reinterpret_cast<char*>(p.lag_q) +
                                          ((int64_t)c * kLagRows + (slot << p.lag_gp_log2)) * p.row_bytes);
    for (int i = tid; i < G * ppr; i += 64 * NW) dst[i] = src[i];
    __syncthreads();
    if (tid == 0) p.lag_n[(int64_t)c * kLagCalls + slot] = n_new;
    if (tid < G) p.lag_cnt[(int64_t)c * G + tid] = slot + 1;
  }
}

}  // namespace baklava
#endif
