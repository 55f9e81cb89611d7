// Device-side pieces of the token assignment that more than one translation unit uses (hipcc only).
#pragma once
#include "si_internal.h"

namespace si {

__device__ inline bool route_better(float v, int i, float ov, int oi) {
  // true when (ov, oi) should replace (v, i): larger logit, or equal logit and lower index
  return ov > v || (ov == v && oi < i);
}

// One wave selects the top-k experts of one token (Section II-A: the gating function): k rounds of a butterfly
// arg-max over the raw logits, ties to the lower expert index, then the softmax over the k selected logits.
// sel (LDS, >= k floats) receives the k logits.  E <= 256.
__device__ inline void topk_token(const float* __restrict__ l, int E, int k, int lane, int32_t* __restrict__ idx_out,
                                  float* __restrict__ w_out, float* sel) {
  constexpr int WAVE = 64;
  float v[4];
  unsigned taken = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int e = lane + WAVE * i;
    v[i] = e < E ? l[e] : 0.f;
    if (e >= E) taken |= 1u << i;
  }
  for (int s = 0; s < k; ++s) {
    float bv = 0.f;
    int bi = 0x7fffffff;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (!(taken & (1u << i))) {
        int e = lane + WAVE * i;
        if (bi == 0x7fffffff || route_better(bv, bi, v[i], e)) { bv = v[i]; bi = e; }
      }
    }
#pragma unroll
    for (int d = 1; d < WAVE; d <<= 1) {
      float ov = __shfl_xor(bv, d, WAVE);
      int oi = __shfl_xor(bi, d, WAVE);
      bool take = (oi != 0x7fffffff) && (bi == 0x7fffffff || route_better(bv, bi, ov, oi));
      if (take) { bv = ov; bi = oi; }
    }
    // every lane now holds the same winner
    if ((bi & (WAVE - 1)) == lane) taken |= 1u << (bi / WAVE);
    if (lane == 0) { idx_out[s] = bi; sel[s] = bv; }
  }
  if (lane == 0) {
    // softmax over the k selected logits; sel[0] is the maximum.  Sequential, slot order.
    float l0 = sel[0];
    float sum = 0.f;
    for (int s = 0; s < k; ++s) sum += expf(sel[s] - l0);
    for (int s = 0; s < k; ++s) w_out[s] = expf(sel[s] - l0) / sum;
  }
}

}  // namespace si
