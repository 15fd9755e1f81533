// Device-side routing of one token by one lane group; shared by hmoe_route and the fused
// small-batch front end.
#pragma once

#include "common.h"

namespace hmoe {

// A group of G lanes (G = 8, 16, 32 or 64, the power of two >= min(E, 64)) holds a token's E logits,
// VPL per lane.  K rounds of a butterfly arg-max over (value, expert id) with the order "larger value
// first, equal values: smaller id first" pick the K experts; every lane of the group ends each round
// with the same winner, whose owner lane then retires it.  The softmax needs only the K winners.
// `gl` = lane within the group; `live` must be uniform over the group.
template <int G, int VPL>
__device__ __forceinline__ void route_token(const float* __restrict__ logits, int n_experts, int top_k, long token,
                                            bool live, int gl, int32_t* __restrict__ topk_idx,
                                            float* __restrict__ topk_w) {
  const float NEG_INF = -__builtin_inff();
  float v[VPL];
#pragma unroll
  for (int i = 0; i < VPL; ++i) {
    const int e = gl + i * G;
    v[i] = (live && e < n_experts) ? logits[token * n_experts + e] : NEG_INF;
  }
  float win_v[VPL];  // winner j is kept by lane j % G in register j / G
  int win_i[VPL];
#pragma unroll
  for (int i = 0; i < VPL; ++i) { win_v[i] = NEG_INF; win_i[i] = 0; }

  float v_max = 0.0f, denom = 0.0f;
  for (int j = 0; j < top_k; ++j) {
    float bv = v[0];
    int bi = gl;
#pragma unroll
    for (int i = 1; i < VPL; ++i) {  // ascending ids: strict > keeps the smaller id on ties
      if (v[i] > bv) { bv = v[i]; bi = gl + i * G; }
    }
#pragma unroll
    for (int off = G / 2; off >= 1; off >>= 1) {
      const float ov = __shfl_xor(bv, off);
      const int oi = __shfl_xor(bi, off);
      if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
    }
    if (j == 0) v_max = bv;
    denom += expf(bv - v_max);
#pragma unroll
    for (int i = 0; i < VPL; ++i) {
      if (bi == gl + i * G) v[i] = NEG_INF;          // retire the winner
      if (j == gl + i * G) { win_v[i] = bv; win_i[i] = bi; }
    }
  }
  if (!live) return;
  const float inv = 1.0f / denom;
#pragma unroll
  for (int i = 0; i < VPL; ++i) {
    const int j = gl + i * G;
    if (j < top_k) {
      const int e = win_i[i] < n_experts ? win_i[i] : n_experts - 1;  // only reachable with non-finite input
      topk_idx[token * top_k + j] = e;
      topk_w[token * top_k + j] = expf(win_v[i] - v_max) * inv;
    }
  }
}

}  // namespace hmoe
