// hmoe_route: Softmax(TopK(logits)) of Eq. (1), one lane group per token.
//
// A group of G lanes (G = 8, 16, 32 or 64, the power of two >= E, at most one wavefront)
// holds a token's E logits, VPL per lane.  K rounds of a butterfly arg-max over
// (value, expert id) with the order "larger value first, equal values: smaller id first"
// pick the K experts; every lane of the group ends each round with the same winner, whose
// owner lane then retires it.  The softmax needs only the K winners.
#include "common.h"

namespace hmoe {

template <int G, int VPL>
__global__ __launch_bounds__(256) void route_kernel(const float* __restrict__ logits, int n_tokens, int n_experts,
                                                    int top_k, int32_t* __restrict__ topk_idx,
                                                    float* __restrict__ topk_w) {
  const int gl = threadIdx.x % G;  // lane within the group
  const long token = ((long)blockIdx.x * blockDim.x + threadIdx.x) / G;
  const bool live = token < n_tokens;  // uniform over the group
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

template <int G, int VPL>
static void launch_route(const float* logits, int T, int E, int K, int32_t* idx, float* w, hipStream_t s) {
  const int tokens_per_block = 256 / G;
  const int blocks = (T + tokens_per_block - 1) / tokens_per_block;
  hipLaunchKernelGGL((route_kernel<G, VPL>), dim3(blocks), dim3(256), 0, s, logits, T, E, K, idx, w);
}

}  // namespace hmoe

extern "C" int32_t hmoe_route(const hmoe_layer_desc* desc, const float* logits, int32_t T, int32_t* topk_idx,
                              float* topk_w, void* stream) {
  int rc = hmoe::check_desc(desc);
  if (rc != HMOE_OK) return rc;
  if (T < 0) return HMOE_ERR_INVALID_ARG;
  if (T == 0) return HMOE_OK;
  if (!logits || !topk_idx || !topk_w) return HMOE_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(logits) | reinterpret_cast<uintptr_t>(topk_idx) |
       reinterpret_cast<uintptr_t>(topk_w)) & 3u)
    return HMOE_ERR_INVALID_ARG;
  hipStream_t s = (hipStream_t)stream;
  const int E = desc->n_experts, K = desc->top_k;
  using namespace hmoe;
  if (E <= 8) launch_route<8, 1>(logits, T, E, K, topk_idx, topk_w, s);
  else if (E <= 16) launch_route<16, 1>(logits, T, E, K, topk_idx, topk_w, s);
  else if (E <= 32) launch_route<32, 1>(logits, T, E, K, topk_idx, topk_w, s);
  else if (E <= 64) launch_route<64, 1>(logits, T, E, K, topk_idx, topk_w, s);
  else if (E <= 128) launch_route<64, 2>(logits, T, E, K, topk_idx, topk_w, s);
  else launch_route<64, 4>(logits, T, E, K, topk_idx, topk_w, s);
  HMOE_HIP(hipGetLastError());
  return HMOE_OK;
}
