// hmoe_route: Softmax(TopK(logits)) of Eq. (1), one lane group per token (route_body.h).
#include "route_body.h"

namespace hmoe {

template <int G, int VPL>
__global__ __launch_bounds__(256) void route_kernel(const float* __restrict__ logits, int n_tokens, int n_experts,
                                                    int top_k, int32_t* __restrict__ topk_idx,
                                                    float* __restrict__ topk_w) {
  const long token = ((long)blockIdx.x * blockDim.x + threadIdx.x) / G;
  route_token<G, VPL>(logits, n_experts, top_k, token, token < n_tokens, threadIdx.x % G, topk_idx, topk_w);
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
