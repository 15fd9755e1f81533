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

// Batch-mean full softmax per expert (the routing scores s of Eq. (3)).  A block takes 256 tokens, a
// wave walks its 64 tokens in order with the E logits spread over its lanes (VPL per lane), sums stay in
// registers; waves, then blocks, are added in a fixed order, so the result does not depend on timing.
constexpr int SC_TOKENS = 256;
template <int VPL>
__global__ __launch_bounds__(256) void route_scores_kernel(const float* __restrict__ logits, int n_tokens, int n_experts,
                                                           float* __restrict__ partial) {
  __shared__ float wsum[4][64 * VPL];
  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
  const float NEG_INF = -__builtin_inff();
  float acc[VPL];
#pragma unroll
  for (int i = 0; i < VPL; ++i) acc[i] = 0.0f;
  const long t0 = (long)blockIdx.x * SC_TOKENS + wave * 64;
  for (int i = 0; i < 64; ++i) {
    const long t = t0 + i;
    if (t >= n_tokens) break;  // uniform over the wave
    float v[VPL], m = NEG_INF;
#pragma unroll
    for (int j = 0; j < VPL; ++j) {
      const int e = lane + j * 64;
      v[j] = e < n_experts ? logits[t * n_experts + e] : NEG_INF;
      m = fmaxf(m, v[j]);
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
    float sum = 0.0f;
#pragma unroll
    for (int j = 0; j < VPL; ++j) { v[j] = expf(v[j] - m); sum += v[j]; }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) sum += __shfl_xor(sum, off);
    const float inv = 1.0f / sum;
#pragma unroll
    for (int j = 0; j < VPL; ++j) acc[j] += v[j] * inv;
  }
#pragma unroll
  for (int j = 0; j < VPL; ++j) wsum[wave][lane + j * 64] = acc[j];
  __syncthreads();
  for (int e = threadIdx.x; e < n_experts; e += 256)
    partial[(long)blockIdx.x * n_experts + e] = ((wsum[0][e] + wsum[1][e]) + wsum[2][e]) + wsum[3][e];
}

__global__ __launch_bounds__(256) void route_scores_finish_kernel(const float* __restrict__ partial, int n_blocks,
                                                                  int n_experts, float inv_tokens,
                                                                  float* __restrict__ scores) {
  const int e = blockIdx.x * 256 + threadIdx.x;
  if (e >= n_experts) return;
  float s = 0.0f;
  for (int b = 0; b < n_blocks; ++b) s += partial[(long)b * n_experts + e];
  scores[e] = s * inv_tokens;
}

}  // namespace hmoe

extern "C" size_t hmoe_route_scores_workspace_bytes(const hmoe_layer_desc* desc, int32_t T) {
  if (hmoe::check_desc(desc) != HMOE_OK || T < 0) return 0;
  const size_t blocks = ((size_t)T + hmoe::SC_TOKENS - 1) / hmoe::SC_TOKENS;
  return (blocks > 0 ? blocks : 1) * desc->n_experts * sizeof(float) + 256;
}

extern "C" int32_t hmoe_route_scores(const hmoe_layer_desc* desc, const float* logits, int32_t T, float* scores,
                                     float* h_scores_pinned, void* workspace, size_t workspace_bytes, void* stream) {
  using namespace hmoe;
  int rc = check_desc(desc);
  if (rc != HMOE_OK) return rc;
  if (T <= 0 || !logits || !scores) return HMOE_ERR_INVALID_ARG;
  if (!workspace || workspace_bytes < hmoe_route_scores_workspace_bytes(desc, T)) return HMOE_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(workspace) & 3u) return HMOE_ERR_INVALID_ARG;
  hipStream_t s = (hipStream_t)stream;
  const int E = desc->n_experts, blocks = (T + SC_TOKENS - 1) / SC_TOKENS;
  float* partial = (float*)workspace;
  if (E <= 64) hipLaunchKernelGGL((route_scores_kernel<1>), dim3(blocks), dim3(256), 0, s, logits, T, E, partial);
  else if (E <= 128) hipLaunchKernelGGL((route_scores_kernel<2>), dim3(blocks), dim3(256), 0, s, logits, T, E, partial);
  else hipLaunchKernelGGL((route_scores_kernel<4>), dim3(blocks), dim3(256), 0, s, logits, T, E, partial);
  hipLaunchKernelGGL(route_scores_finish_kernel, dim3((E + 255) / 256), dim3(256), 0, s, partial, blocks, E, 1.0f / (float)T,
                     scores);
  HMOE_HIP(hipGetLastError());
  if (h_scores_pinned)
    HMOE_HIP(hipMemcpyAsync(h_scores_pinned, scores, (size_t)E * sizeof(float), hipMemcpyDeviceToHost, s));
  return HMOE_OK;
}

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
