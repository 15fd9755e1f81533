// hmoe_combine: the gate-weighted sum of Eq. (1) in gather form,
//   y[t] = sum_{j<K} w[t,j] * o_perm[inv_perm[t*K+j]] (+ o_shared[t]),
// j ascending then the shared term, fp32 accumulation, one rounding.  No atomics: every output
// element is produced by one lane, so results do not depend on scheduling.
// Also: hmoe_router_logits (x . W_g), the small GEMM in front of the router.
#include "router_body.h"

namespace hmoe {

__global__ __launch_bounds__(256) void combine_bf16_kernel(const uint4* __restrict__ o_perm,
                                                           const int32_t* __restrict__ inv_perm,
                                                           const float* __restrict__ topk_w,
                                                           const uint4* __restrict__ o_shared, int top_k, int row_vec,
                                                           uint4* __restrict__ y) {
  const long t = blockIdx.x;
  __shared__ int rows[HMOE_MAX_TOP_K];
  __shared__ float wts[HMOE_MAX_TOP_K];
  if (threadIdx.x < top_k) {
    rows[threadIdx.x] = inv_perm[t * top_k + threadIdx.x];
    wts[threadIdx.x] = topk_w[t * top_k + threadIdx.x];
  }
  __syncthreads();
  for (int c = threadIdx.x; c < row_vec; c += blockDim.x) {
    float acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = 0.0f;
    for (int j = 0; j < top_k; ++j) {
      const uint4 v = o_perm[(long)rows[j] * row_vec + c];
      const float w = wts[j];
      const uint32_t u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        acc[2 * i] += w * __uint_as_float(u[i] << 16);
        acc[2 * i + 1] += w * __uint_as_float(u[i] & 0xffff0000u);
      }
    }
    if (o_shared) {
      const uint4 v = o_shared[t * row_vec + c];
      const uint32_t u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        acc[2 * i] += __uint_as_float(u[i] << 16);
        acc[2 * i + 1] += __uint_as_float(u[i] & 0xffff0000u);
      }
    }
    uint32_t o[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) o[i] = (uint32_t)f32_to_bf16(acc[2 * i]) | ((uint32_t)f32_to_bf16(acc[2 * i + 1]) << 16);
    y[t * row_vec + c] = make_uint4(o[0], o[1], o[2], o[3]);
  }
}

__global__ __launch_bounds__(256) void combine_f32_kernel(const float* __restrict__ o_perm,
                                                          const int32_t* __restrict__ inv_perm,
                                                          const float* __restrict__ topk_w,
                                                          const float* __restrict__ o_shared, int top_k, int hidden,
                                                          float* __restrict__ y) {
  const long t = blockIdx.x;
  for (int c = threadIdx.x; c < hidden; c += blockDim.x) {
    float acc = 0.0f;
    for (int j = 0; j < top_k; ++j)
      acc += topk_w[t * top_k + j] * o_perm[(long)inv_perm[t * top_k + j] * hidden + c];
    if (o_shared) acc += o_shared[t * hidden + c];
    y[t * hidden + c] = acc;
  }
}

// logits[t, e] = sum_h x[t,h] * w_g[e,h], fp32 accumulate.
// fp32 layers: one wavefront per (token, expert) dot product.
__global__ __launch_bounds__(256) void router_logits_f32_kernel(const float* __restrict__ x, const float* __restrict__ w_g,
                                                                int n_tokens, int n_experts, int hidden,
                                                                float* __restrict__ logits) {
  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
  const long pair = (long)blockIdx.x * 4 + wave;
  if (pair >= (long)n_tokens * n_experts) return;
  const long t = pair / n_experts;
  const int e = (int)(pair % n_experts);
  const float* xr = x + t * hidden;
  const float* wr = w_g + (long)e * hidden;
  float acc = 0.0f;
  for (int h = lane; h < hidden; h += 64) acc = fmaf(xr[h], wr[h], acc);
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) acc += __shfl_xor(acc, off);
  if (lane == 0) logits[pair] = acc;
}

// bf16 layers, more than 8 tokens: see router_logits_tokens.
template <int NF>
__global__ __launch_bounds__(256) void router_logits_bf16_kernel(const bf16_t* __restrict__ x,
                                                                 const bf16_t* __restrict__ w_g, int n_tokens,
                                                                 int n_experts, int hidden, float* __restrict__ logits,
                                                                 int tokens_per_block) {
  router_logits_tokens<NF>(x, w_g, n_tokens, n_experts, hidden, logits, tokens_per_block, nullptr);
}

// decode batches (T <= 8): one block, loads kept in flight (router_body.h)
template <int NF>
__global__ __launch_bounds__(256) void router_logits_small_kernel(const bf16_t* __restrict__ x,
                                                                  const bf16_t* __restrict__ w_g, int n_tokens,
                                                                  int n_experts, int hidden, float* __restrict__ logits) {
  router_logits_small<NF>(x, w_g, n_tokens, n_experts, hidden, logits, nullptr);
}

}  // namespace hmoe

extern "C" int32_t hmoe_combine(const hmoe_layer_desc* desc, const void* o_perm, const int32_t* inv_perm,
                                const float* topk_w, const void* o_shared, int32_t T, void* y, void* stream) {
  using namespace hmoe;
  int rc = check_desc(desc);
  if (rc != HMOE_OK) return rc;
  if (T < 0) return HMOE_ERR_INVALID_ARG;
  if (T == 0) return HMOE_OK;
  if (!o_perm || !inv_perm || !topk_w || !y) return HMOE_ERR_INVALID_ARG;
  if (!aligned16(o_perm) || !aligned16(y) || (o_shared && !aligned16(o_shared))) return HMOE_ERR_INVALID_ARG;
  hipStream_t s = (hipStream_t)stream;
  if (desc->dtype != HMOE_F32) {
    if (desc->hidden % 8 != 0) return HMOE_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(combine_bf16_kernel, dim3((unsigned)T), dim3(256), 0, s, (const uint4*)o_perm, inv_perm, topk_w,
                       (const uint4*)o_shared, desc->top_k, desc->hidden / 8, (uint4*)y);
  } else {
    hipLaunchKernelGGL(combine_f32_kernel, dim3((unsigned)T), dim3(256), 0, s, (const float*)o_perm, inv_perm, topk_w,
                       (const float*)o_shared, desc->top_k, desc->hidden, (float*)y);
  }
  HMOE_HIP(hipGetLastError());
  return HMOE_OK;
}

extern "C" int32_t hmoe_router_logits(const hmoe_layer_desc* desc, const void* x, const void* w_g, int32_t T,
                                      float* logits, void* stream) {
  using namespace hmoe;
  int rc = check_desc(desc);
  if (rc != HMOE_OK) return rc;
  if (T < 0) return HMOE_ERR_INVALID_ARG;
  if (T == 0) return HMOE_OK;
  if (!x || !w_g || !logits) return HMOE_ERR_INVALID_ARG;
  hipStream_t s = (hipStream_t)stream;
  const int E = desc->n_experts, H = desc->hidden;
  if (desc->dtype != HMOE_F32) {
    if (H % 16 != 0) return HMOE_ERR_UNSUPPORTED;
    if (!aligned16(x) || !aligned16(w_g)) return HMOE_ERR_INVALID_ARG;
    int tpb = 32;  // tokens per block: fewer while the grid would leave more than half of the CUs without a block
    while (tpb > 4 && (T + tpb - 1) / tpb < 128) tpb /= 2;
    const dim3 grid((unsigned)((T + tpb - 1) / tpb)), block(256);
    const bf16_t* xb = (const bf16_t*)x;
    const bf16_t* wb = (const bf16_t*)w_g;
    if (T <= ROUTER_SMALL_T) {
      if (E <= 32) hipLaunchKernelGGL((router_logits_small_kernel<1>), dim3(1), block, 0, s, xb, wb, T, E, H, logits);
      else if (E <= 64) hipLaunchKernelGGL((router_logits_small_kernel<2>), dim3(1), block, 0, s, xb, wb, T, E, H, logits);
      else if (E <= 128) hipLaunchKernelGGL((router_logits_small_kernel<4>), dim3(1), block, 0, s, xb, wb, T, E, H, logits);
      else hipLaunchKernelGGL((router_logits_small_kernel<8>), dim3(1), block, 0, s, xb, wb, T, E, H, logits);
    } else if (E <= 32) hipLaunchKernelGGL((router_logits_bf16_kernel<1>), grid, block, 0, s, xb, wb, T, E, H, logits, tpb);
    else if (E <= 64) hipLaunchKernelGGL((router_logits_bf16_kernel<2>), grid, block, 0, s, xb, wb, T, E, H, logits, tpb);
    else if (E <= 128) hipLaunchKernelGGL((router_logits_bf16_kernel<4>), grid, block, 0, s, xb, wb, T, E, H, logits, tpb);
    else hipLaunchKernelGGL((router_logits_bf16_kernel<8>), grid, block, 0, s, xb, wb, T, E, H, logits, tpb);
  } else {
    const long pairs = (long)T * E;
    hipLaunchKernelGGL(router_logits_f32_kernel, dim3((unsigned)((pairs + 3) / 4)), dim3(256), 0, s, (const float*)x,
                       (const float*)w_g, T, E, H, logits);
  }
  HMOE_HIP(hipGetLastError());
  return HMOE_OK;
}
