// Reference FFN kernels (HMOE_FFN_REFERENCE): one wavefront per output element, lanes stride
// the reduction dimension.  Any shape; fp32 (plain row-major slots), bf16 (packed slots) and 4-bit
// weights (decoded element by element).
// This is the path of the fp32 toy workload and the in-library cross-check for the MFMA paths.
#include "common.h"

namespace hmoe {

// expert that owns sorted row p: offsets[e] <= p < offsets[e+1]
__device__ __forceinline__ int expert_of_row(const int32_t* __restrict__ offsets, int n_experts, int p) {
  int lo = 0, hi = n_experts;  // invariant: offsets[lo] <= p < offsets[hi]
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (offsets[mid] <= p) lo = mid; else hi = mid;
  }
  return lo;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
  return v;
}

struct RefCtx {
  const int32_t* offsets;
  const int32_t* slot_of;
  const char* slots;
  size_t slot_bytes;
  ActiveMask active;
  int n_experts, hidden, ffn, n_rows;
  const int32_t* row_map;
  int map_div;
};

// returns slot base or nullptr if row p is not to be computed
__device__ __forceinline__ const char* row_slot(const RefCtx& c, int p) {
  const int e = expert_of_row(c.offsets, c.n_experts, p);
  if (!c.active.test(e)) return nullptr;
  const int s = c.slot_of[e];
  if (s < 0) return nullptr;
  return c.slots + (size_t)s * c.slot_bytes;
}

__global__ __launch_bounds__(256) void ref_gateup_f32(RefCtx c, const float* __restrict__ x, float* __restrict__ h) {
  const int p = blockIdx.x, wave = threadIdx.x / 64, lane = threadIdx.x % 64;
  const int f = blockIdx.y * 4 + wave;
  if (f >= c.ffn) return;
  const char* slot = row_slot(c, p);
  if (!slot) return;
  const float* wg = (const float*)slot + (size_t)f * c.hidden;
  const float* wu = wg + (size_t)c.ffn * c.hidden;
  const float* xr = x + (size_t)mapped_row(c.row_map, c.map_div, p) * c.hidden;
  float g = 0.0f, u = 0.0f;
  for (int k = lane; k < c.hidden; k += 64) {
    const float xv = xr[k];
    g = fmaf(wg[k], xv, g);
    u = fmaf(wu[k], xv, u);
  }
  g = wave_sum(g);
  u = wave_sum(u);
  if (lane == 0) h[(size_t)p * c.ffn + f] = g / (1.0f + expf(-g)) * u;
}

__global__ __launch_bounds__(256) void ref_down_f32(RefCtx c, const float* __restrict__ h, float* __restrict__ o) {
  const int p = blockIdx.x, wave = threadIdx.x / 64, lane = threadIdx.x % 64;
  const int n = blockIdx.y * 4 + wave;
  if (n >= c.hidden) return;
  const char* slot = row_slot(c, p);
  if (!slot) return;
  const float* wd = (const float*)slot + 2 * (size_t)c.ffn * c.hidden + (size_t)n * c.ffn;
  const float* hr = h + (size_t)p * c.ffn;
  float acc = 0.0f;
  for (int k = lane; k < c.ffn; k += 64) acc = fmaf(wd[k], hr[k], acc);
  acc = wave_sum(acc);
  if (lane == 0) o[(size_t)p * c.hidden + n] = acc;
}

__global__ __launch_bounds__(256) void ref_gateup_bf16(RefCtx c, const bf16_t* __restrict__ x, bf16_t* __restrict__ h) {
  const int p = blockIdx.x, wave = threadIdx.x / 64, lane = threadIdx.x % 64;
  const int f = blockIdx.y * 4 + wave;
  if (f >= c.ffn) return;
  const char* slot = row_slot(c, p);
  if (!slot) return;
  const bf16_t* wgu = (const bf16_t*)slot;
  const int kt = c.hidden / TILE_K;
  const int n_gate = 2 * TILE_N * (f / TILE_N) + f % TILE_N, n_up = n_gate + TILE_N;
  const bf16_t* xr = x + (size_t)mapped_row(c.row_map, c.map_div, p) * c.hidden;
  float g = 0.0f, u = 0.0f;
  for (int k = lane; k < c.hidden; k += 64) {
    const float xv = bf16_to_f32(xr[k]);
    g = fmaf(bf16_to_f32(wgu[packed_index(n_gate, k, kt)]), xv, g);
    u = fmaf(bf16_to_f32(wgu[packed_index(n_up, k, kt)]), xv, u);
  }
  g = wave_sum(g);
  u = wave_sum(u);
  if (lane == 0) h[(size_t)p * c.ffn + f] = f32_to_bf16(g / (1.0f + expf(-g)) * u);
}

__global__ __launch_bounds__(256) void ref_down_bf16(RefCtx c, const bf16_t* __restrict__ h, bf16_t* __restrict__ o) {
  const int p = blockIdx.x, wave = threadIdx.x / 64, lane = threadIdx.x % 64;
  const int n = blockIdx.y * 4 + wave;
  if (n >= c.hidden) return;
  const char* slot = row_slot(c, p);
  if (!slot) return;
  const bf16_t* wd = (const bf16_t*)slot + 2 * (size_t)c.ffn * c.hidden;
  const int kt = c.ffn / TILE_K;
  const bf16_t* hr = h + (size_t)p * c.ffn;
  float acc = 0.0f;
  for (int k = lane; k < c.ffn; k += 64) acc = fmaf(bf16_to_f32(wd[packed_index(n, k, kt)]), bf16_to_f32(hr[k]), acc);
  acc = wave_sum(acc);
  if (lane == 0) o[(size_t)p * c.hidden + n] = f32_to_bf16(acc);
}

// 4-bit weights: value of W[n][k] of a matrix with K columns stored at `units` / `scales`
__device__ __forceinline__ float w4_value(const uint32_t* __restrict__ units, const bf16_t* __restrict__ scales, int n, int k,
                                          int K) {
  const int q = (units[w4_dword_index(n, k, K)] >> w4_code_shift(k)) & 15;
  return (float)(q - 8) * bf16_to_f32(scales[w4_scale_index(n, k / W4_GROUP, K / W4_GROUP)]);
}

__global__ __launch_bounds__(256) void ref_gateup_w4(RefCtx c, const bf16_t* __restrict__ x, bf16_t* __restrict__ h) {
  const int p = blockIdx.x, wave = threadIdx.x / 64, lane = threadIdx.x % 64;
  const int f = blockIdx.y * 4 + wave;
  if (f >= c.ffn) return;
  const char* slot = row_slot(c, p);
  if (!slot) return;
  const W4Offsets off = w4_offsets((size_t)c.hidden, (size_t)c.ffn);
  const uint32_t* units = (const uint32_t*)slot;
  const bf16_t* scales = (const bf16_t*)(slot + off.gate_up_scales);
  const int n_gate = 32 * (f / 16) + f % 16, n_up = n_gate + 16;  // gate and up interleaved in 16-row groups
  const bf16_t* xr = x + (size_t)mapped_row(c.row_map, c.map_div, p) * c.hidden;
  float g = 0.0f, u = 0.0f;
  for (int k = lane; k < c.hidden; k += 64) {
    const float xv = bf16_to_f32(xr[k]);
    g = fmaf(w4_value(units, scales, n_gate, k, c.hidden), xv, g);
    u = fmaf(w4_value(units, scales, n_up, k, c.hidden), xv, u);
  }
  g = wave_sum(g);
  u = wave_sum(u);
  if (lane == 0) h[(size_t)p * c.ffn + f] = f32_to_bf16(g / (1.0f + expf(-g)) * u);
}

__global__ __launch_bounds__(256) void ref_down_w4(RefCtx c, const bf16_t* __restrict__ h, bf16_t* __restrict__ o) {
  const int p = blockIdx.x, wave = threadIdx.x / 64, lane = threadIdx.x % 64;
  const int n = blockIdx.y * 4 + wave;
  if (n >= c.hidden) return;
  const char* slot = row_slot(c, p);
  if (!slot) return;
  const W4Offsets off = w4_offsets((size_t)c.hidden, (size_t)c.ffn);
  const uint32_t* units = (const uint32_t*)(slot + off.down_units);
  const bf16_t* scales = (const bf16_t*)(slot + off.down_scales);
  const bf16_t* hr = h + (size_t)p * c.ffn;
  float acc = 0.0f;
  for (int k = lane; k < c.ffn; k += 64) acc = fmaf(w4_value(units, scales, n, k, c.ffn), bf16_to_f32(hr[k]), acc);
  acc = wave_sum(acc);
  if (lane == 0) o[(size_t)p * c.hidden + n] = f32_to_bf16(acc);
}

int launch_ffn_reference(const FfnArgs& a) {
  const hmoe_layer_desc& d = *a.desc;
  if (a.n_rows == 0) return HMOE_OK;
  if ((d.ffn + 3) / 4 > 65535 || (d.hidden + 3) / 4 > 65535) return HMOE_ERR_UNSUPPORTED;
  RefCtx c{a.offsets, a.slot_of, a.slots, a.slot_bytes, a.active, d.n_experts, d.hidden, d.ffn, a.n_rows, a.row_map, a.map_div};
  const dim3 g1((unsigned)a.n_rows, (unsigned)((d.ffn + 3) / 4)), g2((unsigned)a.n_rows, (unsigned)((d.hidden + 3) / 4));
  probe_before(a.stream);
  if (d.dtype == HMOE_F32)
    hipLaunchKernelGGL(ref_gateup_f32, g1, dim3(256), 0, a.stream, c, (const float*)a.x_perm, (float*)a.h);
  else if (d.dtype == HMOE_BF16_W4)
    hipLaunchKernelGGL(ref_gateup_w4, g1, dim3(256), 0, a.stream, c, (const bf16_t*)a.x_perm, (bf16_t*)a.h);
  else
    hipLaunchKernelGGL(ref_gateup_bf16, g1, dim3(256), 0, a.stream, c, (const bf16_t*)a.x_perm, (bf16_t*)a.h);
  probe_after(a.stream);
  probe_before(a.stream);
  if (d.dtype == HMOE_F32)
    hipLaunchKernelGGL(ref_down_f32, g2, dim3(256), 0, a.stream, c, (const float*)a.h, (float*)a.o_perm);
  else if (d.dtype == HMOE_BF16_W4)
    hipLaunchKernelGGL(ref_down_w4, g2, dim3(256), 0, a.stream, c, (const bf16_t*)a.h, (bf16_t*)a.o_perm);
  else
    hipLaunchKernelGGL(ref_down_bf16, g2, dim3(256), 0, a.stream, c, (const bf16_t*)a.h, (bf16_t*)a.o_perm);
  probe_after(a.stream);
  HMOE_HIP(hipGetLastError());
  return HMOE_OK;
}

}  // namespace hmoe
