// Decode FFN (HMOE_FFN_SKINNY): every touched expert's weights are streamed from HBM exactly
// once, straight into MFMA operand registers.
//
// With a handful of rows per expert the expert FFN is bound by reading its weights (the paper
// observes GPU expert time flat in the workload at small batch, Section III / Fig. 3(f)), so the
// kernel is organised around the weight stream: a block owns one 32-row group of one matrix of
// one expert (for gate/up: the matching gate and up groups), its NW waves split the K range, and
// each wave issues U consecutive 1 KiB tile loads (one fully coalesced 16-byte load per lane,
// already in 32x32x16 bf16 MFMA operand order thanks to the packed slot layout) before it
// multiplies.  Tokens ride along as the other MFMA operand (up to 32 rows, zero padded), read
// from the L1/L2-resident activation rows.  Partial sums of the waves meet in LDS; wave 0 applies
// SwiGLU / rounds and stores.
#include <algorithm>

#include "common.h"

namespace hmoe {

struct SkinnyCtx {
  const int32_t* offsets;
  const int32_t* slot_of;
  const char* slots;
  size_t slot_bytes;
  ActiveMask active;
  int n_experts, hidden, ffn;
};

// id of the `want`-th expert (ascending) that is active, resident and has rows; -1 if fewer
__device__ __forceinline__ int nth_busy_expert(const SkinnyCtx& c, int want, int lane) {
  int seen = 0;
  for (int base = 0; base < c.n_experts; base += 64) {
    const int e = base + lane;
    const bool busy = e < c.n_experts && c.active.test(e) && c.slot_of[e] >= 0 && c.offsets[e + 1] > c.offsets[e];
    uint64_t m = __ballot(busy);
    const int n = __popcll(m);
    if (want < seen + n) {
      for (int i = seen; i < want; ++i) m &= m - 1;
      return base + __ffsll((long long)m) - 1;
    }
    seen += n;
  }
  return -1;
}

// GATEUP: in = x_perm [A, H], out = h [A, F];  else: in = h [A, F], out = o_perm [A, H].
// NW waves per block, MR = rows kept per pass (8 or 32), U = tiles in flight per wave and matrix.
template <bool GATEUP, int NW, int MR, int U>
__global__ __launch_bounds__(64 * NW) void ffn_skinny_kernel(SkinnyCtx c, const bf16_t* __restrict__ in,
                                                              bf16_t* __restrict__ out) {
  constexpr int NMAT = GATEUP ? 2 : 1;
  constexpr int RR = MR == 8 ? 4 : 16;  // accumulator registers that can hold valid rows
  __shared__ float red[(NW - 1) * NMAT * RR * 64];

  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
  const int e = nth_busy_expert(c, blockIdx.y, lane);
  if (e < 0) return;  // uniform over the block
  const int row_first = c.offsets[e], row_end = c.offsets[e + 1];
  const int K = GATEUP ? c.hidden : c.ffn;        // reduction length
  const int n_out = GATEUP ? c.ffn : c.hidden;    // row length of `out`
  const int kt = K / TILE_K;
  const char* slot = c.slots + (size_t)c.slot_of[e] * c.slot_bytes;
  // this block's 32-row group(s)
  const u32x4* w0;
  const u32x4* w1 = nullptr;
  if (GATEUP) {
    w0 = (const u32x4*)slot + (size_t)(2 * blockIdx.x) * kt * 64;
    w1 = w0 + (size_t)kt * 64;
  } else {
    w0 = (const u32x4*)(slot + 4 * (size_t)c.ffn * c.hidden) + (size_t)blockIdx.x * kt * 64;
  }
  // this wave's share of the K tiles
  const int per_wave = (kt + NW - 1) / NW;
  const int kb0 = min(wave * per_wave, kt), kb1 = min(kb0 + per_wave, kt);
  const int half = lane / 32, col = lane % 32;

  for (int row0 = row_first; row0 < row_end; row0 += MR) {
    const int rows = min(MR, row_end - row0);
    const bool has_row = col < rows;
    const u32x4* xin = (const u32x4*)(in + (size_t)(row0 + (has_row ? col : 0)) * K) + half;
    f32x16_t acc0 = {0}, acc1 = {0};
    for (int kb = kb0; kb < kb1; kb += U) {
      u32x4 wa[U], wb[U], xa[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const bool in_range = kb + u < kb1;
        const size_t t = (size_t)(kb + u) * 64 + lane;
        wa[u] = in_range ? __builtin_nontemporal_load(w0 + t) : u32x4{0, 0, 0, 0};
        if (GATEUP) wb[u] = in_range ? __builtin_nontemporal_load(w1 + t) : u32x4{0, 0, 0, 0};
        xa[u] = (in_range && has_row) ? xin[(size_t)(kb + u) * 2] : u32x4{0, 0, 0, 0};
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        acc0 = mfma_32x32x16_bf16(xa[u], wa[u], acc0);
        if (GATEUP) acc1 = mfma_32x32x16_bf16(xa[u], wb[u], acc1);
      }
    }
    // accumulator register r of lane (half, col) is row 8*(r/4) + 4*half + r%4, output column col
    if (wave > 0) {
      float* dst = red + (size_t)(wave - 1) * NMAT * RR * 64;
#pragma unroll
      for (int r = 0; r < RR; ++r) {
        if ((r / 4) * 8 < rows) {
          dst[r * 64 + lane] = acc0[r];
          if (GATEUP) dst[(RR + r) * 64 + lane] = acc1[r];
        }
      }
    }
    __syncthreads();
    if (wave == 0) {
#pragma unroll
      for (int r = 0; r < RR; ++r) {
        if ((r / 4) * 8 < rows) {
          float g = acc0[r], u = GATEUP ? acc1[r] : 0.0f;
          for (int w = 0; w < NW - 1; ++w) {
            g += red[((size_t)w * NMAT * RR + r) * 64 + lane];
            if (GATEUP) u += red[((size_t)w * NMAT * RR + RR + r) * 64 + lane];
          }
          const int m = (r / 4) * 8 + half * 4 + (r % 4);
          if (m < rows) {
            const float v = GATEUP ? silu_f32(g) * u : g;
            out[(size_t)(row0 + m) * n_out + blockIdx.x * TILE_N + col] = f32_to_bf16(v);
          }
        }
      }
    }
    __syncthreads();
  }
}

template <bool GATEUP, int NW, int MR>
static void launch_one(const SkinnyCtx& c, int groups, int busy_max, const bf16_t* in, bf16_t* out, hipStream_t s) {
  hipLaunchKernelGGL((ffn_skinny_kernel<GATEUP, NW, MR, 4>), dim3((unsigned)groups, (unsigned)busy_max), dim3(64 * NW), 0,
                     s, c, in, out);
}

template <bool GATEUP>
static void launch_stage(const SkinnyCtx& c, int groups, int busy_max, int max_rows, int kt, const bf16_t* in,
                         bf16_t* out, hipStream_t s) {
  if (max_rows > 8) {
    launch_one<GATEUP, 4, 32>(c, groups, busy_max, in, out, s);
    return;
  }
  // enough waves to keep HBM busy (about 16 per CU), but at least 4 K tiles per wave
  int nw = 4;
  while (nw < 16 && (long)groups * busy_max * nw < 4096 && kt / (nw * 2) >= 4) nw *= 2;
  if (nw == 4) launch_one<GATEUP, 4, 8>(c, groups, busy_max, in, out, s);
  else if (nw == 8) launch_one<GATEUP, 8, 8>(c, groups, busy_max, in, out, s);
  else launch_one<GATEUP, 16, 8>(c, groups, busy_max, in, out, s);
}

int launch_ffn_skinny(const FfnArgs& a) {
  const hmoe_layer_desc& d = *a.desc;
  if (d.dtype != HMOE_BF16) return HMOE_ERR_UNSUPPORTED;
  if (a.n_rows == 0) return HMOE_OK;
  SkinnyCtx c{a.offsets, a.slot_of, a.slots, a.slot_bytes, a.active, d.n_experts, d.hidden, d.ffn};
  const int busy_max = std::min(d.n_experts, a.n_rows);     // every busy expert has at least one row
  const int max_rows = std::max(1, a.n_rows / d.top_k);     // a token names an expert at most once
  probe_before(a.stream);
  launch_stage<true>(c, d.ffn / TILE_N, busy_max, max_rows, d.hidden / TILE_K, (const bf16_t*)a.x_perm, (bf16_t*)a.h,
                     a.stream);
  probe_after(a.stream);
  launch_stage<false>(c, d.hidden / TILE_N, busy_max, max_rows, d.ffn / TILE_K, (const bf16_t*)a.h, (bf16_t*)a.o_perm,
                      a.stream);
  HMOE_HIP(hipGetLastError());
  return HMOE_OK;
}

}  // namespace hmoe
