// Router logits x . W_g (Eq. (1), Section II-A) of a decode batch by ONE block; shared by
// hmoe_router_logits (T <= 8) and the fused decode front end.
#pragma once

#include "common.h"

namespace hmoe {

constexpr int ROUTER_SMALL_T = 8;  // tokens the one-block body handles

// 256 threads.  bf16 operands, K-contiguous rows: lanes load 32x32x16 MFMA fragments straight from
// global memory (token or expert row = lane % 32, 8 k values at 8 * (lane / 32)); the 4 waves split K
// into 4 contiguous ranges and add their partial sums in wave order, which is the summation order of
// the many-token kernel, so both produce the same bits.  With at most 8 tokens only accumulator
// registers 0..3 hold rows (register r of lane (half, col) is token 4 * half + r, expert col).
// Two register sets of U k-tiles alternate so that loads stay in flight while the other set is
// multiplied: a decode router is a chain of dependent memory round trips, not a bandwidth problem.
//   logits [T, E] global out; lds_logits [T * E] the same values in LDS, or NULL.
// Ends with a block barrier.
template <int NF>
__device__ __forceinline__ void router_logits_small(const bf16_t* __restrict__ x, const bf16_t* __restrict__ w_g,
                                                    int n_tokens, int n_experts, int hidden,
                                                    float* __restrict__ logits, float* lds_logits) {
  constexpr int U = NF == 1 ? 8 : NF == 2 ? 4 : NF == 4 ? 2 : 1;
  __shared__ float red[3 * NF * 4 * 64];
  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64, half = lane / 32, col = lane % 32;
  const int kt = hidden / 16, per_wave = (kt + 3) / 4;
  const int kb0 = min(wave * per_wave, kt), kb1 = min(kb0 + per_wave, kt);
  const bool has_tok = col < n_tokens;
  const u32x4* xp = (const u32x4*)(x + (long)(has_tok ? col : 0) * hidden) + half;
  const u32x4* wp[NF];
  bool has_exp[NF];
#pragma unroll
  for (int j = 0; j < NF; ++j) {
    has_exp[j] = j * 32 + col < n_experts;
    wp[j] = (const u32x4*)(w_g + (long)(has_exp[j] ? j * 32 + col : 0) * hidden) + half;
  }
  f32x16_t acc[NF];
#pragma unroll
  for (int j = 0; j < NF; ++j) acc[j] = f32x16_t{0};
  u32x4 xa[2][U], wb[2][U][NF];
  auto load = [&](int set, int kb) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const bool in_range = kb + u < kb1;
      xa[set][u] = (in_range && has_tok) ? xp[(long)(kb + u) * 2] : u32x4{0, 0, 0, 0};
#pragma unroll
      for (int j = 0; j < NF; ++j)
        wb[set][u][j] = (in_range && has_exp[j]) ? wp[j][(long)(kb + u) * 2] : u32x4{0, 0, 0, 0};
    }
  };
  auto multiply = [&](int set) {
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int j = 0; j < NF; ++j) acc[j] = mfma_32x32x16_bf16(xa[set][u], wb[set][u][j], acc[j]);
  };
  load(0, kb0);
  for (int kb = kb0; kb < kb1; kb += 2 * U) {
    load(1, kb + U);
    multiply(0);
    load(0, kb + 2 * U);
    multiply(1);
  }
  if (wave > 0) {
#pragma unroll
    for (int j = 0; j < NF; ++j)
#pragma unroll
      for (int r = 0; r < 4; ++r) red[(((wave - 1) * NF + j) * 4 + r) * 64 + lane] = acc[j][r];
  }
  __syncthreads();
  if (wave == 0) {
#pragma unroll
    for (int j = 0; j < NF; ++j) {
      const int e = j * 32 + col;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        float v = acc[j][r];
        for (int w = 0; w < 3; ++w) v += red[((w * NF + j) * 4 + r) * 64 + lane];
        const int t = half * 4 + r;
        if (t < n_tokens && e < n_experts) {
          logits[(long)t * n_experts + e] = v;
          if (lds_logits) lds_logits[t * n_experts + e] = v;
        }
      }
    }
  }
  __syncthreads();
}

// bf16 layers: a block takes tokens_per_block (at most 32) tokens and all experts; both operands are K-contiguous
// rows, so lanes load MFMA fragments straight from global memory (token or expert row = lane%32, 8 k values
// at 8*(lane/32)).  The 4 waves split K and meet in LDS.  NF = ceil(E/32) expert fragments.  The launch gives a
// block fewer than 32 tokens when that is what it takes to have blocks for half of the CUs (the rows of the MFMA
// that stay empty cost nothing; a token's sum runs in the same order whatever the block holds).
template <int NF>
__device__ __forceinline__ void router_logits_tokens(const bf16_t* __restrict__ x, const bf16_t* __restrict__ w_g,
                                                     int n_tokens, int n_experts, int hidden,
                                                     float* __restrict__ logits, int tokens_per_block,
                                                     float* lds_logits) {
  __shared__ float red[3 * NF * 16 * 64];
  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64, half = lane / 32, col = lane % 32;
  const long t0 = (long)blockIdx.x * tokens_per_block;
  const int kt = hidden / 16, per_wave = (kt + 3) / 4;
  const int kb0 = min(wave * per_wave, kt), kb1 = min(kb0 + per_wave, kt);
  const bool has_tok = col < tokens_per_block && t0 + col < n_tokens;
  const u32x4* xp = (const u32x4*)(x + (t0 + (has_tok ? col : 0)) * hidden) + half;
  const u32x4* wp[NF];
  bool has_exp[NF];
#pragma unroll
  for (int j = 0; j < NF; ++j) {
    has_exp[j] = j * 32 + col < n_experts;
    wp[j] = (const u32x4*)(w_g + (long)(has_exp[j] ? j * 32 + col : 0) * hidden) + half;
  }
  f32x16_t acc[NF];
#pragma unroll
  for (int j = 0; j < NF; ++j) acc[j] = f32x16_t{0};
  // two register sets of U k-tiles alternate: the loads of one are in flight while the other is multiplied
  constexpr int U = NF == 1 ? 8 : NF == 2 ? 4 : NF == 4 ? 2 : 1;
  u32x4 xa[2][U], wb[2][U][NF];
  auto load = [&](int set, int kb) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const bool in_range = kb + u < kb1;
      xa[set][u] = (in_range && has_tok) ? xp[(long)(kb + u) * 2] : u32x4{0, 0, 0, 0};
#pragma unroll
      for (int j = 0; j < NF; ++j)
        wb[set][u][j] = (in_range && has_exp[j]) ? wp[j][(long)(kb + u) * 2] : u32x4{0, 0, 0, 0};
    }
  };
  auto multiply = [&](int set) {
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int j = 0; j < NF; ++j) acc[j] = mfma_32x32x16_bf16(xa[set][u], wb[set][u][j], acc[j]);
  };
  load(0, kb0);
  for (int kb = kb0; kb < kb1; kb += 2 * U) {
    load(1, kb + U);
    multiply(0);
    load(0, kb + 2 * U);
    multiply(1);
  }
  if (wave > 0) {
#pragma unroll
    for (int j = 0; j < NF; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) red[(((wave - 1) * NF + j) * 16 + r) * 64 + lane] = acc[j][r];
  }
  __syncthreads();
  if (wave == 0) {
#pragma unroll
    for (int j = 0; j < NF; ++j) {
      const int e = j * 32 + col;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float v = acc[j][r];
        for (int w = 0; w < 3; ++w) v += red[((w * NF + j) * 16 + r) * 64 + lane];
        const int row = (r / 4) * 8 + half * 4 + (r % 4);
        const long t = t0 + row;
        if (row < tokens_per_block && t < n_tokens && e < n_experts) {
          logits[t * n_experts + e] = v;
          if (lds_logits) lds_logits[row * n_experts + e] = v;
        }
      }
    }
  }
  __syncthreads();  // the LDS copy of the logits is complete
}

}  // namespace hmoe
