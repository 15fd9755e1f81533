// Prefill FFN (HMOE_FFN_TILED): grouped GEMM on bf16 MFMA with LDS-staged tiles.
//
// Two launches per call:  h = silu(X Wgate^T) * (X Wup^T)   and   O = h Wdown^T,
// each a grouped GEMM  C[rows of expert e, N] = A[rows, K] * W_e[N, K]^T  over the ragged row
// groups that the permutation produced (expert_offsets), with W_e found through the
// expert-id -> slot table.  All dispatch happens on the device: a block turns its index into
// (expert, m-tile, n-tile) by walking expert_offsets, so the host never reads the routing result.
//
// Block tile BM x BN, K step 64, WM x WN waves, each wave owns (BM/WM) x (BN/WN) of the tile as
// 32x32x16 bf16 MFMA fragments with fp32 accumulators.
//   * Weights arrive pre-tiled (packed slot layout): a 32-row x 16-k tile is 1 KiB in MFMA operand
//     order, so it is copied to LDS verbatim and read back with one conflict-free 16-byte read per
//     lane.
//   * Activation rows are row-major; they are stored in LDS with their 16-byte chunks XOR-swizzled
//     by (row/2)%8 so that both the stores and the fragment reads spread over all banks.
//   * Global loads of K step t+1 are issued before the MFMAs of step t and written to the other LDS
//     buffer afterwards (one barrier per K step).
//   * Gate and up rows are interleaved in 32-row groups, so a wave's even fragments are gate and
//     its odd fragments the matching up columns: SwiGLU is applied to registers.
//   * Tiles are numbered expert-major, then n-tile, then m-tile, and block ids are dealt to the
//     8 XCDs in contiguous ranges so that blocks sharing a weight panel share an L2.
#include <algorithm>

#include "common.h"

namespace hmoe {

constexpr int BK = 64;  // K elements per step

struct TiledCtx {
  const int32_t* offsets;
  const int32_t* slot_of;
  const char* slots;
  size_t slot_bytes;
  ActiveMask active;
  int n_experts, hidden, ffn;
  int n_tiles_n;  // n-tiles per expert
  int grid_padded;
};

template <bool GATEUP, int BM, int BN, int WM, int WN>
__global__ __launch_bounds__(64 * WM * WN) void ffn_tiled_kernel(TiledCtx c, const bf16_t* __restrict__ in,
                                                                  bf16_t* __restrict__ out) {
  constexpr int NT = 64 * WM * WN;         // threads
  constexpr int WTM = BM / WM, WTN = BN / WN;
  constexpr int FM = WTM / 32, FN = WTN / 32;
  constexpr int A_CHUNKS = BM * (BK / 8) / NT;   // 16-byte chunks per thread per step
  constexpr int B_CHUNKS = BN * (BK / 8) / NT;
  static_assert(FM >= 1 && FN >= 1 && A_CHUNKS >= 1 && B_CHUNKS >= 1, "tile too small for the block");
  static_assert(!GATEUP || FN % 2 == 0, "a wave needs gate/up fragment pairs");
  __shared__ u32x4 lds_a[2][BM * BK / 8];
  __shared__ u32x4 lds_b[2][BN * BK / 8];

  // ---- which tile -------------------------------------------------------------------
  // XCD-aware numbering: hardware deals consecutive block ids round-robin to the 8 XCDs;
  // give each XCD one contiguous range of the logical tile list.
  const int per_xcd = c.grid_padded / 8;
  const int tile_id = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  int e = -1, row_first = 0, m_rows = 0, mt = 0, nt = 0;
  {
    int cum = 0;
    for (int i = 0; i < c.n_experts; ++i) {
      const int r0 = c.offsets[i], r1 = c.offsets[i + 1];
      if (r1 <= r0 || !c.active.test(i) || c.slot_of[i] < 0) continue;
      const int mts = (r1 - r0 + BM - 1) / BM;
      const int tiles = mts * c.n_tiles_n;
      if (tile_id < cum + tiles) {
        const int within = tile_id - cum;
        e = i; row_first = r0; m_rows = r1 - r0;
        nt = within / mts; mt = within % mts;
        break;
      }
      cum += tiles;
    }
  }
  if (e < 0) return;  // uniform

  const int K = GATEUP ? c.hidden : c.ffn;
  const int n_out = GATEUP ? c.ffn : c.hidden;   // row length of out
  const int n_groups = (GATEUP ? 2 * c.ffn : c.hidden) / TILE_N;  // packed 32-row groups of W
  const int kt16 = K / TILE_K;
  const char* slot = c.slots + (size_t)c.slot_of[e] * c.slot_bytes;
  const u32x4* w = GATEUP ? (const u32x4*)slot : (const u32x4*)(slot + 4 * (size_t)c.ffn * c.hidden);
  const int group0 = nt * (BN / TILE_N);
  const int m0 = mt * BM;  // first row of the tile within the expert

  const int tid = threadIdx.x, wave = tid / 64, lane = tid % 64;
  const int wm = wave / WN, wn = wave % WN;
  const int half = lane / 32, col = lane % 32;

  // ---- global -> register staging -----------------------------------------------------
  u32x4 ra[A_CHUNKS], rb[B_CHUNKS];
  const u32x4* a_src[A_CHUNKS];
  bool a_ok[A_CHUNKS];
  int a_dst[A_CHUNKS];
#pragma unroll
  for (int i = 0; i < A_CHUNKS; ++i) {
    const int ci = tid + i * NT, r = ci / 8, cc = ci % 8;
    a_ok[i] = m0 + r < m_rows;
    a_src[i] = (const u32x4*)(in + (size_t)(row_first + m0 + (a_ok[i] ? r : 0)) * K) + cc;
    a_dst[i] = r * 8 + (cc ^ ((r >> 1) & 7));
  }
  const u32x4* b_src[B_CHUNKS];
  bool b_ok[B_CHUNKS];
#pragma unroll
  for (int i = 0; i < B_CHUNKS; ++i) {
    const int ci = tid + i * NT, g = ci / 256, within = ci % 256;  // 256 chunks = 4 tiles of one group
    b_ok[i] = group0 + g < n_groups;
    b_src[i] = w + ((size_t)(b_ok[i] ? group0 + g : 0) * kt16) * 64 + within;
  }
  auto load_step = [&](int kstep) {
#pragma unroll
    for (int i = 0; i < A_CHUNKS; ++i) ra[i] = a_ok[i] ? a_src[i][(size_t)kstep * (BK / 8)] : u32x4{0, 0, 0, 0};
#pragma unroll
    for (int i = 0; i < B_CHUNKS; ++i) rb[i] = b_ok[i] ? b_src[i][(size_t)kstep * 256] : u32x4{0, 0, 0, 0};
  };
  auto store_step = [&](int buf) {
#pragma unroll
    for (int i = 0; i < A_CHUNKS; ++i) lds_a[buf][a_dst[i]] = ra[i];
#pragma unroll
    for (int i = 0; i < B_CHUNKS; ++i) lds_b[buf][tid + i * NT] = rb[i];
  };

  f32x16_t acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j) acc[i][j] = f32x16_t{0};

  const int k_steps = K / BK;
  load_step(0);
  store_step(0);
  __syncthreads();
  for (int ks = 0; ks < k_steps; ++ks) {
    const int buf = ks & 1;
    if (ks + 1 < k_steps) load_step(ks + 1);
#pragma unroll
    for (int kk = 0; kk < BK / TILE_K; ++kk) {
      u32x4 fa[FM], fb[FN];
#pragma unroll
      for (int i = 0; i < FM; ++i) {
        const int r = wm * WTM + i * 32 + col;
        fa[i] = lds_a[buf][r * 8 + ((kk * 2 + half) ^ ((r >> 1) & 7))];
      }
#pragma unroll
      for (int j = 0; j < FN; ++j) fb[j] = lds_b[buf][((wn * FN + j) * 4 + kk) * 64 + lane];
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) acc[i][j] = mfma_32x32x16_bf16(fa[i], fb[j], acc[i][j]);
    }
    if (ks + 1 < k_steps) store_step(buf ^ 1);
    __syncthreads();
  }

  // ---- epilogue -----------------------------------------------------------------------
  // accumulator register r of lane (half, col): row 8*(r/4) + 4*half + r%4, column col
#pragma unroll
  for (int i = 0; i < FM; ++i) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int m = m0 + wm * WTM + i * 32 + (r / 4) * 8 + half * 4 + (r % 4);
      if (m >= m_rows) continue;
      bf16_t* orow = out + (size_t)(row_first + m) * n_out;
      if (GATEUP) {
#pragma unroll
        for (int j = 0; j < FN; j += 2) {
          const int f = nt * (BN / 2) + ((wn * FN + j) / 2) * 32 + col;
          if (f < n_out) orow[f] = f32_to_bf16(silu_f32(acc[i][j][r]) * acc[i][j + 1][r]);
        }
      } else {
#pragma unroll
        for (int j = 0; j < FN; ++j) {
          const int n = nt * BN + (wn * FN + j) * 32 + col;
          if (n < n_out) orow[n] = f32_to_bf16(acc[i][j][r]);
        }
      }
    }
  }
}

template <bool GATEUP, int BM, int BN, int WM, int WN>
static void launch_cfg(TiledCtx c, int n_rows, const bf16_t* in, bf16_t* out, hipStream_t s) {
  const int n_total = GATEUP ? 2 * c.ffn : c.hidden;
  c.n_tiles_n = (n_total + BN - 1) / BN;
  const int busy_max = std::min(c.n_experts, n_rows);
  const long m_tiles_max = n_rows / BM + busy_max;  // sum over experts of ceil(rows/BM) is at most this
  const long tiles = m_tiles_max * c.n_tiles_n;
  c.grid_padded = (int)((tiles + 7) / 8 * 8);
  hipLaunchKernelGGL((ffn_tiled_kernel<GATEUP, BM, BN, WM, WN>), dim3((unsigned)c.grid_padded), dim3(64 * WM * WN), 0, s,
                     c, in, out);
}

int launch_ffn_tiled(const FfnArgs& a) {
  const hmoe_layer_desc& d = *a.desc;
  if (d.dtype != HMOE_BF16) return HMOE_ERR_UNSUPPORTED;
  if (a.n_rows == 0) return HMOE_OK;
  TiledCtx c{a.offsets, a.slot_of, a.slots, a.slot_bytes, a.active, d.n_experts, d.hidden, d.ffn, 0, 0};
  const bf16_t* x = (const bf16_t*)a.x_perm;
  bf16_t* h = (bf16_t*)a.h;
  bf16_t* o = (bf16_t*)a.o_perm;
  const int avg_rows = a.n_rows / std::min(d.n_experts, std::max(1, a.n_rows));
  probe_before(a.stream);
  if (avg_rows >= 192) launch_cfg<true, 256, 256, 2, 4>(c, a.n_rows, x, h, a.stream);
  else launch_cfg<true, 128, 256, 2, 4>(c, a.n_rows, x, h, a.stream);
  probe_after(a.stream);
  if (avg_rows >= 192) launch_cfg<false, 256, 256, 2, 4>(c, a.n_rows, h, o, a.stream);
  else launch_cfg<false, 128, 256, 2, 4>(c, a.n_rows, h, o, a.stream);
  HMOE_HIP(hipGetLastError());
  return HMOE_OK;
}

}  // namespace hmoe
