// Prefill FFN over 4-bit expert weights (HMOE_BF16_W4, HMOE_FFN_TILED): the grouped GEMM of ffn_tiled.hip
// with the arithmetic of the 4-bit decode kernel.
//
// Tile: 64 rows of one expert x 256 packed weight rows (gate/up: 128 features as 8 gate/up pairs of 16; down:
// 256 output columns), 8 waves.  A wave owns two packed 16-row units of the weight matrix and all 64 rows, as
// 4 x 2 accumulator tiles of v_mfma_f32_16x16x32_bf16 (tokens are the A operand, weights the B operand); twice
// the running sums (one set per scale group, one for the result) make 128 rows too many registers.
//   * K advances one scale group (128 k) per step.  The activation tile of a step (64 rows x 128 k, 16 KiB)
//     sits in LDS, two stages; the following two travel global -> registers -> LDS while this one is multiplied.
//     A row is 16 chunks of 16 bytes; chunk c of row r is stored at position c ^ (r % 16), so the 16 lanes
//     that read the same k block of 16 consecutive rows hit all banks.
//   * The codes of a unit and group are 1 KiB (16 bytes per lane) in operand order and go from global memory
//     to registers, four groups ahead; one bfloat16 scale per lane (= per weight row) and group with them.
//   * As in the decode kernel a dword of eight codes becomes the four operand registers of bfloat16 values
//     128 + q, and   sum_k x_k (q_k - 8) = sum_k x_k (128 + q_k) - 136 sum_k x_k.   The row sums of the
//     activation tile are the same for all waves: wave w < 4 computes those of rows 16 w .. + 16 with one MFMA per
//     k-step against a tile of ones and leaves them in LDS.  They are needed when a group's partial sums are
//     folded into the running result, and that is done after the next block barrier (at the start of the next
//     step), so no barrier is added for them.
//   * Rows past the end of the expert and units past the end of the matrix are computed from clamped
//     addresses and never stored.
#include <stdlib.h>

#include <algorithm>

#include "common.h"
#include "tile_locate.h"

namespace hmoe {

constexpr int W4T_WAVES = 8;
constexpr int W4T_NU = 2;        // packed 16-row units per wave
constexpr int W4T_UNITS = W4T_WAVES * W4T_NU;  // per tile: 256 packed rows

// W4T_BM: rows per tile (a multiple of 32); W4T_RING: scale groups of codes in flight per wave
template <bool GATEUP, int W4T_BM, int W4T_RING>
__global__ __launch_bounds__(64 * W4T_WAVES) void ffn_tile_w4_kernel(TiledCtx c, const bf16_t* __restrict__ in,
                                                                      bf16_t* __restrict__ out) {
  static_assert(W4T_RING % 2 == 0, "the two activation register sets alternate with the unrolled steps");
  constexpr int W4T_FM = W4T_BM / 16;
  constexpr int W4T_CHUNKS = W4T_BM * 16;                       // 16-byte chunks of an activation stage
  constexpr int W4T_COPIES = W4T_CHUNKS / (64 * W4T_WAVES);     // per thread and stage
  __shared__ u32x4 a_lds[2][W4T_CHUNKS];
  __shared__ __attribute__((aligned(16))) float xs[2][W4T_BM];
  TileLoc loc;
  if (!locate_tile<W4T_BM>(c, loc)) return;  // uniform over the block
  const int K = GATEUP ? c.hidden : c.ffn;
  const int n_out = GATEUP ? c.ffn : c.hidden;
  const int n_groups = K / W4_GROUP;
  const int units_total = (GATEUP ? 2 * c.ffn : c.hidden) / 16;
  const int m0 = loc.mt * W4T_BM;
  const int tid = threadIdx.x, wave = tid / 64, lane = tid % 64;
  const int j = lane % 16, kblk = lane / 16;

  const char* slot = c.slots + (size_t)loc.slot * c.slot_bytes;
  const W4Offsets off = w4_offsets((size_t)c.hidden, (size_t)c.ffn);
  const u32x4* units = (const u32x4*)(slot + (GATEUP ? 0 : off.down_units));
  const bf16_t* scales = (const bf16_t*)(slot + (GATEUP ? off.gate_up_scales : off.down_scales));
  const u32x4* wq[W4T_NU];
  const bf16_t* ws[W4T_NU];
  const int unit0 = loc.nt * W4T_UNITS + wave * W4T_NU;  // gate/up: the gate and up unit of features 8 * unit0 .. + 16
#pragma unroll
  for (int u = 0; u < W4T_NU; ++u) {
    const size_t unit = unit0 + u < units_total ? unit0 + u : 0;  // clamped: never stored
    wq[u] = units + unit * (size_t)n_groups * 64 + lane;
    ws[u] = scales + unit * (size_t)n_groups * 16 + j;
  }
  // the W4T_COPIES chunks of an activation stage this thread moves: chunk id = i * 512 + tid -> row id / 16, k chunk id % 16
  const u32x4* a_src[W4T_COPIES];
  int a_dst[W4T_COPIES];
#pragma unroll
  for (int i = 0; i < W4T_COPIES; ++i) {
    const int id = i * 64 * W4T_WAVES + tid;
    const int r = id / 16, ch = id % 16;
    const int row = m0 + r < loc.m_rows ? m0 + r : loc.m_rows - 1;  // clamped: never stored
    const int in_row = GATEUP ? mapped_row(c.row_map, c.map_div, loc.row_first + row) : loc.row_first + row;
    a_src[i] = (const u32x4*)(in + (size_t)in_row * K) + ch;
    a_dst[i] = r * 16 + (ch ^ (r % 16));
  }

  u32x4 codes[W4T_RING][W4T_NU];
  uint32_t scale_bits[W4T_RING][W4T_NU];  // raw bfloat16, converted at use
  auto load_codes = [&](int ring_slot, int g) {
    const int gc = g < n_groups ? g : n_groups - 1;  // clamped: a group past the end is never multiplied
#pragma unroll
    for (int u = 0; u < W4T_NU; ++u) {
      codes[ring_slot][u] = __builtin_nontemporal_load(wq[u] + (size_t)gc * 64);
      scale_bits[ring_slot][u] = (uint32_t)ws[u][(size_t)gc * 16];
    }
  };

  f32x4_t acc[W4T_FM][W4T_NU], part[W4T_FM][W4T_NU];
#pragma unroll
  for (int i = 0; i < W4T_FM; ++i)
#pragma unroll
    for (int u = 0; u < W4T_NU; ++u) acc[i][u] = part[i][u] = f32x4_t{0, 0, 0, 0};
  float sc_prev[W4T_NU] = {0.0f, 0.0f};
  const u32x4 ones = {0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u};

  // acc += scale * (part - 136 * row sums) for row fragment i of the group whose partial sums `part` holds
  auto fold = [&](int i, const f32x4_t xv) {
#pragma unroll
    for (int u = 0; u < W4T_NU; ++u)
#pragma unroll
      for (int r = 0; r < 4; ++r) acc[i][u][r] += sc_prev[u] * (part[i][u][r] - 136.0f * xv[r]);
  };
  // accumulator register r is row 4 kblk + r of its 16-row fragment
  auto row_sums = [&](int stage, int i) { return *(const f32x4_t*)&xs[stage][i * 16 + 4 * kblk]; };

  // the four operand registers (bfloat16 values 128 + q) of one k-step from its dword of eight codes
  // (the mask lives in a vector register the compiler cannot see through: an and-or with two literal constants
  // would need two instructions, with one operand in a register it is one)
  uint32_t nibbles;
  asm volatile("v_mov_b32 %0, 0x000f000f" : "=v"(nibbles));
  auto unpack = [nibbles](uint32_t d) {
    return u32x4{(d & nibbles) | 0x43004300u, ((d >> 4) & nibbles) | 0x43004300u, ((d >> 8) & nibbles) | 0x43004300u,
                 ((d >> 12) & nibbles) | 0x43004300u};
  };
  u32x4 w[2][W4T_NU], fa[2][W4T_FM];

  // ---- prologue: codes of the first groups, activation stage 0 ----------------------------------
#pragma unroll
  for (int s = 0; s < W4T_RING; ++s) load_codes(s, s);
  // activation stages travel two steps ahead: the loads of step g + 2 are issued when step g starts and reach LDS
  // when step g + 1 ends, so a load has two steps of multiplying to arrive
  u32x4 ahead[2][W4T_COPIES];
  auto load_stage = [&](int set, int g) {
    const int gc = g < n_groups ? g : n_groups - 1;  // clamped: never multiplied
#pragma unroll
    for (int i = 0; i < W4T_COPIES; ++i) ahead[set][i] = a_src[i][(size_t)gc * 16];
  };
  load_stage(0, 0);
  load_stage(1, 1);
#pragma unroll
  for (int i = 0; i < W4T_COPIES; ++i) a_lds[0][a_dst[i]] = ahead[0][i];
  if (tid < W4T_BM) xs[1][tid] = 0.0f;  // the first step folds an empty group: scale 0, partial sums 0, these row sums
#pragma unroll
  for (int u = 0; u < W4T_NU; ++u) w[0][u] = unpack(codes[0][u][0]);
  __builtin_amdgcn_sched_barrier(0);
  __syncthreads();

  for (int g0 = 0; g0 < n_groups; g0 += W4T_RING) {
#pragma unroll
    for (int rs = 0; rs < W4T_RING; ++rs) {
      const int g = g0 + rs;
      if (g < n_groups) {  // uniform
        const int stage = g & 1;
        const bool more = g + 1 < n_groups;
        load_stage(rs & 1, g + 2);  // this register set's previous content (step g) is in LDS
        f32x4_t xv[W4T_FM];  // row sums of the previous group, for its fold below
#pragma unroll
        for (int i = 0; i < W4T_FM; ++i) xv[i] = row_sums(stage ^ 1, i);
        __builtin_amdgcn_sched_barrier(0);
        // row sums of this stage: rows 16 * wave .. + 16
        if (wave < W4T_FM) {
          f32x4_t xsum = {0, 0, 0, 0};
#pragma unroll
          for (int t = 0; t < 4; ++t)
            xsum = mfma_16x16x32_bf16(a_lds[stage][(wave * 16 + j) * 16 + ((t * 4 + kblk) ^ j)], ones, xsum);
          if (j == 0) *(f32x4_t*)&xs[stage][wave * 16 + 4 * kblk] = xsum;  // every column holds the same sums
        }
        // this group's partial sums.  The previous group is folded into the running result fragment by fragment
        // right before the first k-step overwrites that fragment's partial sums, and the operand registers of
        // k-step t + 1 are unpacked during k-step t; the scheduling hints deal the vector ALU instructions out
        // between the matrix instructions.  (Measured on this part: a SIMD overlaps about one vector ALU
        // instruction with each matrix instruction and no more, so the time of a step is close to the sum of
        // the two kinds; what limits this kernel is the count of vector ALU instructions per matrix instruction
        // -- 7 per k-step and unit to unpack, 2 per accumulator register and group to fold.)
        // (activation fragments are read one k-step ahead as well: an LDS read takes longer than the two matrix
        // instructions it feeds)
        auto read_frags = [&](int set, int t) {
#pragma unroll
          for (int i = 0; i < W4T_FM; ++i) fa[set][i] = a_lds[stage][(i * 16 + j) * 16 + ((t * 4 + kblk) ^ j)];
        };
        read_frags(0, 0);
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          if (t < 3) read_frags((t + 1) & 1, t + 1);
          // operand registers of the next k-step: the next dword of this group, or the first of the next group
#pragma unroll
          for (int u = 0; u < W4T_NU; ++u) w[(t + 1) & 1][u] = unpack(t < 3 ? codes[rs][u][t + 1] : codes[(rs + 1) % W4T_RING][u][0]);
#pragma unroll
          for (int i = 0; i < W4T_FM; ++i) {
            if (t == 0) fold(i, xv[i]);
#pragma unroll
            for (int u = 0; u < W4T_NU; ++u)  // the first k-step of a group starts its partial sums
              part[i][u] = mfma_16x16x32_bf16(fa[t & 1][i], w[t & 1][u], t == 0 ? f32x4_t{0, 0, 0, 0} : part[i][u]);
          }
#pragma unroll
          for (int i = 0; i < W4T_FM; ++i) {
            if (t < 3) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // one fragment read for the next k-step
#pragma unroll
            for (int u = 0; u < W4T_NU; ++u) {
              if (t == 0) __builtin_amdgcn_sched_group_barrier(0x002, 10, 0);  // vector ALU: unpacking, and the fold
              else __builtin_amdgcn_sched_group_barrier(0x002, 2, 0);
              __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                // one matrix instruction
            }
          }
          __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int u = 0; u < W4T_NU; ++u) sc_prev[u] = __uint_as_float(scale_bits[rs][u] << 16);
        __builtin_amdgcn_sched_barrier(0);
        // the other stage was last read in the previous step, before the barrier that opened this one
        if (more) {
#pragma unroll
          for (int i = 0; i < W4T_COPIES; ++i) a_lds[stage ^ 1][a_dst[i]] = ahead[(rs + 1) & 1][i];
        }
        load_codes(rs, g + W4T_RING);
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
      }
    }
  }
#pragma unroll
  for (int i = 0; i < W4T_FM; ++i) fold(i, row_sums((n_groups - 1) & 1, i));

  // ---- epilogue: accumulator register r of lane (j, kblk) is row 16 i + 4 kblk + r, weight row j of the unit ----
  // A wave's results are 16 (gate/up) or 32 (down) columns wide, a fraction of a 128-byte line.  The tile's results
  // are collected as bf16 in the idle activation stages, [rows][OUTC columns], and stored as whole lines, 16 bytes per
  // thread.  Units past the end (gate/up and down both hold an even number: a wave's pair is all or nothing) are
  // neither collected nor stored.
  constexpr int OUTC = GATEUP ? W4T_WAVES * 16 : W4T_WAVES * 32;
  static_assert(W4T_BM * OUTC * 2 <= 2 * W4T_CHUNKS * 16, "the tile's results must fit the activation stages");
  bf16_t* staged = (bf16_t*)&a_lds[0][0];
  __syncthreads();  // every wave has read its last activation fragments
  if (unit0 < units_total) {
#pragma unroll
    for (int i = 0; i < W4T_FM; ++i) {
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        bf16_t* srow = staged + (i * 16 + 4 * kblk + r) * OUTC;
        if (GATEUP) {
          srow[wave * 16 + j] = f32_to_bf16(silu_f32(acc[i][0][r]) * acc[i][1][r]);
        } else {
          srow[wave * 32 + j] = f32_to_bf16(acc[i][0][r]);
          srow[wave * 32 + 16 + j] = f32_to_bf16(acc[i][1][r]);
        }
      }
    }
  }
  __syncthreads();
  const int col0 = loc.nt * OUTC;
#pragma unroll
  for (int id = tid; id < W4T_BM * OUTC / 8; id += 64 * W4T_WAVES) {
    const int row = id / (OUTC / 8), cc = (id % (OUTC / 8)) * 8;
    const int m = m0 + row;
    if (m < loc.m_rows && col0 + cc < n_out)
      *(u32x4*)(out + (size_t)(loc.row_first + m) * n_out + col0 + cc) = *(const u32x4*)(staged + row * OUTC + cc);
  }
}

template <bool GATEUP, int BM, int RING>
static void launch_stage_tile_w4(TiledCtx c, int n_rows, const bf16_t* in, bf16_t* out, hipStream_t s) {
  const int units_total = (GATEUP ? 2 * c.ffn : c.hidden) / 16;
  c.n_tiles_n = (units_total + W4T_UNITS - 1) / W4T_UNITS;
  c.grid_padded = (int)((tiles_upper_bound(c, n_rows, BM) + 7) / 8 * 8);
  hipLaunchKernelGGL((ffn_tile_w4_kernel<GATEUP, BM, RING>), dim3((unsigned)c.grid_padded), dim3(64 * W4T_WAVES), 0, s, c, in, out);
}

int launch_ffn_tiled_w4(const FfnArgs& a) {
  const hmoe_layer_desc& d = *a.desc;
  if (d.dtype != HMOE_BF16_W4) return HMOE_ERR_UNSUPPORTED;
  if (a.n_rows == 0) return HMOE_OK;
  TiledCtx c{a.offsets, a.slot_of, a.slots, a.slot_bytes, a.active, d.n_experts, d.hidden, d.ffn, 0, 0, a.row_map, a.map_div};
  probe_before(a.stream);
  launch_stage_tile_w4<true, 64, 4>(c, a.n_rows, (const bf16_t*)a.x_perm, (bf16_t*)a.h, a.stream);
  probe_after(a.stream);
  probe_before(a.stream);
  launch_stage_tile_w4<false, 64, 4>(c, a.n_rows, (const bf16_t*)a.h, (bf16_t*)a.o_perm, a.stream);
  probe_after(a.stream);
  HMOE_HIP(hipGetLastError());
  return HMOE_OK;
}

}  // namespace hmoe
