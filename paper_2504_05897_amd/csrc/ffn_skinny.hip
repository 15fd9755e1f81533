// Decode FFN (HMOE_FFN_SKINNY): every touched expert's weights are streamed from HBM exactly
// once, straight into MFMA operand registers.
//
// With a handful of rows per expert the expert FFN is bound by reading its weights (the paper
// observes GPU expert time flat in the workload at small batch, Section III / Fig. 3(f)), so the
// kernel is organised around the weight stream:
//   * a block owns `gpb` consecutive 32-row groups of one matrix of one expert (for gate/up: the
//     matching gate and up groups); its NW waves split K in batches of U tiles dealt round-robin, so
//     at any moment the block reads one contiguous stretch of the group's stream (measured 3-5 %
//     faster than a contiguous K range per wave: consecutive tiles share DRAM pages);
//   * a tile is one fully coalesced 16-byte non-temporal load per lane and is already in 32x32x16
//     bf16 MFMA operand order (packed slot layout), so it goes from HBM to the matrix core through
//     registers only; two register sets of U tiles alternate, so U tiles per matrix are always in
//     flight per wave, across group boundaries too;
//   * tokens ride along as the other MFMA operand (up to MR rows, zero padded), read from the
//     L1/L2-resident activation rows;
//   * at the end of a group the waves' partial sums meet in LDS (double buffered, one barrier per
//     group); wave 0 applies SwiGLU / rounds and stores.
#include <stdio.h>
#include <stdlib.h>

#include <algorithm>

#include "common.h"

namespace hmoe {

// A dense FFN over the first `rows` rows of its own input that rides along in the launches of the routed
// experts (the shared experts of a layer, Section II-A): the first grid_rows grid rows hold its 32-row
// groups, gridDim.x of them per grid row, the routed experts follow.  Its blocks come first because they are
// dispatched first and may be the longest of the launch (the down projection's K is the dense FFN's width).
// grid_rows == 0: none.
struct SkinnyShared {
  const char* slot;     // packed weights
  const bf16_t* x;      // [rows, H]
  bf16_t* h;            // [rows, ffn]
  bf16_t* o;            // [rows, H]
  int ffn, rows, grid_rows;
};

// The weighted sum of Eq. (1) inside the down projection's launch (decode batches).  Every block that has stored
// its piece of o_perm / o_shared (device-scope stores) draws a ticket from the counter of its column block; the block
// that draws the last one finds all pieces of those columns complete and adds them up, for every token, in the order of hmoe_combine
// (j ascending, then the shared term; the bf16 values that were stored), so y has the bits of the separate call.
// No block waits for another.  The counters are zero when the launch starts and the last block leaves them zero.
// on == 0: none.
struct SkinnyCombine {
  const int32_t* inv_perm;
  const float* topk_w;
  const bf16_t* o_perm;     // [A, H], what the routed blocks store
  const bf16_t* o_shared;   // [T, H] or NULL
  bf16_t* y;                // [T, H]
  unsigned int* tickets;    // one counter per column block
  int n_tokens, top_k, on;
};

struct SkinnyCtx {
  const int32_t* offsets;
  const int32_t* slot_of;
  const char* slots;
  size_t slot_bytes;
  ActiveMask active;
  int n_experts, hidden, ffn;
  int gpb;  // 32-row groups per block
  const int32_t* row_map;  // gate/up only: input row of sorted row p is row_map[p] / map_div
  int map_div;
  SkinnyShared shared;
  SkinnyCombine combine;
};

// number of experts that are active, resident and have rows
__device__ __forceinline__ int count_busy_experts(const SkinnyCtx& c, int lane) {
  int seen = 0;
  for (int base = 0; base < c.n_experts; base += 64) {
    const int e = base + lane;
    const bool busy = e < c.n_experts && c.active.test(e) && c.slot_of[e] >= 0 && c.offsets[e + 1] > c.offsets[e];
    seen += __popcll(__ballot(busy));
  }
  return seen;
}

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
// NW waves per block, MR = rows kept per pass (8 or 32), U = tiles per register set and matrix.
template <bool GATEUP, int NW, int MR, int U>
__global__ __launch_bounds__(64 * NW) void ffn_skinny_kernel(SkinnyCtx c, const bf16_t* __restrict__ in,
                                                              bf16_t* __restrict__ out) {
  constexpr int NMAT = GATEUP ? 2 : 1;
  constexpr int RR = MR == 8 ? 4 : 16;  // accumulator registers that can hold valid rows
  constexpr int RED = (NW > 1 ? NW - 1 : 1) * NMAT * RR * 64;
  __shared__ float red[2][RED];

  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
  // what this block works on: a routed expert's rows, or (the first shared.grid_rows grid rows) the dense FFN
  // that shares the launch.  Everything below is uniform over the block.
  const bool dense = (int)blockIdx.y < c.shared.grid_rows;
  int row_first, row_end, ffn, block_in_matrix;
  const char* slot;
  const int32_t* row_map = nullptr;
  if (dense) {
    row_first = 0;
    row_end = c.shared.rows;
    ffn = c.shared.ffn;
    slot = c.shared.slot;
    block_in_matrix = (int)blockIdx.y * (int)gridDim.x + (int)blockIdx.x;
    in = GATEUP ? c.shared.x : c.shared.h;
    out = GATEUP ? c.shared.h : c.shared.o;
  } else {
    const int e = nth_busy_expert(c, (int)blockIdx.y - c.shared.grid_rows, lane);
    if (e < 0) return;
    row_first = c.offsets[e];
    row_end = c.offsets[e + 1];
    ffn = c.ffn;
    slot = c.slots + (size_t)c.slot_of[e] * c.slot_bytes;
    block_in_matrix = blockIdx.x;
    row_map = c.row_map;
  }
  const int K = GATEUP ? c.hidden : ffn;        // reduction length
  const int n_out = GATEUP ? ffn : c.hidden;    // row length of `out`
  const int kt = K / TILE_K;
  const int g_begin = block_in_matrix * c.gpb, g_end = min(g_begin + c.gpb, n_out / TILE_N);
  if (g_begin >= g_end) return;
  const u32x4* wbase = GATEUP ? (const u32x4*)slot : (const u32x4*)(slot + 4 * (size_t)ffn * c.hidden);
  const size_t group_stride = (size_t)kt * 64 * NMAT;  // u32x4 per group (gate/up: the pair)
  // batches of U tiles per wave and group (the last ones may lie partly or wholly past the end of K)
  const int per_wave = ((kt + NW - 1) / NW + U - 1) / U * U;
  const int bpg = per_wave / U;                    // batches per group
  const int half = lane / 32, col = lane % 32;
  const int n_batches = (g_end - g_begin) * bpg;

  for (int row0 = row_first; row0 < row_end; row0 += MR) {
    const int rows = min(MR, row_end - row0);
    const bool has_row = col < rows;
    const int in_row = GATEUP ? mapped_row(row_map, c.map_div, row0 + (has_row ? col : 0)) : row0 + (has_row ? col : 0);
    const u32x4* xin = (const u32x4*)(in + (size_t)in_row * K) + half;

    u32x4 wa[2][U], wb[2][U], xa[2][U];
    int load_g = g_begin, load_j = 0;  // cursor of the next batch to load
    auto load_batch = [&](int set, bool live) {
      const u32x4* w0 = wbase + (size_t)load_g * group_stride;
      const int kb = (load_j * NW + wave) * U;  // batches dealt round-robin: the block sweeps its stream front to back
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const bool ok = live && kb + u < kt;
        const size_t t = (size_t)(kb + u) * 64 + lane;
        wa[set][u] = ok ? __builtin_nontemporal_load(w0 + t) : u32x4{0, 0, 0, 0};
        if (GATEUP) wb[set][u] = ok ? __builtin_nontemporal_load(w0 + (size_t)kt * 64 + t) : u32x4{0, 0, 0, 0};
        xa[set][u] = (ok && has_row) ? xin[(size_t)(kb + u) * 2] : u32x4{0, 0, 0, 0};
      }
      if (++load_j == bpg) { load_j = 0; ++load_g; }
    };

    f32x16_t acc0 = {0}, acc1 = {0};
    int cur_g = g_begin, cur_j = 0;  // cursor of the batch being multiplied
    auto compute_batch = [&](int set) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        acc0 = mfma_32x32x16_bf16(xa[set][u], wa[set][u], acc0);
        if (GATEUP) acc1 = mfma_32x32x16_bf16(xa[set][u], wb[set][u], acc1);
      }
      if (++cur_j < bpg) return;
      // ---- end of a group: cross-wave reduction, epilogue, store --------------------------
      // accumulator register r of lane (half, col) is row 8*(r/4) + 4*half + r%4, output column col
      float* area = red[cur_g & 1];
      if (NW > 1 && wave > 0) {
        float* dst = area + (size_t)(wave - 1) * NMAT * RR * 64;
#pragma unroll
        for (int r = 0; r < RR; ++r) {
          if ((r / 4) * 8 < rows) {
            dst[r * 64 + lane] = acc0[r];
            if (GATEUP) dst[(RR + r) * 64 + lane] = acc1[r];
          }
        }
      }
      if (NW > 1) __syncthreads();
      if (wave == 0) {
#pragma unroll
        for (int r = 0; r < RR; ++r) {
          if ((r / 4) * 8 < rows) {
            float g = acc0[r], u = GATEUP ? acc1[r] : 0.0f;
            for (int w = 0; w < NW - 1; ++w) {
              g += area[((size_t)w * NMAT * RR + r) * 64 + lane];
              if (GATEUP) u += area[((size_t)w * NMAT * RR + RR + r) * 64 + lane];
            }
            const int m = (r / 4) * 8 + half * 4 + (r % 4);
            if (m < rows) {
              const float v = GATEUP ? silu_f32(g) * u : g;
              bf16_t* dst = out + (size_t)(row0 + m) * n_out + cur_g * TILE_N + col;
              if (!GATEUP && c.combine.on)  // read by another block of this launch: a store that is visible device-wide
                __hip_atomic_store(dst, f32_to_bf16(v), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
              else
                *dst = f32_to_bf16(v);
            }
          }
        }
      }
      acc0 = f32x16_t{0};
      acc1 = f32x16_t{0};
      cur_j = 0;
      ++cur_g;
    };

    load_batch(0, true);
    for (int b = 0; b < n_batches; b += 2) {
      load_batch(1, b + 1 < n_batches);
      compute_batch(0);
      load_batch(0, b + 2 < n_batches);
      if (b + 1 < n_batches) compute_batch(1);
    }
    if (NW > 1) __syncthreads();  // the reduction areas are reused by the next row pass
  }

  if constexpr (!GATEUP) {
    if (c.combine.on) {  // uniform over the launch
      // Wave 0 stored this block's results with device-scope stores (they go through to memory instead of staying in
      // this die's L2) and waits until all of them have been performed before it draws the ticket; the block that draws
      // the last ticket reads the others' results with device-scope loads.  (Fences would do the same for ordinary
      // stores and loads, but a device-scope fence writes back and invalidates the whole L2 of the die, in every block:
      // measured, that made the decode layers 15-55 % slower than the separate combine launch.)
      // Only wave 0 stays for this: the other waves are done, and the wave slots they free let the CU's next block
      // start while this one waits for its ticket.
      if (wave != 0) return;
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      const int expected = count_busy_experts(c, lane) + (c.shared.grid_rows > 0 ? 1 : 0);
      int ticket = 0;
      if (lane == 0)
        ticket = (int)__hip_atomic_fetch_add(&c.combine.tickets[block_in_matrix], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (__shfl(ticket, 0) == expected - 1) {
        const SkinnyCombine& cb = c.combine;
        auto load16 = [](const uint4* p) {  // 16 bytes as two device-scope 8-byte loads
          const unsigned long long* q = (const unsigned long long*)p;
          const unsigned long long lo = __hip_atomic_load(q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          const unsigned long long hi = __hip_atomic_load(q + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          return make_uint4((uint32_t)lo, (uint32_t)(lo >> 32), (uint32_t)hi, (uint32_t)(hi >> 32));
        };
        const int chunks = (g_end - g_begin) * (TILE_N / 8);  // 16-byte pieces of a row that this column block owns
        const int row_vec = c.hidden / 8;
        const uint4* o_perm = (const uint4*)cb.o_perm;
        const uint4* o_shared = (const uint4*)cb.o_shared;
        for (int id = lane; id < cb.n_tokens * chunks; id += 64) {
          const int t = id / chunks, cv = g_begin * (TILE_N / 8) + id % chunks;
          float acc[8];
#pragma unroll
          for (int i = 0; i < 8; ++i) acc[i] = 0.0f;
          for (int j = 0; j < cb.top_k; ++j) {
            const uint4 v = load16(o_perm + (long)cb.inv_perm[t * cb.top_k + j] * row_vec + cv);
            const float w = cb.topk_w[t * cb.top_k + j];
            const uint32_t u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              acc[2 * i] += w * __uint_as_float(u[i] << 16);
              acc[2 * i + 1] += w * __uint_as_float(u[i] & 0xffff0000u);
            }
          }
          if (o_shared) {
            const uint4 v = load16(o_shared + (long)t * row_vec + cv);
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
          ((uint4*)cb.y)[(long)t * row_vec + cv] = make_uint4(o[0], o[1], o[2], o[3]);
        }
        if (lane == 0)  // zero again for the next launch
          __hip_atomic_exchange(&c.combine.tickets[block_in_matrix], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
  }
}

typedef void (*skinny_launch_fn)(const SkinnyCtx&, dim3, const bf16_t*, bf16_t*, hipStream_t);
template <bool GATEUP, int NW, int MR, int U>
static void launch_one(const SkinnyCtx& c, dim3 grid, const bf16_t* in, bf16_t* out, hipStream_t s) {
  hipLaunchKernelGGL((ffn_skinny_kernel<GATEUP, NW, MR, U>), grid, dim3(64 * NW), 0, s, c, in, out);
}

// K-split widths and tile batch sizes built into the library
struct SkinnyShape { int nw, u; };
static const SkinnyShape kShapes[] = {{1, 4}, {2, 4}, {4, 4}, {8, 4}, {8, 2}, {16, 2}};
constexpr int kNumShapes = sizeof(kShapes) / sizeof(kShapes[0]);
template <bool GATEUP, int MR>
static skinny_launch_fn pick(int shape) {
  if constexpr (MR == 32) {
    // up to 32 rows: the reduction area grows with the rows, so at most 4 waves split K
    switch (kShapes[shape].nw) {
      case 1: return launch_one<GATEUP, 1, 32, 4>;
      case 2: return launch_one<GATEUP, 2, 32, 4>;
      default: return launch_one<GATEUP, 4, 32, 4>;
    }
  } else {
    switch (shape) {
      case 0: return launch_one<GATEUP, 1, MR, 4>;
      case 1: return launch_one<GATEUP, 2, MR, 4>;
      case 2: return launch_one<GATEUP, 4, MR, 4>;
      case 3: return launch_one<GATEUP, 8, MR, 4>;
      case 4: return launch_one<GATEUP, 8, MR, 2>;
      default: return launch_one<GATEUP, 16, MR, 2>;
    }
  }
}

// Work split for one of the two GEMVs: n_groups 32-row groups per expert, at most busy_max experts
// with rows.  Measured on the decode shapes, 8 waves per block with 2 tiles per register set and one
// group per block is at or near the best everywhere; very few (expert, group) tasks get 16 waves.
// n_groups_dense: 32-row groups of the dense FFN that shares the launch (0: none); they fill extra grid rows.
template <bool GATEUP>
static void launch_stage(SkinnyCtx c, int n_groups, int busy_max, int max_rows, int n_groups_dense, const bf16_t* in,
                         bf16_t* out, hipStream_t s) {
  const long tasks = (long)n_groups * busy_max + n_groups_dense;
  int shape = tasks < 200 ? 5 : 4;
  int gpb = 1;
  if (const char* env = getenv("HMOE_SKINNY")) {  // tuning override: "<shape>,<groups per block>"
    int es = -1, eg = -1;
    if (sscanf(env, "%d,%d", &es, &eg) >= 1 && es >= 0 && es < kNumShapes) shape = es;
    if (eg > 0) gpb = eg;
  }
  c.gpb = std::min(gpb, n_groups);
  const int grid_x = (n_groups + c.gpb - 1) / c.gpb;
  c.shared.grid_rows = 0;
  if (n_groups_dense > 0) {
    const int blocks_dense = (n_groups_dense + c.gpb - 1) / c.gpb;
    c.shared.grid_rows = (blocks_dense + grid_x - 1) / grid_x;
  }
  const dim3 grid((unsigned)grid_x, (unsigned)(c.shared.grid_rows + busy_max));
  (max_rows > 8 ? pick<GATEUP, 32>(shape) : pick<GATEUP, 8>(shape))(c, grid, in, out, s);
}

// dense (or NULL): a dense FFN of the same hidden size over dense->n_rows rows (one resident expert: weights
// at dense->slots, offsets {0, n_rows} implied), computed by extra blocks of the same two launches.
int launch_ffn_skinny(const FfnArgs& a, const FfnArgs* dense, const CombineArgs* combine) {
  const hmoe_layer_desc& d = *a.desc;
  if (d.dtype != HMOE_BF16) return HMOE_ERR_UNSUPPORTED;
  if (dense && (dense->desc->dtype != HMOE_BF16 || dense->desc->hidden != d.hidden)) return HMOE_ERR_UNSUPPORTED;
  if (dense && dense->n_rows == 0) dense = nullptr;
  if (combine && a.n_rows == 0) return HMOE_ERR_INVALID_ARG;  // without routed rows nothing would draw the tickets
  if (a.n_rows == 0 && !dense) return HMOE_OK;
  SkinnyCtx c{a.offsets, a.slot_of, a.slots, a.slot_bytes, a.active, d.n_experts, d.hidden, d.ffn, 1, a.row_map, a.map_div, {}, {}};
  int ffn_dense = 0;
  if (dense) {
    ffn_dense = dense->desc->ffn;
    c.shared = SkinnyShared{dense->slots, (const bf16_t*)dense->x_perm, (bf16_t*)dense->h, (bf16_t*)dense->o_perm, ffn_dense,
                            dense->n_rows, 0};
  }
  const int busy_max = std::min(d.n_experts, a.n_rows);     // every busy expert has at least one row
  int max_rows = std::max(1, a.n_rows / d.top_k);           // a token names an expert at most once
  if (dense) max_rows = std::max(max_rows, dense->n_rows);
  probe_before(a.stream);
  launch_stage<true>(c, d.ffn / TILE_N, busy_max, max_rows, ffn_dense / TILE_N, (const bf16_t*)a.x_perm, (bf16_t*)a.h, a.stream);
  probe_after(a.stream);
  probe_before(a.stream);
  if (combine) {
    c.combine = SkinnyCombine{combine->inv_perm, combine->topk_w, (const bf16_t*)a.o_perm, dense ? (const bf16_t*)dense->o_perm : nullptr,
                              (bf16_t*)combine->y, combine->tickets, combine->n_tokens, d.top_k, 1};
  }
  launch_stage<false>(c, d.hidden / TILE_N, busy_max, max_rows, dense ? d.hidden / TILE_N : 0, (const bf16_t*)a.h,
                      (bf16_t*)a.o_perm, a.stream);
  probe_after(a.stream);
  HMOE_HIP(hipGetLastError());
  return HMOE_OK;
}

// ---------------------------------------------------------------------------------------------
// 4-bit weights (HMOE_BF16_W4): the same organisation around the weight stream, a quarter of the bytes.
//
// A block owns two adjacent packed 16-row groups of one busy expert: gate and up of 16 features, or 32
// features of the down projection.  The unit of work is a scale
// group of 128 k: one 1 KiB unit of codes per 16-row group (one 16-byte non-temporal load per lane), four
// token fragments and one scale per lane and 16-row group.  Scale groups are dealt round-robin to the NW
// waves (the block sweeps a contiguous stretch of the stream) and the codes of DEPTH groups are in
// flight per wave: a group is multiplied in a fraction of the memory latency, so a single group of
// lookahead would leave the wave waiting.
//
// The matrix instruction is v_mfma_f32_16x16x32_bf16: up to 16 tokens x 16 features x 32 k, four
// accumulator registers, which suits decode (the 32x32x16 shape spends twice the cycles and four times the
// registers on rows that are padding).  Codes go to it without an integer-to-float conversion: a dword of
// 8 codes becomes the four operand registers of bfloat16 values 128 + q with one shift and one and-or
// each (see the layout note in common.h).  The offset is taken out again with one more MFMA per k-step
// against a tile of ones, which yields sum_k x_k per token in the accumulator layout:
//     sum_k x_k (q_k - 8) = sum_k x_k (128 + q_k) - 136 sum_k x_k,
// and the group's scale (per feature = per lane) multiplies that difference as it is added to the
// running fp32 result.  Products x * (128 + q) are exact in fp32; the cancellation costs about 5 of
// its 24 mantissa bits.
template <bool GATEUP, int NW>
__global__ __launch_bounds__(64 * NW) void ffn_skinny_w4_kernel(SkinnyCtx c, const bf16_t* __restrict__ in,
                                                                 bf16_t* __restrict__ out) {
  constexpr int NU = 2;                    // packed 16-row groups per block
  constexpr int FEAT = GATEUP ? 16 : 32;   // output features per block
  constexpr int MR = 16;              // rows per pass
  constexpr int DEPTH = 4;
  __shared__ float red[(NW > 1 ? NW - 1 : 1) * NU * 4 * 64];

  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
  const int e = nth_busy_expert(c, blockIdx.y, lane);
  if (e < 0) return;  // uniform over the block
  const int row_first = c.offsets[e], row_end = c.offsets[e + 1];
  const int K = GATEUP ? c.hidden : c.ffn;      // reduction length
  const int n_out = GATEUP ? c.ffn : c.hidden;  // row length of `out`
  const int n_groups = K / W4_GROUP;
  const int fb = blockIdx.x;                    // features [FEAT fb, FEAT fb + FEAT) of `out`
  if (fb >= n_out / FEAT) return;
  const int j = lane % 16, kblk = lane / 16;
  const char* slot = c.slots + (size_t)c.slot_of[e] * c.slot_bytes;
  const W4Offsets off = w4_offsets((size_t)c.hidden, (size_t)c.ffn);
  const u32x4* units = (const u32x4*)(slot + (GATEUP ? 0 : off.down_units));
  const bf16_t* scales = (const bf16_t*)(slot + (GATEUP ? off.gate_up_scales : off.down_scales));
  // packed 16-row group 2 fb + u: gate/up u = 0, 1 are gate and up of features 16 fb .. + 16; down u = 0, 1 are
  // features 32 fb .. + 16 and the next 16
  const u32x4* wq[NU];
  const bf16_t* ws[NU];
#pragma unroll
  for (int u = 0; u < NU; ++u) {
    const size_t grp = (size_t)NU * fb + u;
    wq[u] = units + grp * (size_t)n_groups * 64 + lane;
    ws[u] = scales + grp * (size_t)n_groups * 16 + j;
  }
  const int per_wave = (n_groups + NW - 1) / NW;  // scale groups per wave (the last ones may lie past the end)
  const u32x4 ones = {0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u};

  for (int row0 = row_first; row0 < row_end; row0 += MR) {
    const int rows = min(MR, row_end - row0);
    const int tok = j < rows ? j : 0;  // lane (j, kblk) supplies token j, k block kblk of the token operand (clamped)
    const int in_row = GATEUP ? mapped_row(c.row_map, c.map_div, row0 + tok) : row0 + tok;
    const u32x4* xin = (const u32x4*)(in + (size_t)in_row * K) + kblk;

    // ring of DEPTH scale groups per wave: codes, scales and the matching token fragments (the fragments
    // come from L1/L2, but a group is multiplied faster than even that latency).  Every load is issued
    // unconditionally from a clamped, valid address -- no branches around loads, so the compiler's count
    // of outstanding loads stays exact and a multiply waits only for its own group.  A group past the end
    // contributes nothing because its scale is replaced by zero at use; token rows past `rows` only reach
    // accumulator rows that are never stored.
    u32x4 codes[DEPTH][NU], xa[DEPTH][4];
    uint32_t scale_bits[DEPTH][NU];  // raw bfloat16: converting here would make the wave wait for the load at once
    bool live[DEPTH];
    auto load_group = [&](int slot_id, int i) {
      const int g = i * NW + wave;
      live[slot_id] = i < per_wave && g < n_groups;
      const int gc = min(g, n_groups - 1);
#pragma unroll
      for (int u = 0; u < NU; ++u) {
        codes[slot_id][u] = __builtin_nontemporal_load(wq[u] + (size_t)gc * 64);
        scale_bits[slot_id][u] = (uint32_t)ws[u][(size_t)gc * 16];
      }
#pragma unroll
      for (int t = 0; t < 4; ++t) xa[slot_id][t] = xin[(size_t)(16 * gc + 4 * t)];
    };

    f32x4_t acc[NU];
#pragma unroll
    for (int u = 0; u < NU; ++u) acc[u] = f32x4_t{0, 0, 0, 0};
    auto multiply_group = [&](int slot_id) {
      f32x4_t part[NU], xsum = {0, 0, 0, 0};
#pragma unroll
      for (int u = 0; u < NU; ++u) part[u] = f32x4_t{0, 0, 0, 0};
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        xsum = mfma_16x16x32_bf16(xa[slot_id][t], ones, xsum);
#pragma unroll
        for (int u = 0; u < NU; ++u) {
          const uint32_t d = codes[slot_id][u][t];
          const u32x4 w = {(d & 0x000F000Fu) | 0x43004300u, ((d >> 4) & 0x000F000Fu) | 0x43004300u,
                           ((d >> 8) & 0x000F000Fu) | 0x43004300u, ((d >> 12) & 0x000F000Fu) | 0x43004300u};
          part[u] = mfma_16x16x32_bf16(xa[slot_id][t], w, part[u]);
        }
      }
#pragma unroll
      for (int u = 0; u < NU; ++u) {
        const float sc = live[slot_id] ? __uint_as_float(scale_bits[slot_id][u] << 16) : 0.0f;
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[u][r] += sc * (part[u][r] - 136.0f * xsum[r]);
      }
    };

    // the scheduling barriers keep the loads where they are written: left alone, the compiler moves them
    // down to their uses to save registers, and with them the lookahead
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) load_group(d, d);
    __builtin_amdgcn_sched_barrier(0);
    for (int i = 0; i < per_wave; i += DEPTH) {
#pragma unroll
      for (int d = 0; d < DEPTH; ++d) {
        multiply_group(d);
        __builtin_amdgcn_sched_barrier(0);
        load_group(d, i + d + DEPTH);
        __builtin_amdgcn_sched_barrier(0);
      }
    }

    // ---- cross-wave reduction, epilogue, store ---------------------------------------------
    // accumulator register r of lane (j, kblk) is token 4 kblk + r, feature j of the 16-row group
    if (NW > 1 && wave > 0) {
      float* dst = red + (size_t)(wave - 1) * NU * 4 * 64;
#pragma unroll
      for (int u = 0; u < NU; ++u)
#pragma unroll
        for (int r = 0; r < 4; ++r) dst[(u * 4 + r) * 64 + lane] = acc[u][r];
    }
    if (NW > 1) __syncthreads();
    if (wave == 0) {
#pragma unroll
      for (int u = 0; u < NU; ++u)
#pragma unroll
        for (int r = 0; r < 4; ++r)
          for (int w = 0; w < NW - 1; ++w) acc[u][r] += red[((size_t)w * NU * 4 + u * 4 + r) * 64 + lane];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int m = 4 * kblk + r;
        if (m >= rows) continue;
        bf16_t* orow = out + (size_t)(row0 + m) * n_out + FEAT * fb + j;
        if (GATEUP) {
          orow[0] = f32_to_bf16(silu_f32(acc[0][r]) * acc[1][r]);
        } else {
          orow[0] = f32_to_bf16(acc[0][r]);
          orow[16] = f32_to_bf16(acc[1][r]);
        }
      }
    }
    if (NW > 1) __syncthreads();  // the reduction area is reused by the next row pass
  }
}

template <bool GATEUP>
static void launch_stage_w4(const SkinnyCtx& c, int n_out, int busy_max, const bf16_t* in, bf16_t* out, hipStream_t s) {
  const dim3 grid((unsigned)(n_out / (GATEUP ? 16 : 32)), (unsigned)busy_max);
  // Waves per block (they split K).  A wave that walks many scale groups keeps its ring of loads full; a
  // block whose waves each see only a few groups spends its life filling and draining it.  So: as few waves
  // per block as still put about eight waves on every CU (measured: one wave per block is best for the wide
  // gate/up launch, eight for the down projection of two experts).
  const long blocks = (long)grid.x * grid.y;
  const int n_groups = (GATEUP ? c.hidden : c.ffn) / W4_GROUP;
  int waves = 1;
  while (waves < 8 && blocks * waves < 2048 && n_groups / (2 * waves) >= 2) waves *= 2;
  if (const char* env = getenv("HMOE_W4_WAVES")) waves = atoi(env);  // tuning override: 1, 2, 4 or 8
  switch (waves) {
    case 1: hipLaunchKernelGGL((ffn_skinny_w4_kernel<GATEUP, 1>), grid, dim3(64), 0, s, c, in, out); break;
    case 2: hipLaunchKernelGGL((ffn_skinny_w4_kernel<GATEUP, 2>), grid, dim3(128), 0, s, c, in, out); break;
    case 4: hipLaunchKernelGGL((ffn_skinny_w4_kernel<GATEUP, 4>), grid, dim3(256), 0, s, c, in, out); break;
    default: hipLaunchKernelGGL((ffn_skinny_w4_kernel<GATEUP, 8>), grid, dim3(512), 0, s, c, in, out); break;
  }
}

int launch_ffn_skinny_w4(const FfnArgs& a) {
  const hmoe_layer_desc& d = *a.desc;
  if (d.dtype != HMOE_BF16_W4) return HMOE_ERR_UNSUPPORTED;
  if (a.n_rows == 0) return HMOE_OK;
  SkinnyCtx c{a.offsets, a.slot_of, a.slots, a.slot_bytes, a.active, d.n_experts, d.hidden, d.ffn, 1, a.row_map, a.map_div, {}, {}};
  const int busy_max = std::min(d.n_experts, a.n_rows);  // every busy expert has at least one row
  probe_before(a.stream);
  launch_stage_w4<true>(c, d.ffn, busy_max, (const bf16_t*)a.x_perm, (bf16_t*)a.h, a.stream);
  probe_after(a.stream);
  probe_before(a.stream);
  launch_stage_w4<false>(c, d.hidden, busy_max, (const bf16_t*)a.h, (bf16_t*)a.o_perm, a.stream);
  probe_after(a.stream);
  HMOE_HIP(hipGetLastError());
  return HMOE_OK;
}

}  // namespace hmoe
