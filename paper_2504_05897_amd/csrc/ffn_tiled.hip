// Prefill FFN (HMOE_FFN_TILED): grouped GEMM on bf16 MFMA, weights streamed past LDS.
//
// Two launches per call:  h = silu(X Wgate^T) * (X Wup^T)   and   O = h Wdown^T,
// each a grouped GEMM  C[rows of expert e, N] = A[rows, K] * W_e[N, K]^T  over the ragged row
// groups that the permutation produced (expert_offsets), with W_e found through the
// expert-id -> slot table.  All dispatch happens on the device: a block turns its index into
// (expert, m-tile, n-tile) by walking expert_offsets, so the host never reads the routing result.
//
// A block owns a tile of up to BM rows and 32 * FN * waves columns; every wave spans all rows and owns
// FN 32-row weight groups, as 32x32x16 bf16 MFMA fragments with fp32 accumulators.
//   * Weights arrive pre-tiled (packed slot layout): a 32-row x 16-k tile is 1 KiB in MFMA operand
//     order.  Each wave streams the tiles of its groups straight from global memory into a ring of
//     registers, DB k-substeps ahead; they never touch LDS.
//   * Activation tiles travel global -> LDS without passing through registers (global_load_lds_dwordx4:
//     every lane supplies a global address, the wave's 64 x 16 bytes land contiguously in LDS), into a
//     ring of SA stages; one barrier per K step of 64.  Rows are row-major; the lane that fills LDS chunk
//     (row, slot) fetches global chunk slot ^ f(row), an XOR swizzle that spreads the fragment reads over
//     all banks.
//   * Rows past the end of an expert and weight groups past N are loaded from a clamped (valid)
//     address instead of being zero-filled; their products land in accumulators that are never
//     stored.
//   * Gate and up rows are interleaved in 32-row groups, so with FN = 2 a wave's even fragments are gate
//     and its odd fragments the matching up columns: SwiGLU is applied to registers.
//   * Tiles are numbered expert-major, then n-tile, then m-tile, and block ids are dealt to the
//     8 XCDs in contiguous ranges so that blocks sharing a weight panel share an L2.
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <type_traits>

#include "common.h"
#include "tile_locate.h"

namespace hmoe {

// One 16-byte global -> LDS copy per lane; the wave's 64 chunks land at lds_base .. +1024 in lane
// order.  lds_base must be wave-uniform.  Completion is tracked by vmcnt like any vector load.
__device__ __forceinline__ void load_to_lds_16(const void* gptr, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
               :
               : "v"(gptr), "s"(__builtin_amdgcn_readfirstlane(lds_base))
               : "memory", "m0");
}
// 16-byte global store issued by hand (a kernel that keeps hand-issued loads in flight across its epilogue issues
// every vector-memory operation itself, so that the compiler never waits for, or counts, any of them)
__device__ __forceinline__ void store_16(void* gptr, const u32x4& v) {
  asm volatile("global_store_dwordx4 %0, %1, off" ::"v"(gptr), "v"(v) : "memory");
}
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
// The two marks below put no instruction into the kernel; they are comments in the device assembly that the
// build's listing check (asm_check.py) reads to recount the hand-counted waits: where the copies of one activation
// stage end, and which wait opens a stage of a ring of SA.
__device__ __forceinline__ void mark_stage_issued() { asm volatile("; hmoe: activation stage issued" ::: "memory"); }
template <int N, int SA>
__device__ __forceinline__ void wait_vmcnt_opens_stage() {
  asm volatile("s_waitcnt vmcnt(%0) ; hmoe: opens an activation stage, ring of %1" ::"n"(N), "n"(SA) : "memory");
}
// Workgroup barrier that the compiler may not move LDS accesses across.  (No fence instruction:
// the waits that make the data visible are issued explicitly by the caller.)
__device__ __forceinline__ void block_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

// ---------------------------------------------------------------------------------------------
// The tile.
//
// All NWV waves of a block span the whole BM rows; a wave owns 64 packed weight rows (one gate/up
// pair, or 64 output columns of the down projection; 32 with FN = 1).  Activation tiles go through the
// LDS ring (every wave needs all of them); weight tiles are 1 KiB each in MFMA operand order, so each wave
// streams its own straight from global memory into a ring of DB register slots, DB k-substeps ahead.
// Compared with staging both operands in LDS this removes the LDS fill and the LDS reads of the weight
// operand (about 40 % of the LDS traffic of a 256x256 tile) and keeps DB KiB per matrix in flight per wave,
// which is what the weight-streaming shapes need.
//
// Every vector-memory operation is issued by hand in a fixed order per k-substep
//   [FN weight-tile loads for substep s+DB] [this substep's share of the LDS copies for step t+SA-1]
// so the number of younger operations at each wait is a compile-time constant: N_B for a weight tile,
// N_A for an activation stage.  In the last steps the same operations are still issued, with the
// step clamped (their results are never used), which keeps the counts valid.
//
// NT: weight loads carry the non-temporal hint.  It pays when an expert has one or two m-tiles (each
// weight byte is used about once); with many m-tiles per expert the blocks of an XCD share the panel
// through L2 and plain loads are faster.
template <bool NT>
__device__ __forceinline__ u32x4 load_stream_16(const void* gptr) {
  u32x4 v;
  if (NT)
    asm volatile("global_load_dwordx4 %0, %1, off nt" : "=v"(v) : "v"(gptr) : "memory");
  else
    asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(v) : "v"(gptr) : "memory");
  return v;
}
// the same from a wave-uniform address (held in scalar registers) plus a byte offset per lane
template <bool NT>
__device__ __forceinline__ u32x4 load_stream_16(const void* uniform, uint32_t lane_bytes) {
  u32x4 v;
  if (NT)
    asm volatile("global_load_dwordx4 %0, %1, %2 nt" : "=v"(v) : "v"(lane_bytes), "s"(uniform) : "memory");
  else
    asm volatile("global_load_dwordx4 %0, %1, %2" : "=v"(v) : "v"(lane_bytes), "s"(uniform) : "memory");
  return v;
}
// wait until at most N younger vector-memory operations are outstanding; the operands tie the wait
// to the registers whose loads it covers, so their uses cannot be scheduled above it
template <int N>
__device__ __forceinline__ void wait_vmcnt_regs(u32x4& a, u32x4& b) {
  asm volatile("s_waitcnt vmcnt(%2)" : "+v"(a), "+v"(b) : "n"(N) : "memory");
}
template <int N>
__device__ __forceinline__ void wait_vmcnt_regs(u32x4& a) {
  asm volatile("s_waitcnt vmcnt(%1)" : "+v"(a) : "n"(N) : "memory");
}

// FMC (0: off): the tile multiplies only its first FMC 32-row fragments and consecutive m-tiles of an expert
// start 32 * FMC rows apart (the activation copies still move BM rows).  The kernel picks FMC per expert so
// that the expert's m-tiles are equally high (see ffn_tile_fit_kernel).
//
// FN_ (2 or 1): 32-row weight groups per wave.  With one group a wave needs half the accumulators per row, which is
// what lets a tile span 256 rows (an expert of up to 256 rows then reads its weights once, in one block, instead of
// twice in two blocks that must keep pace to share them through L2); the gate and the up half of a SwiGLU pair then
// sit in neighbouring waves and meet through LDS in the epilogue.  Tiles higher than 128 rows copy only the rows
// they multiply (rounded up to what one copy instruction per thread moves).
// TR (with ILV): the weight tile is the first operand of the matrix instruction, so the accumulators hold the transposed
// block: a lane owns one row per fragment and, per weight group, four runs of four consecutive columns, which the
// epilogues turn into 8-byte pieces of an output row (a quarter of the conversions and LDS writes of the other form).
template <bool GATEUP_, int BM_, int NWV, int SA, bool NT, int DB = 8, int FMC = 0, int FN_ = 2, bool ILV = false, bool TR = false>
struct StreamTile {
  static constexpr bool GATEUP = GATEUP_;
  static constexpr int BM = BM_;
  static constexpr int FN = FN_, BN = NWV * 32 * FN, BKT = 64, KK = 4;
  static constexpr int FM = FMC > 0 ? FMC : BM / 32;   // fragments multiplied
  static constexpr int MSTRIDE = 32 * FM;              // rows between the starts of consecutive m-tiles
  static_assert(FM * 32 <= BM && (FN == 1 || FN == 2) && (!TR || (ILV && FN == 2)), "");
  static_assert(DB % KK == 0, "the weight ring holds whole K steps");
  static constexpr int CPR = BKT / 8, RP = 256 / (BKT * 2);
  static constexpr int ROWS_PER_OP = 64 * NWV / CPR;   // rows one copy instruction of every thread moves
  static constexpr int A_ROWS = BM > 128 ? (FM * 32 + ROWS_PER_OP - 1) / ROWS_PER_OP * ROWS_PER_OP : BM;
  static constexpr int A_CHUNKS = A_ROWS * CPR;
  static constexpr int A_OPS = A_CHUNKS / (64 * NWV);
  static_assert(A_OPS >= 1 && A_OPS * 64 * NWV == A_CHUNKS, "activation tile must split evenly over the waves");
  static_assert(SA >= 3, "the activation ring needs three stages");
  static constexpr int OPS3 = A_OPS - A_OPS * 3 / KK;  // copies issued in the last substep of a step
  static constexpr int N_B = (DB - 1) * FN + (DB / KK) * A_OPS;
  static constexpr int N_A = (SA - 3) * (KK * FN + A_OPS) + 3 * FN + A_OPS - OPS3;
  static_assert(N_B <= 63 && N_A + FN - 1 <= 63, "vmcnt range");
  // ILV (one wave per SIMD): the substep's work is issued between its matrix instructions, in the order [weight group
  // 0] [copies] [weight group 1]; a wait for both groups of a ring slot then has one substep's copies fewer behind it.
  // The count uses the largest piece of copies, so it is exact or one operation stricter.
  static constexpr int N_B_ILV = N_B - (A_OPS + KK - 1) / KK;
  static constexpr int THREADS = 64 * NWV;
  // 16-byte units between ring stages: the tile's own rows, or with TR (blocks that go from tile to tile, whose next
  // tile is already being copied in while this one is multiplied) the rows of the highest tile, whatever FM is
  static constexpr int STAGE_CHUNKS = TR ? BM * CPR : A_CHUNKS;
  static constexpr int LDS_VEC = SA * STAGE_CHUNKS;  // 16-byte units
  typedef f32x16_t Acc[FM][FN];

  // Where a thread's copies and weight loads start: a_src[i] is the 16-byte chunk of the activation tile that copy i
  // of this thread moves (rows past the expert's end clamped to its last row), b_src[j] the thread's piece of the
  // first weight tile of the wave's group j (groups past N clamped to group 0).  m0 is the tile's first row within
  // the expert.  NA may exceed A_OPS (a caller that serves tile types of several heights with one set of pointers).
  // In two steps, so that a caller can put other work between the lookups and their use.
  //
  // Sorted rows of the thread's copies, and with a row map (the gather folded into gate/up) what the map holds for
  // them: all lookups are issued before the first is used, one trip to memory per tile.
  template <int NA>
  static __device__ __forceinline__ void fetch_rows(const TiledCtx& c, const TileLoc& loc, int m0, int wave, int lane,
                                                    int (&rows)[NA]) {
#pragma unroll
    for (int i = 0; i < NA; ++i) {
      const int r = ((i * NWV + wave) * 64 + lane) / CPR;
      rows[i] = loc.row_first + (m0 + r < loc.m_rows ? m0 + r : loc.m_rows - 1);
    }
    if (GATEUP && c.row_map) {
#pragma unroll
      for (int i = 0; i < NA; ++i) rows[i] = c.row_map[rows[i]];
    }
  }
  // ... the input rows from what the map holds
  template <int NA>
  static __device__ __forceinline__ void input_rows(const TiledCtx& c, int (&rows)[NA]) {
    if (GATEUP && c.row_map) {
#pragma unroll
      for (int i = 0; i < NA; ++i) rows[i] = div_by_map(c, rows[i]);
    }
  }
  // ... and the pointers from the input rows
  template <int NA>
  static __device__ __forceinline__ void set_sources_from(const TiledCtx& c, const bf16_t* __restrict__ in, const TileLoc& loc,
                                                          const int (&rows)[NA], int k_begin, int wave, int lane,
                                                          const u32x4* (&a_src)[NA], const u32x4* (&b_src)[FN]) {
    const int K = GATEUP ? c.hidden : c.ffn;
    const int n_groups = (GATEUP ? 2 * c.ffn : c.hidden) / TILE_N;
    const int kt16 = K / TILE_K;
    const char* slot = c.slots + (size_t)loc.slot * c.slot_bytes;
    const u32x4* w = GATEUP ? (const u32x4*)slot : (const u32x4*)(slot + 4 * (size_t)c.ffn * c.hidden);
#pragma unroll
    for (int i = 0; i < NA; ++i) {
      const int ci = (i * NWV + wave) * 64 + lane;
      const int r = ci / CPR, sl = ci % CPR;
      const int chunk = sl ^ ((r / RP) % CPR);
      a_src[i] = (const u32x4*)(in + (size_t)rows[i] * K) + chunk + (size_t)k_begin * CPR;
    }
#pragma unroll
    for (int j = 0; j < FN; ++j) {
      const int g = loc.nt * (BN / TILE_N) + wave * FN + j;
      b_src[j] = w + ((size_t)(g < n_groups ? g : 0) * kt16 + (size_t)k_begin * KK) * 64 + lane;
    }
  }
  template <int NA>
  static __device__ __forceinline__ void set_sources(const TiledCtx& c, const bf16_t* __restrict__ in, const TileLoc& loc,
                                                     int m0, int k_begin, int wave, int lane, const u32x4* (&a_src)[NA],
                                                     const u32x4* (&b_src)[FN]) {
    int rows[NA];
    fetch_rows(c, loc, m0, wave, lane, rows);
    input_rows(c, rows);
    set_sources_from(c, in, loc, rows, k_begin, wave, lane, a_src, b_src);
  }
  // copy `op` of this thread for K step `kstep` (clamped to the last step) into ring stage `stage`
  template <int NA>
  static __device__ __forceinline__ void issue_a_op(const u32x4* (&a_src)[NA], uint32_t lds0, int wave, int k_steps,
                                                    int stage, int kstep, int op) {
    copy_to_stage(a_src[op] + (size_t)(kstep < k_steps ? kstep : k_steps - 1) * CPR, lds0, wave, stage, op);
  }
  // copy `op` of this thread, from `from`, into ring stage `stage`
  static __device__ __forceinline__ void copy_to_stage(const u32x4* from, uint32_t lds0, int wave, int stage, int op) {
    const uint32_t base = lds0 + (uint32_t)stage * STAGE_CHUNKS * 16;
    load_to_lds_16(from, base + (uint32_t)((op * NWV + wave) * 64) * 16);
  }
  // piece `piece` (of KK) of the copies of one stage
  template <int NA>
  static __device__ __forceinline__ void issue_a_piece(const u32x4* (&a_src)[NA], uint32_t lds0, int wave, int k_steps,
                                                       int stage, int kstep, int piece) {
#pragma unroll
    for (int op = 0; op < A_OPS; ++op)
      if (op >= A_OPS * piece / KK && op < A_OPS * (piece + 1) / KK) issue_a_op(a_src, lds0, wave, k_steps, stage, kstep, op);
    if (piece == KK - 1) mark_stage_issued();
  }
  // The start of a tile: fill the weight ring and SA-1 activation stages.  Nothing is waited for.
  template <int NA>
  static __device__ __forceinline__ void issue_prologue(const u32x4* (&a_src)[NA], const u32x4* (&b_src)[FN], uint32_t lds0,
                                                        int wave, int k_steps, u32x4 (&ring)[DB][FN]) {
    const int n_sub = k_steps * KK;
#pragma unroll
    for (int s = 0; s < DB; ++s)
#pragma unroll
      for (int j = 0; j < FN; ++j) ring[s][j] = load_stream_16<NT>(b_src[j] + (size_t)(s < n_sub ? s : n_sub - 1) * 64);
#pragma unroll
    for (int st = 0; st < SA - 1; ++st)
#pragma unroll
      for (int p = 0; p < KK; ++p) issue_a_piece(a_src, lds0, wave, k_steps, st, st, p);
  }

  // acc += A[rows of the tile, k range] * W[columns of the tile, k range]^T for the k_steps steps of BKT
  // that start at step k_begin.  On return every copy into LDS has landed.
  static __device__ __forceinline__ void mainloop(const TiledCtx& c, const bf16_t* __restrict__ in, const TileLoc& loc,
                                                  int k_begin, int k_steps, u32x4* lds, Acc& acc) {
    const int tid = threadIdx.x, lane = tid % 64;
    const int wave = __builtin_amdgcn_readfirstlane(tid / 64);  // uniform: LDS bases and weight groups stay scalar
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) u32x4*)lds;
    const u32x4* a_src[A_OPS];
    const u32x4* b_src[FN];
    set_sources(c, in, loc, loc.mt * MSTRIDE, k_begin, wave, lane, a_src, b_src);
    u32x4 ring[DB][FN];
    issue_prologue(a_src, b_src, lds0, wave, k_steps, ring);
    steps(a_src, b_src, lds, wave, lane, k_steps, ring, acc);
  }

  // fragment i (rows 32 i ..) of k-substep kk of a ring stage, for the lane that owns (half, col) of the operand
  static __device__ __forceinline__ u32x4 read_fragment(const u32x4* lds, int stage, int kk, int i, int half, int col) {
    const int r = i * 32 + col;
    return lds[stage * STAGE_CHUNKS + r * CPR + ((kk * 2 + half) ^ ((r / RP) % CPR))];
  }
  // One k-substep of a wave that has its SIMD to itself (ILV): nothing else fills the matrix pipe while this wave issues
  // anything else, so all other work of the substep sits between its matrix instructions, one piece behind each: the
  // next substep's fragment reads behind the first FM, which multiply weight group 0; then the reload of group 0's
  // ring slot, this substep's activation copies, and behind the last one the reload of group 1.  Vector-memory order
  // per substep: [group 0] [copies] [group 1].  kk: substep within the K step; sl: its ring slot; w_next: where the
  // reloads read (16-byte units from b_src); koff: where the copies read (from a_src), into fill_stage.
  // Where the operands of a tile come from.  As pointers per thread: a[op] is the thread's 16 bytes of copy op at the
  // tile's first K step, b[j] its piece of the first weight tile of group j.
  template <int NA>
  struct PtrSrc {
    const u32x4* (&a)[NA];
    const u32x4* (&b)[FN];
    __device__ __forceinline__ const u32x4* a_at(int op, size_t koff) const { return a[op] + koff; }
    __device__ __forceinline__ u32x4 b_at(int j, size_t w) const { return load_stream_16<NT>(b[j] + w); }
  };
  // Or, for a block that goes from tile to tile and holds two tiles' sources over a K loop, in half the registers:
  // the input ROW of each copy (the thread's place within a row, a_lane, is the same for every copy and tile), and
  // wave-uniform weight addresses in scalar registers with the lane's offset added by the load.
  struct RowSrc {
    const u32x4* a_lane;  // input + the thread's chunk within a row
    uint32_t pitch;       // 16-byte units per input row
    const int (&rows)[7];
    const u32x4* b[2];    // wave-uniform
    uint32_t lane_bytes;
    __device__ __forceinline__ const u32x4* a_at(int op, size_t koff) const {
      return a_lane + ((size_t)(uint32_t)rows[op] * pitch + koff);
    }
    __device__ __forceinline__ u32x4 b_at(int j, size_t w) const { return load_stream_16<NT>(b[j] + w, lane_bytes); }
  };
  template <class SRC, int NF>
  static __device__ __forceinline__ void ilv_substep(int kk, int sl, int stage, int next_stage, int fill_stage, size_t w_next,
                                                     size_t koff, const SRC& src, const u32x4* lds, uint32_t lds0, int wave,
                                                     int half, int col, u32x4 (&ring)[DB][FN], u32x4 (&fa)[NF][FM],
                                                     Acc& acc) {
    static_assert(FN == 2 && NF == 2, "");
    wait_vmcnt_regs<N_B_ILV>(ring[sl][0], ring[sl][1]);
#pragma unroll
    for (int m = 0; m < 2 * FM; ++m) {
      const int i = m % FM, j = m / FM;
      acc[i][j] = TR ? mfma_32x32x16_bf16(ring[sl][j], fa[kk & 1][i], acc[i][j])
                     : mfma_32x32x16_bf16(fa[kk & 1][i], ring[sl][j], acc[i][j]);
      if (m < FM)
        fa[(kk + 1) & 1][m] = kk == KK - 1 ? read_fragment(lds, next_stage, 0, m, half, col)
                                           : read_fragment(lds, stage, kk + 1, m, half, col);
      if (m == FM) ring[sl][0] = src.b_at(0, w_next);
#pragma unroll
      for (int op = 0; op < A_OPS; ++op)
        if (op >= A_OPS * kk / KK && op < A_OPS * (kk + 1) / KK) {
          const int at = FM + 1 + (op - A_OPS * kk / KK);
          if (m == (at < 2 * FM - 1 ? at : 2 * FM - 1)) copy_to_stage(src.a_at(op, koff), lds0, wave, fill_stage, op);
        }
      if (m == 2 * FM - 1) {
        if (kk == KK - 1) mark_stage_issued();
        ring[sl][1] = src.b_at(1, w_next);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  }

  // The K loop of a tile whose prologue has been issued (by this thread, into `ring` and the first SA-1 stages).
  // On return every vector-memory operation of the thread has completed.
  template <int NA>
  static __device__ __forceinline__ void steps(const u32x4* (&a_src)[NA], const u32x4* (&b_src)[FN], u32x4* lds, int wave,
                                               int lane, int k_steps, u32x4 (&ring)[DB][FN], Acc& acc) {
    const int half = lane / 32, col = lane % 32;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) u32x4*)lds;
    const int n_sub = k_steps * KK;
    // Activation fragments: two sets with two weight groups per wave (the next substep's set is read while this one
    // is multiplied); one set with one group, where a fragment feeds a single MFMA and is refilled right behind it.
    constexpr int FA_SETS = FN == 1 ? 1 : 2;
    u32x4 fa[FA_SETS][FM];
    auto read_frag = [&](int stage, int kk, int i) { return read_fragment(lds, stage, kk, i, half, col); };
    auto read_a = [&](int buf, int stage, int kk) {
      const u32x4* sa = lds + stage * STAGE_CHUNKS;
#pragma unroll
      for (int i = 0; i < FM; ++i) {
        const int r = i * 32 + col;
        fa[buf][i] = sa[r * CPR + ((kk * 2 + half) ^ ((r / RP) % CPR))];
      }
    };

    // ---- the prologue's loads and copies: wait for all of them ----
    wait_vmcnt<0>();
    block_barrier();
    read_a(0, 0, 0);

    int stage = 0;  // ring stage of step tt
    // one K step; hc carries h, the step's place in the weight ring (a compile-time constant: the ring is registers)
    auto k_step = [&](int tt, auto hc) __attribute__((always_inline)) {
        constexpr int h = decltype(hc)::value;
        {
          const int next_stage = stage + 1 == SA ? 0 : stage + 1;
          const int fill_stage = stage == 0 ? SA - 1 : stage - 1;  // held step tt-1, free since this step opened
#pragma unroll
          for (int kk = 0; kk < KK; ++kk) {
            if (kk == KK - 1) {
              // open step tt+1: its activation tile has landed once at most N_A younger operations are out
              wait_vmcnt_opens_stage<ILV ? N_A + FN - 1 : N_A, SA>();
              __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): this step's last fragments are in registers
              block_barrier();
              if constexpr (FN == 2 && !ILV) read_a((kk + 1) & 1, next_stage, 0);
            } else {
              if constexpr (FN == 2 && !ILV) read_a((kk + 1) & 1, stage, kk + 1);
            }
            __builtin_amdgcn_sched_barrier(0);
            const int sl = h * KK + kk;  // ring slot of substep 4*tt + kk
            if constexpr (FN == 2 && ILV) {
              const int s_next = tt * KK + kk + DB;
              const int copy_step = tt + SA - 1;
              ilv_substep(kk, sl, stage, next_stage, fill_stage, (size_t)(s_next < n_sub ? s_next : n_sub - 1) * 64,
                          (size_t)(copy_step < k_steps ? copy_step : k_steps - 1) * CPR, PtrSrc<NA>{a_src, b_src}, lds, lds0, wave,
                          half, col, ring, fa, acc);
            } else if constexpr (FN == 2) {
              wait_vmcnt_regs<N_B>(ring[sl][0], ring[sl][1]);
#pragma unroll
              for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j) acc[i][j] = mfma_32x32x16_bf16(fa[kk & 1][i], ring[sl][j], acc[i][j]);
            } else {
              wait_vmcnt_regs<N_B>(ring[sl][0]);
#pragma unroll
              for (int i = 0; i < FM; ++i) {
                acc[i][0] = mfma_32x32x16_bf16(fa[0][i], ring[sl][0], acc[i][0]);
                fa[0][i] = kk == KK - 1 ? read_frag(next_stage, 0, i) : read_frag(stage, kk + 1, i);
              }
            }
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (!ILV) {
              const int s_next = tt * KK + kk + DB;
#pragma unroll
              for (int j = 0; j < FN; ++j)
                ring[sl][j] = load_stream_16<NT>(b_src[j] + (size_t)(s_next < n_sub ? s_next : n_sub - 1) * 64);
              issue_a_piece(a_src, lds0, wave, k_steps, fill_stage, tt + SA - 1, kk);
            }
          }
          stage = next_stage;
        }
    };
    static_assert(DB / KK == 1 || DB / KK == 2, "the weight ring holds one or two K steps");
    if constexpr (ILV && DB / KK == 2) {
      // Pairs of steps without a condition inside the loop, then the odd step if there is one: accumulators that
      // pass through a conditional block inside the loop are more than the register allocator handles when they
      // fill the second register file.
      int t = 0;
      for (; t + 2 <= k_steps; t += 2) {
        k_step(t, std::integral_constant<int, 0>{});
        k_step(t + 1, std::integral_constant<int, 1>{});
      }
      if (t < k_steps) k_step(t, std::integral_constant<int, 0>{});
    } else {
      for (int t = 0; t < k_steps; t += DB / KK) {
        k_step(t, std::integral_constant<int, 0>{});
        if constexpr (DB / KK == 2)
          if (t + 1 < k_steps) k_step(t + 1, std::integral_constant<int, 1>{});
      }
    }
    wait_vmcnt<0>();  // the clamped tail copies must not outlive the block's LDS
    // The tail's weight loads are never multiplied.  The compiler knows nothing of their latency: without a use
    // after the wait it may give two of them the same destination, or build the next address in a register that
    // a load still in flight is about to overwrite.  Keeping every ring slot alive up to here rules that out.
#pragma unroll
    for (int s = 0; s < DB; ++s)
#pragma unroll
      for (int j = 0; j < FN; ++j) asm volatile("" ::"v"(ring[s][j]));
  }

  // The K loop of a block that goes from tile to tile (TR).  On entry the weight ring and the first two activation
  // stages of the tile have landed (the thread's own part; a barrier here covers the other waves'): they were issued
  // by the previous tile's last two K steps, or by the block's first prologue.  The last two K steps of this tile in
  // turn issue the first loads of the NEXT tile, from the sources that `then()` returns (called when the other steps
  // are through), in place of loads this tile has no use for: they run the same code with their step numbers counted
  // from the next tile's start.  No operation changes its place in the
  // vector-memory order, so every hand-counted wait stands.  The ring holds two K steps: k_steps must be even, and at
  // least 6.
  // stage: the ring stage of the tile's first step, on return that of the next tile's first step.
  // On return the next tile's first loads and copies are in flight.
  template <class THEN>
  static __device__ __forceinline__ void steps_walk(const RowSrc& now, THEN then, u32x4* lds, int wave, int lane, int k_steps,
                                                    int& stage, u32x4 (&ring)[DB][FN], Acc& acc) {
    static_assert(TR && ILV && FN == 2 && DB == 2 * KK && SA == 3, "");
    const int half = lane / 32, col = lane % 32;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) u32x4*)lds;
    u32x4 fa[2][FM];
    block_barrier();  // the copies of every wave into the first stage have landed (each waited for its own)
#pragma unroll
    for (int i = 0; i < FM; ++i) fa[0][i] = read_fragment(lds, stage, 0, i, half, col);
    // one K step; hc: its place in the weight ring; first: the step that src counts from
    auto k_step = [&](int tt, auto hc, const RowSrc& src, int first) __attribute__((always_inline)) {
      constexpr int h = decltype(hc)::value;
      const int next_stage = stage + 1 == SA ? 0 : stage + 1;
      const int fill_stage = stage == 0 ? SA - 1 : stage - 1;  // held step tt-1, free since this step opened
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) {
        if (kk == KK - 1) {
          wait_vmcnt_opens_stage<N_A + FN - 1, SA>();  // open step tt+1
          __builtin_amdgcn_s_waitcnt(0xC07F);          // lgkmcnt(0): this step's last fragments are in registers
          block_barrier();
        }
        __builtin_amdgcn_sched_barrier(0);
        ilv_substep(kk, h * KK + kk, stage, next_stage, fill_stage, (size_t)((tt - first) * KK + kk + DB) * 64,
                    (size_t)(tt - first + SA - 1) * CPR, src, lds, lds0, wave, half, col, ring, fa, acc);
        __builtin_amdgcn_sched_barrier(0);
      }
      stage = next_stage;
    };
    // The first two steps stand apart: the accumulators start at zero (the caller's zero_acc), so their first matrix
    // instructions take the constant as their addend and nothing has to be cleared.
    k_step(0, std::integral_constant<int, 0>{}, now, 0);
    k_step(1, std::integral_constant<int, 1>{}, now, 0);
    // (a loop that always runs: with a way round it, registers with loads in flight would meet at the far end)
    int t = 2;
#pragma nounroll
    do {
      k_step(t, std::integral_constant<int, 0>{}, now, 0);
      k_step(t + 1, std::integral_constant<int, 1>{}, now, 0);
      t += 2;
    } while (t + 2 < k_steps);
    const RowSrc after = then();
    k_step(t, std::integral_constant<int, 0>{}, after, k_steps);
    k_step(t + 1, std::integral_constant<int, 1>{}, after, k_steps);
  }
  // The sources of a tile, given the input rows of its copies
  static __device__ __forceinline__ RowSrc row_sources(const TiledCtx& c, const bf16_t* __restrict__ in, const TileLoc& loc,
                                                       const int (&rows)[7], int wave, int lane) {
    const int K = GATEUP ? c.hidden : c.ffn;
    const int n_groups = (GATEUP ? 2 * c.ffn : c.hidden) / TILE_N;
    const int kt16 = K / TILE_K;
    const char* slot = c.slots + (size_t)loc.slot * c.slot_bytes;
    const u32x4* w = GATEUP ? (const u32x4*)slot : (const u32x4*)(slot + 4 * (size_t)c.ffn * c.hidden);
    // the thread's chunk within a row: the same for every copy (32 rows apart, and the swizzle repeats every 16 rows)
    const int ci = wave * 64 + lane;
    const int chunk = (ci % CPR) ^ (((ci / CPR) / RP) % CPR);
    const int g0 = loc.nt * (BN / TILE_N) + wave * FN;
    return RowSrc{(const u32x4*)in + chunk, (uint32_t)(K / 8), rows,
                  {w + (size_t)(g0 < n_groups ? g0 : 0) * kt16 * 64, w + (size_t)(g0 + 1 < n_groups ? g0 + 1 : 0) * kt16 * 64},
                  (uint32_t)lane * 16};
  }

  static __device__ __forceinline__ void epilogue(const TiledCtx& c, bf16_t* __restrict__ out, const TileLoc& loc,
                                                  const Acc& acc, u32x4* lds) {
    if constexpr (GATEUP && FN == 1) epilogue_pairs(c, out, loc, acc, lds);
    else if constexpr (GATEUP) epilogue_lines(c, out, loc, acc, lds);
    else if constexpr (FN == 2) epilogue_lines_down(c, out, loc, acc, lds);
    else epilogue_lines_block(c, out, loc, acc, lds);
  }
  // Gate/up with one weight group per wave: wave 2p holds the gate half and wave 2p+1 the up half of pair p, for all
  // rows.  The gate wave finishes the first HALF fragments and the up wave the others; each passes the partner the
  // accumulators the partner finishes, through the (now idle) activation ring in LDS.
  static constexpr int HALF = (FM + 1) / 2;
  static __device__ __forceinline__ void epilogue_pairs(const TiledCtx& c, bf16_t* __restrict__ out, const TileLoc& loc,
                                                        const Acc& acc, u32x4* lds) {
    static_assert(NWV % 2 == 0 && NWV * HALF * 1024 <= LDS_VEC * 4, "the exchange must fit the activation ring");
    const int row_first = loc.row_first, m_rows = loc.m_rows, nt = loc.nt;
    const int n_out = c.ffn;
    const int m0 = loc.mt * MSTRIDE;
    const int tid = threadIdx.x, wave = tid / 64, lane = tid % 64;
    const int half = lane / 32, col = lane % 32;
    const bool up_wave = wave & 1;
    float* mine = (float*)lds + (size_t)wave * HALF * 1024;          // what this wave hands over
    const float* theirs = (const float*)lds + (size_t)(wave ^ 1) * HALF * 1024;
    block_barrier();  // every wave has read its last activation fragments
#pragma unroll
    for (int i = 0; i < FM; ++i) {
      if ((i < HALF) == up_wave) {  // uniform per wave: a fragment the partner finishes
        const int fi = i < HALF ? i : i - HALF;
#pragma unroll
        for (int r = 0; r < 16; ++r) mine[(fi * 16 + r) * 64 + lane] = acc[i][0][r];
      }
    }
    __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0)
    block_barrier();
    const int f = (nt * (BN / 64) + wave / 2) * 32 + col;
#pragma unroll
    for (int i = 0; i < FM; ++i) {
      if ((i < HALF) != up_wave) {
        const int fi = i < HALF ? i : i - HALF;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float other = theirs[(fi * 16 + r) * 64 + lane];
          const float g = up_wave ? other : acc[i][0][r];
          const float u = up_wave ? acc[i][0][r] : other;
          const int m = m0 + i * 32 + (r / 4) * 8 + half * 4 + (r % 4);
          if (m < m_rows && f < n_out) out[(size_t)(row_first + m) * n_out + f] = f32_to_bf16(silu_f32(g) * u);
        }
      }
    }
  }
  // Gate/up with two weight groups per wave: a wave's SwiGLU results are 32 columns wide, half a 128-byte line of h,
  // and written as such they cost the launch 6-10 % (partial lines, the other half arriving from another wave at
  // another time).  Waves 2p and 2p+1 own neighbouring columns: both put their results into one [rows][64] block in
  // the idle activation ring, then each stores half of the rows as whole lines, 16 bytes per lane.
  static __device__ __forceinline__ void epilogue_lines(const TiledCtx& c, bf16_t* __restrict__ out, const TileLoc& loc,
                                                        const Acc& acc, u32x4* lds) {
    static_assert(NWV % 2 == 0 && (NWV / 2) * FM * 32 * 8 <= LDS_VEC, "the staging blocks must fit the activation ring");
    const int row_first = loc.row_first, m_rows = loc.m_rows, nt = loc.nt;
    const int n_out = c.ffn;
    const int m0 = loc.mt * MSTRIDE;
    const int tid = threadIdx.x, wave = tid / 64, lane = tid % 64;
    const int half = lane / 32, col = lane % 32;
    bf16_t* block = (bf16_t*)(lds + (wave / 2) * FM * 32 * 8);  // [FM * 32 rows][64 columns]
    block_barrier();  // every wave has read its last activation fragments
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = i * 32 + (r / 4) * 8 + half * 4 + (r % 4);
        block[row * 64 + (wave % 2) * 32 + col] = f32_to_bf16(silu_f32(acc[i][0][r]) * acc[i][1][r]);
      }
    __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0)
    block_barrier();
    const int f = nt * (BN / 2) + (wave / 2) * 64 + (lane % 8) * 8;
#pragma unroll
    for (int k = 0; k < 2 * FM; ++k) {
      const int row = (wave % 2) * FM * 16 + k * 8 + lane / 8;
      const u32x4 v = *(const u32x4*)(block + row * 64 + (lane % 8) * 8);
      const int m = m0 + row;
      if (m < m_rows && f < n_out) *(u32x4*)(out + (size_t)(row_first + m) * n_out + f) = v;
    }
  }
  // Down projection with two weight groups per wave: the wave's 64 columns are one 128-byte line per row.  The wave
  // turns its accumulators into rows in a block of its own in the idle activation ring, two fragments (64 rows) at a
  // time, and stores whole lines, 16 bytes per lane.  (LDS serves a wave's accesses in order: no barrier in between.)
  static __device__ __forceinline__ void epilogue_lines_down(const TiledCtx& c, bf16_t* __restrict__ out, const TileLoc& loc,
                                                             const Acc& acc, u32x4* lds) {
    static_assert(NWV * 64 * 8 <= LDS_VEC, "the staging blocks must fit the activation ring");
    const int row_first = loc.row_first, m_rows = loc.m_rows, nt = loc.nt;
    const int n_out = c.hidden;
    const int m0 = loc.mt * MSTRIDE;
    const int tid = threadIdx.x, wave = tid / 64, lane = tid % 64;
    const int half = lane / 32, col = lane % 32;
    bf16_t* block = (bf16_t*)(lds + wave * 64 * 8);  // [64 rows][64 columns]
    const int n = nt * BN + wave * 64 + (lane % 8) * 8;
    block_barrier();  // every wave has read its last activation fragments
#pragma unroll
    for (int pass = 0; pass < (FM + 1) / 2; ++pass) {
#pragma unroll
      for (int ii = 0; ii < 2; ++ii) {
        const int i = pass * 2 + ii;
        if (i < FM) {
#pragma unroll
          for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r)
              block[(ii * 32 + (r / 4) * 8 + half * 4 + (r % 4)) * 64 + j * 32 + col] = f32_to_bf16(acc[i][j][r]);
        }
      }
      __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0)
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        const int row = k * 8 + lane / 8;
        if (pass * 2 + row / 32 < FM) {  // uniform per k: the second fragment of the last pass may not exist
          const u32x4 v = *(const u32x4*)(block + row * 64 + (lane % 8) * 8);
          const int m = m0 + pass * 64 + row;
          if (m < m_rows && n < n_out) *(u32x4*)(out + (size_t)(row_first + m) * n_out + n) = v;
        }
      }
      __builtin_amdgcn_s_waitcnt(0xC07F);  // the rows are in registers before the next pass overwrites the block
    }
  }
  // The two epilogues of a block that goes on to another tile (transposed product, TR).  The staging blocks lie in a
  // region of their own (`staging`: the activation ring is already being filled for the next tile) and the stores are
  // issued by hand; the previous tile's reads of the staging blocks are separated from these writes by that tile's
  // whole K loop.  The accumulators are pinned where they are on entry: without that the compiler starts to copy them
  // out of the second register file before the next tile's loads are issued, into registers it frees by moving
  // others; the scheduling fences keep the tile's arithmetic from spreading over the registers of loads in flight.
  // Staging blocks are rows of 128 bytes in eight 16-byte slots; row r keeps slot s at s ^ ((r / 2) % 8), so that the 8-byte writes of a wave (32 rows, two
  // neighbouring half slots each) and the 16-byte reads (8 rows x 8 slots) both spread over all banks.
  static __device__ __forceinline__ uint32_t staged_at(int row, int slot) {
    return (uint32_t)(row * 128 + ((slot ^ ((row >> 1) & 7)) << 4));
  }
  static __device__ __forceinline__ void epilogue_lines_walk_tr(const TiledCtx& c, bf16_t* __restrict__ out, const TileLoc& loc,
                                                                Acc& acc, u32x4* staging, int wave, int lane) {
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
      for (int j = 0; j < FN; ++j) asm volatile("" : "+a"(acc[i][j]));
    const int row_first = loc.row_first, m_rows = loc.m_rows, nt = loc.nt;
    const int n_out = c.ffn;
    const int m0 = loc.m0;
    const int half = lane / 32, rl = lane % 32;
    char* block = (char*)(staging + (wave / 2) * FM * 32 * 8);  // [FM * 32 rows][64 columns] of waves 2p, 2p+1
#pragma unroll
    for (int i = 0; i < FM; ++i) {
      const int row = i * 32 + rl;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        float v[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) v[t] = silu_f32(acc[i][0][q * 4 + t]) * acc[i][1][q * 4 + t];
        uint2 pk;
        pk.x = f32_to_bf16_pair(v[0], v[1]);
        pk.y = f32_to_bf16_pair(v[2], v[3]);
        *(uint2*)(block + staged_at(row, (wave % 2) * 4 + q) + half * 8) = pk;
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0)
    block_barrier();
    // (the reads of up to four rows are issued together, then their stores: one trip to LDS per batch, not per store)
    const int f = nt * (BN / 2) + (wave / 2) * 64 + (lane % 8) * 8;
#pragma unroll
    for (int k0 = 0; k0 < 2 * FM; k0 += 4) {
      u32x4 v[4];
#pragma unroll
      for (int k = k0; k < k0 + 4 && k < 2 * FM; ++k)
        v[k - k0] = *(const u32x4*)(block + staged_at((wave % 2) * FM * 16 + k * 8 + lane / 8, lane % 8));
      __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0)
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int k = k0; k < k0 + 4 && k < 2 * FM; ++k) {
        const int m = m0 + (wave % 2) * FM * 16 + k * 8 + lane / 8;
        if (m < m_rows && f < n_out) store_16(out + (size_t)(row_first + m) * n_out + f, v[k - k0]);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  }
  static __device__ __forceinline__ void epilogue_lines_down_walk_tr(const TiledCtx& c, bf16_t* __restrict__ out,
                                                                     const TileLoc& loc, Acc& acc, u32x4* staging, int wave,
                                                                     int lane) {
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
      for (int j = 0; j < FN; ++j) asm volatile("" : "+a"(acc[i][j]));
    const int row_first = loc.row_first, m_rows = loc.m_rows, nt = loc.nt;
    const int n_out = c.hidden;
    const int m0 = loc.m0;
    const int half = lane / 32, rl = lane % 32;
    char* block = (char*)(staging + wave * 64 * 8);  // two [32 rows][64 columns] halves, the wave's own
    const int n = nt * BN + wave * 64 + (lane % 8) * 8;
    // Fragment by fragment through the two halves in turn: the next fragment is converted and written while the reads
    // of this one are on their way, so the trips to LDS overlap the conversions instead of following them.  (LDS
    // serves a wave's accesses in order: the reads see the writes before them, and a half is written again only
    // after its reads have come back, two fragments later.)
    auto write_fragment = [&](int i) {
      const int row = (i % 2) * 32 + rl;
#pragma unroll
      for (int j = 0; j < FN; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          uint2 pk;
          pk.x = f32_to_bf16_pair(acc[i][j][q * 4 + 0], acc[i][j][q * 4 + 1]);
          pk.y = f32_to_bf16_pair(acc[i][j][q * 4 + 2], acc[i][j][q * 4 + 3]);
          *(uint2*)(block + staged_at(row, j * 4 + q) + half * 8) = pk;
        }
    };
    write_fragment(0);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < FM; ++i) {
      u32x4 v[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) v[k] = *(const u32x4*)(block + staged_at((i % 2) * 32 + k * 8 + lane / 8, lane % 8));
      __builtin_amdgcn_sched_barrier(0);
      if (i + 1 < FM) write_fragment(i + 1);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const int m = m0 + i * 32 + k * 8 + lane / 8;
        if (m < m_rows && n < n_out) store_16(out + (size_t)(row_first + m) * n_out + n, v[k]);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  }
  // Down projection with one weight group per wave: a wave's 32 columns are a quarter of a line.  The block collects
  // the tile's bf16 results in the idle activation ring, [rows][32 * NWV columns], and every thread stores whole
  // 16-byte pieces of whole lines.
  static __device__ __forceinline__ void epilogue_lines_block(const TiledCtx& c, bf16_t* __restrict__ out, const TileLoc& loc,
                                                              const Acc& acc, u32x4* lds) {
    static_assert(FM * 32 * BN * 2 <= LDS_VEC * 16, "the tile's results must fit the activation ring");
    const int row_first = loc.row_first, m_rows = loc.m_rows, nt = loc.nt;
    const int n_out = c.hidden;
    const int m0 = loc.mt * MSTRIDE;
    const int tid = threadIdx.x, wave = tid / 64, lane = tid % 64;
    const int half = lane / 32, col = lane % 32;
    bf16_t* staged = (bf16_t*)lds;
    block_barrier();  // every wave has read its last activation fragments
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        staged[(i * 32 + (r / 4) * 8 + half * 4 + (r % 4)) * BN + wave * 32 + col] = f32_to_bf16(acc[i][0][r]);
    __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0)
    block_barrier();
#pragma unroll
    for (int id = tid; id < FM * 32 * BN / 8; id += THREADS) {
      const int row = id / (BN / 8), cc = (id % (BN / 8)) * 8;
      const int m = m0 + row, n = nt * BN + cc;
      if (m < m_rows && n < n_out)
        *(u32x4*)(out + (size_t)(row_first + m) * n_out + n) = *(const u32x4*)(staged + row * BN + cc);
    }
  }
};

// ---------------------------------------------------------------------------------------------
// Kernels over a tile type.

template <class TILE>
__device__ __forceinline__ void zero_acc(typename TILE::Acc& acc) {
#pragma unroll
  for (int i = 0; i < TILE::FM; ++i)
#pragma unroll
    for (int j = 0; j < TILE::FN; ++j) acc[i][j] = f32x16_t{0};
}

template <class TILE>
__device__ __forceinline__ void run_tile(const TiledCtx& c, const bf16_t* __restrict__ in, bf16_t* __restrict__ out,
                                         const TileLoc& loc, u32x4* lds) {
  typename TILE::Acc acc;
  zero_acc<TILE>(acc);
  // A 224-row tile with two weight groups per wave keeps its accumulators in the second half of the register file
  // (one wave per SIMD, 512 registers).  A fitted instantiation needs fewer of them than the full tile, and the
  // register allocator would park weight-ring values in the free ones -- copying a register whose hand-issued load
  // has not landed.  Holding the unused accumulator registers over the tile leaves it nowhere to park.
  constexpr int HELD = TILE::BM == 224 && TILE::FN == 2 ? 14 - TILE::FM * TILE::FN : 0;
  f32x16_t held[HELD > 0 ? HELD : 1];
#pragma unroll
  for (int i = 0; i < HELD; ++i) asm volatile("" : "=a"(held[i]));
  TILE::mainloop(c, in, loc, 0, (TILE::GATEUP ? c.hidden : c.ffn) / TILE::BKT, lds, acc);
  TILE::epilogue(c, out, loc, acc, lds);
#pragma unroll
  for (int i = 0; i < HELD; ++i) asm volatile("" ::"a"(held[i]));
}

// One block per tile, tile height fitted to the expert.  An expert of R rows has ceil(R / 128) m-tiles whatever
// their height; instead of 128 rows each (the last one mostly padding when R is just above a multiple of 128)
// they all get ceil(R / tiles) rows, rounded up to whole 32-row fragments, and the block runs the tile type
// that multiplies that many fragments.  The m-tiles of one weight panel stay equally long -- their blocks run
// side by side and share the panel through L2, which uneven tiles would break -- and the padding rows that are
// multiplied drop from up to 127 to at most 31 per m-tile.
//
// Two waves per SIMD either way (the second launch bound caps the kernel at 256 registers): one block of 8 waves, or
// two blocks of 4 waves whose ring fill and epilogue overlap each other's main loop.  Left to itself the compiler
// gives the 4-wave kernel 480 registers and the CU a single block.  With 256 registers the 4-wave tile has room for
// a weight ring of one K step only.
template <bool GATEUP, int NWV, bool NT>
__global__ __launch_bounds__(64 * NWV, 2) void ffn_tile_fit_kernel(TiledCtx c, const bf16_t* __restrict__ in,
                                                                 bf16_t* __restrict__ out) {
  constexpr int RING = NWV == 4 ? 4 : 8;
  typedef StreamTile<GATEUP, 128, NWV, 4, NT, RING, 4> FULL;
  __shared__ u32x4 lds[FULL::LDS_VEC];
  TileLoc loc;
  if (!locate_tile<128>(c, loc)) return;  // uniform over the block
  const int tiles = (loc.m_rows + 127) / 128;
  const int fragments = ((loc.m_rows + tiles - 1) / tiles + 31) / 32;  // per m-tile, 1..4; uniform
  if (fragments == 4) run_tile<FULL>(c, in, out, loc, lds);
  else if (fragments == 3) run_tile<StreamTile<GATEUP, 128, NWV, 4, NT, RING, 3>>(c, in, out, loc, lds);
  else if (fragments == 2) run_tile<StreamTile<GATEUP, 128, NWV, 4, NT, RING, 2>>(c, in, out, loc, lds);
  else run_tile<StreamTile<GATEUP, 128, NWV, 4, NT, RING, 1>>(c, in, out, loc, lds);
}

template <bool GATEUP, int NWV, bool NT>
static void launch_tiles_fit(TiledCtx c, int n_rows, const bf16_t* in, bf16_t* out, hipStream_t s) {
  const int n_total = GATEUP ? 2 * c.ffn : c.hidden;
  c.n_tiles_n = (n_total + NWV * 64 - 1) / (NWV * 64);
  c.grid_padded = (int)((tiles_upper_bound(c, n_rows, 128) + 7) / 8 * 8);
  hipLaunchKernelGGL((ffn_tile_fit_kernel<GATEUP, NWV, NT>), dim3((unsigned)c.grid_padded), dim3(64 * NWV), 0, s, c, in, out);
}

// The same with tiles of up to 256 rows and one weight group per wave (tile width 32 * NWV columns): an expert of
// 129..256 rows takes one m-tile instead of two.  Heights come in steps of two fragments.
template <bool GATEUP, int NWV, bool NT>
__global__ __launch_bounds__(64 * NWV) void ffn_tile_fit256_kernel(TiledCtx c, const bf16_t* __restrict__ in,
                                                                    bf16_t* __restrict__ out) {
  typedef StreamTile<GATEUP, 256, NWV, 4, NT, 8, 8, 1> FULL;
  __shared__ u32x4 lds[FULL::LDS_VEC];
  TileLoc loc;
  if (!locate_tile<256>(c, loc)) return;  // uniform over the block
  const int tiles = (loc.m_rows + 255) / 256;
  const int fragments = ((loc.m_rows + tiles - 1) / tiles + 31) / 32;  // per m-tile, 1..8; uniform
  if (fragments > 6) run_tile<FULL>(c, in, out, loc, lds);
  else if (fragments > 4) run_tile<StreamTile<GATEUP, 256, NWV, 4, NT, 8, 6, 1>>(c, in, out, loc, lds);
  else if (fragments > 2) run_tile<StreamTile<GATEUP, 256, NWV, 4, NT, 8, 4, 1>>(c, in, out, loc, lds);
  else run_tile<StreamTile<GATEUP, 256, NWV, 4, NT, 8, 2, 1>>(c, in, out, loc, lds);
}

template <bool GATEUP, int NWV, bool NT>
static void launch_tiles_fit256(TiledCtx c, int n_rows, const bf16_t* in, bf16_t* out, hipStream_t s) {
  const int n_total = GATEUP ? 2 * c.ffn : c.hidden;
  c.n_tiles_n = (n_total + NWV * 32 - 1) / (NWV * 32);
  c.grid_padded = (int)((tiles_upper_bound(c, n_rows, 256) + 7) / 8 * 8);
  hipLaunchKernelGGL((ffn_tile_fit256_kernel<GATEUP, NWV, NT>), dim3((unsigned)c.grid_padded), dim3(64 * NWV), 0, s, c, in, out);
}

// Tiles of up to 224 rows with TWO weight groups per wave: 224x256 with four waves, one wave per SIMD, the 224
// accumulator registers of a wave in the second half of its register file (256 rows would fill that half to the last
// register, which the register allocator does not manage without spilling).  A CU then pulls (224 + 256) * 2 bytes
// per k for 224 x 256 products, against (128 + 256) * 2 for 128 x 256 with two resident 128x256 blocks.  With one
// wave per SIMD nothing hides what a wave issues between its matrix instructions: see ILV in StreamTile::steps.
// Gate/up only (a tuning variant; the walking blocks below are what the library chooses).
template <bool GATEUP, bool NT>
__global__ __launch_bounds__(256) void ffn_tile_fit256w_kernel(TiledCtx c, const bf16_t* __restrict__ in,
                                                                bf16_t* __restrict__ out) {
  typedef StreamTile<GATEUP, 224, 4, 4, NT, 8, 7, 2, true> FULL;
  __shared__ u32x4 lds[FULL::LDS_VEC];
  TileLoc loc;
  if (!locate_tile<224>(c, loc)) return;  // uniform over the block
  const int tiles = (loc.m_rows + 223) / 224;
  const int fragments = ((loc.m_rows + tiles - 1) / tiles + 31) / 32;  // per m-tile, 1..7; uniform
  if (fragments > 6) run_tile<FULL>(c, in, out, loc, lds);
  else if (fragments > 5) run_tile<StreamTile<GATEUP, 224, 4, 4, NT, 8, 6, 2, true>>(c, in, out, loc, lds);
  else if (fragments > 4) run_tile<StreamTile<GATEUP, 224, 4, 4, NT, 8, 5, 2, true>>(c, in, out, loc, lds);
  else run_tile<StreamTile<GATEUP, 224, 4, 4, NT, 8, 4, 2, true>>(c, in, out, loc, lds);
}

template <bool GATEUP, bool NT>
static void launch_tiles_fit256w(TiledCtx c, int n_rows, const bf16_t* in, bf16_t* out, hipStream_t s) {
  const int n_total = GATEUP ? 2 * c.ffn : c.hidden;
  c.n_tiles_n = (n_total + 255) / 256;
  c.grid_padded = (int)((tiles_upper_bound(c, n_rows, 224) + 7) / 8 * 8);
  hipLaunchKernelGGL((ffn_tile_fit256w_kernel<GATEUP, NT>), dim3((unsigned)c.grid_padded), dim3(256), 0, s, c, in, out);
}

// The 224x256 tile in a block that works through several tiles (one block per CU, every eighth of the tile list dealt
// to the blocks of one XCD in turn).  A tile's last two K steps issue the first loads and copies of the block's next
// tile (see StreamTile::steps_walk), so their latency passes under those steps and the epilogue instead of in front of
// the next K loop.  The activation ring has three stages of the full tile height whatever the tile's own, and the
// epilogue a staging region of its own; every vector-memory operation of the kernel after the tile table is issued
// by hand, except the row-map lookups at the start of a tile, where nothing else is in flight.
//
// first loads and copies of a block's first tile (fm copies per thread and stage, into stages 0 and 1)
template <class TILE>
__device__ __forceinline__ void walk_issue_prologue(const typename TILE::RowSrc& src, uint32_t lds0, int wave, int fm,
                                                    u32x4 (&ring)[8][2]) {
#pragma unroll
  for (int s = 0; s < 8; ++s)
#pragma unroll
    for (int j = 0; j < 2; ++j) ring[s][j] = src.b_at(j, (size_t)s * 64);
#pragma unroll
  for (int st = 0; st < 2; ++st)
#pragma unroll
    for (int op = 0; op < 7; ++op)
      if (op < fm) TILE::copy_to_stage(src.a_at(op, (size_t)st * 8), lds0, wave, st, op);  // uniform
}
// every vector-memory operation of the thread has completed; the operands tie the weight ring to the wait
__device__ __forceinline__ void walk_wait_ring(u32x4 (&r)[8][2]) {
  asm volatile("s_waitcnt vmcnt(0)"
               : "+v"(r[0][0]), "+v"(r[0][1]), "+v"(r[1][0]), "+v"(r[1][1]), "+v"(r[2][0]), "+v"(r[2][1]), "+v"(r[3][0]),
                 "+v"(r[3][1]), "+v"(r[4][0]), "+v"(r[4][1]), "+v"(r[5][0]), "+v"(r[5][1]), "+v"(r[6][0]), "+v"(r[6][1]),
                 "+v"(r[7][0]), "+v"(r[7][1])
               :
               : "memory");
}

// One tile of fm == FM fragments.  In: loc, ring, stage and the thread's seven input rows at rows_lds (a slot of its own
// per thread and copy, in LDS: registers are short over the K loop) describe the tile, whose first loads have landed.
// Out: the same for the block's next tile (more: whether there is one), its first loads landed as well.
template <bool GATEUP, bool NT, int FM>
__device__ __forceinline__ void walk_one_tile(const TiledCtx& c, const bf16_t* __restrict__ in, bf16_t* __restrict__ out,
                                              const TileWalk<4>& walk, int xcd, int stride, int wave, int lane, int k_steps,
                                              u32x4* lds, uint32_t lds0, TileLoc& loc, int& idx, int& fm, bool& more, int& stage,
                                              int* rows_lds, u32x4 (&ring)[8][2]) {
  typedef StreamTile<GATEUP, 224, 4, 3, NT, 8, FM, 2, true, true> TILE;
  typedef StreamTile<GATEUP, 224, 4, 3, NT, 8, 7, 2, true, true> FULL;
  // The next tile is looked up before this tile's K loop, and the row-map entries of its copies are requested here,
  // where nothing issued by hand is in flight.  A block at its last tile looks that tile up once more, and its last
  // K steps load that tile's first steps once more, unused.
  const TileLoc done = loc;
  idx += stride;
  more = walk.at(xcd, idx, loc);  // leaves loc as it is when there is no further tile
  fm = loc.fm;
  // Input rows of this tile's copies and of the next tile's.  Gate/up (rows looked up in the row map): this tile's
  // come from the thread's slots in LDS, where the next tile's then go until the K loop's other steps are through.
  // Down projection: plain arithmetic, done where the rows are needed.
  int rows[7], rows_next[7];
  if constexpr (GATEUP) {
#pragma unroll
    for (int i = 0; i < 7; ++i) rows[i] = rows_lds[i * 256];
    int lane_rows = lane;  // (opaque copies of the lane id: what is derived from it is recomputed where it is used)
    asm volatile("" : "+v"(lane_rows));
    FULL::fetch_rows(c, loc, loc.m0, wave, lane_rows, rows_next);
  } else {
    int lane_rows = lane;
    asm volatile("" : "+v"(lane_rows));
    FULL::fetch_rows(c, done, done.m0, wave, lane_rows, rows);
  }
  typename TILE::Acc acc;
  zero_acc<TILE>(acc);
  if constexpr (GATEUP) {
    // The lookups are waited for here, before the first load issued by hand (a wait of the compiler's further down
    // would count the hand-issued loads as its own and drain them), and turned into input rows.
#pragma unroll
    for (int i = 0; i < 7; ++i) asm volatile("" : "+v"(rows_next[i]));
    FULL::input_rows(c, rows_next);
#pragma unroll
    for (int i = 0; i < 7; ++i) rows_lds[i * 256] = rows_next[i];
  }
  int lane_steps = lane;
  asm volatile("" : "+v"(lane_steps));
  auto then = [&]() __attribute__((always_inline)) {
    // (made here, so that the next tile's addresses are not held over this tile's other steps)
    int lane_then = lane;
    asm volatile("" : "+v"(lane_then));
    if constexpr (GATEUP) {
#pragma unroll
      for (int i = 0; i < 7; ++i) {
        rows_next[i] = rows_lds[i * 256];
        asm volatile("" : "+v"(rows_next[i]));
      }
    } else {
      FULL::fetch_rows(c, loc, loc.m0, wave, lane_then, rows_next);
    }
    return TILE::row_sources(c, in, loc, rows_next, wave, lane_then);
  };
  TILE::steps_walk(TILE::row_sources(c, in, done, rows, wave, lane_steps), then, lds, wave, lane_steps, k_steps, stage, ring, acc);
  int lane_there = lane;
  asm volatile("" : "+v"(lane_there));
  if constexpr (GATEUP) TILE::epilogue_lines_walk_tr(c, out, done, acc, lds + FULL::LDS_VEC, wave, lane_there);
  else TILE::epilogue_lines_down_walk_tr(c, out, done, acc, lds + FULL::LDS_VEC, wave, lane_there);
  walk_wait_ring(ring);
  // A next tile that is higher than this one: its last rows were not copied (this tile's steps copy FM row blocks).
  if (fm > FM) {  // uniform
    const int s0 = stage, s1 = stage + 1 == 3 ? 0 : stage + 1;
#pragma unroll
    for (int op = FM; op < 7; ++op)
      if (op < fm) {
        const typename FULL::RowSrc src = FULL::row_sources(c, in, loc, rows_next, wave, lane_there);
        FULL::copy_to_stage(src.a_at(op, 0), lds0, wave, s0, op);
        FULL::copy_to_stage(src.a_at(op, 8), lds0, wave, s1, op);
      }
    wait_vmcnt<0>();
  }
}

// DENSE: the launch is a single expert over all rows (a layer's shared experts).  The code is the same; the two are
// separate kernels so that traces and counter runs tell the shared experts' launches from the routed ones, which
// have the same grid.
template <bool GATEUP, bool NT, bool DENSE>
__global__ __launch_bounds__(256) void ffn_tile_walk_kernel(TiledCtx c, const bf16_t* __restrict__ in,
                                                             bf16_t* __restrict__ out) {
  typedef StreamTile<GATEUP, 224, 4, 3, NT, 8, 7, 2, true, true> FULL;
  constexpr int STAGING = 2 * 7 * 32 * 8;  // two [224][64] bf16 blocks, in 16-byte units
  __shared__ u32x4 lds[FULL::LDS_VEC + STAGING];
  __shared__ int walk_table[TileWalk<4>::TABLE_INTS];
  __shared__ int walk_rows[7 * 256];  // input rows of the copies of the tile at hand, then of the next: [copy][thread]
  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) u32x4*)lds;
  const int tid = threadIdx.x, lane = tid % 64;
  const int wave = __builtin_amdgcn_readfirstlane(tid / 64);
  TileWalk<4> walk;
  walk.init(c, walk_table);
  const int xcd = blockIdx.x % 8, stride = gridDim.x / 8;
  int idx = blockIdx.x / 8;
  TileLoc loc;
  if (!walk.at(xcd, idx, loc)) return;  // uniform over the block
  const int k_steps = (GATEUP ? c.hidden : c.ffn) / 64;  // even, at least 6 (the launch sees to it)
  int rows[7];  // input rows of the thread's copies
  u32x4 ring[8][2];
  int fm = loc.fm;
  int stage = 0;
  FULL::fetch_rows(c, loc, loc.m0, wave, lane, rows);
  FULL::input_rows(c, rows);
#pragma unroll
  for (int i = 0; i < 7; ++i) walk_rows[i * 256 + tid] = rows[i];
  walk_issue_prologue<FULL>(FULL::row_sources(c, in, loc, rows, wave, lane), lds0, wave, fm, ring);
  walk_wait_ring(ring);
  bool more = true;
#define HMOE_WALK_TILE(FM_) \
  walk_one_tile<GATEUP, NT, FM_>(c, in, out, walk, xcd, stride, wave, lane, k_steps, lds, lds0, loc, idx, fm, more, stage, \
                                 walk_rows + tid, ring)
  while (more) {
    if (fm == 7) HMOE_WALK_TILE(7);
    else if (fm == 6) HMOE_WALK_TILE(6);
    else if (fm == 5) HMOE_WALK_TILE(5);
    else HMOE_WALK_TILE(4);
  }
#undef HMOE_WALK_TILE
}

template <bool GATEUP, bool NT>
static void launch_tiles_walk(TiledCtx c, int n_rows, const bf16_t* in, bf16_t* out, hipStream_t s) {
  const int n_total = GATEUP ? 2 * c.ffn : c.hidden;
  c.n_tiles_n = (n_total + 255) / 256;
  // The most fragments an m-tile may have.  Lower heights for launches of few rounds (whose partly filled last round
  // weighs more) were measured: a dense expert alone gains 10-23 %, routed experts lose 8 %, and the layer, whose
  // two FFNs overlap, stays where it is; 7 is kept.
  int cap = 7;
  if (const char* env = getenv("HMOE_WALK_CAP")) {  // tuning
    const int want = atoi(env);
    if (want >= 4 && want <= 7) cap = want;
  }
  c.walk_bm = 32 * cap;
  if ((GATEUP ? c.hidden : c.ffn) % 128 != 0 || (GATEUP ? c.hidden : c.ffn) < 384) {  // they need an even number of K steps, 6 or more
    launch_tiles_fit<GATEUP, 4, NT>(c, n_rows, in, out, s);
    return;
  }
  const long bound = (tiles_upper_bound(c, n_rows, c.walk_bm) + 7) / 8 * 8;
  long blocks = bound < 256 ? bound : 256;  // one per CU
  if (const char* env = getenv("HMOE_WALK_BLOCKS")) {  // tuning and tests: fewer blocks, more tiles each
    const long want = atol(env) / 8 * 8;
    if (want >= 8 && want < blocks) blocks = want;
  }
  c.grid_padded = (int)blocks;
  if (!NT && c.n_experts == 1)  // (what the library itself chooses for shared experts: plain loads)
    hipLaunchKernelGGL((ffn_tile_walk_kernel<GATEUP, false, true>), dim3((unsigned)c.grid_padded), dim3(256), 0, s, c, in, out);
  else
    hipLaunchKernelGGL((ffn_tile_walk_kernel<GATEUP, NT, false>), dim3((unsigned)c.grid_padded), dim3(256), 0, s, c, in, out);
}

// Tile shapes built into the library.  hmoe picks one from the average rows per expert; the
// environment variable HMOE_TILED_VARIANT (an index into this table) overrides the choice for
// tuning runs.
typedef void (*tiled_launch_fn)(TiledCtx, int, const bf16_t*, bf16_t*, hipStream_t);
struct TiledVariant {
  const char* name;
  tiled_launch_fn gate_up, down;
};
#define HMOE_STREAM_FIT(NAME, NWV, NT) { NAME, launch_tiles_fit<true, NWV, NT>, launch_tiles_fit<false, NWV, NT> }
#define HMOE_STREAM_FIT256(NAME, NWV_GU, NWV_D, NT) \
  { NAME, launch_tiles_fit256<true, NWV_GU, NT>, launch_tiles_fit256<false, NWV_D, NT> }
enum {
  V_FIT = 0,            // 128x512 tile, 8 waves, tile height fitted to the expert, non-temporal weight loads
  V_FIT_PLAIN = 1,      //   ... with plain weight loads
  V_FIT4 = 2,           // 128x256 tile, 4 waves, half the weight ring: two blocks per CU
  V_FIT4_PLAIN = 3,
  V_FIT256 = 4,         // tiles of up to 256 rows, one weight group per wave: 256x256 (gate/up, 8 waves), 256x128 (down, 4 waves)
  V_FIT256_PLAIN = 5,
  V_FIT256W = 6,        // gate/up: 224x256, 4 waves, two weight groups per wave, one wave per SIMD (down: as 0 / 1)
  V_FIT256W_PLAIN = 7,
  V_WALK = 8,           // the same tile in blocks that work through several tiles each
  V_WALK_PLAIN = 9
};
static const TiledVariant kVariants[] = {
    HMOE_STREAM_FIT("stream 128x512 fit", 8, true),
    HMOE_STREAM_FIT("stream 128x512 fit plain", 8, false),
    HMOE_STREAM_FIT("stream 128x256 fit, 4 waves", 4, true),
    HMOE_STREAM_FIT("stream 128x256 fit, 4 waves, plain", 4, false),
    HMOE_STREAM_FIT256("stream 256x256/128 fit", 8, 4, true),
    HMOE_STREAM_FIT256("stream 256x256/128 fit plain", 8, 4, false),
    {"stream 224x256, 4 waves", launch_tiles_fit256w<true, true>, launch_tiles_fit<false, 8, true>},
    {"stream 224x256, 4 waves, plain", launch_tiles_fit256w<true, false>, launch_tiles_fit<false, 8, false>},
    {"stream 224x256, walking blocks", launch_tiles_walk<true, true>, launch_tiles_walk<false, true>},
    {"stream 224x256, walking blocks, plain", launch_tiles_walk<true, false>, launch_tiles_walk<false, false>},
};
constexpr int kNumVariants = sizeof(kVariants) / sizeof(kVariants[0]);

int launch_ffn_tiled(const FfnArgs& a) {
  const hmoe_layer_desc& d = *a.desc;
  if (d.dtype != HMOE_BF16) return HMOE_ERR_UNSUPPORTED;
  if (a.n_rows == 0) return HMOE_OK;
  TiledCtx c{a.offsets, a.slot_of, a.slots, a.slot_bytes, a.active, d.n_experts, d.hidden, d.ffn, 0, 0, a.row_map, a.map_div};
  set_map_div(c);
  const bf16_t* x = (const bf16_t*)a.x_perm;
  bf16_t* h = (bf16_t*)a.h;
  bf16_t* o = (bf16_t*)a.o_perm;
  // Kernel choice (measured on the workload shapes and on batch-size sweeps of them; the tile counts are the
  // launch's upper bounds).
  //  * Experts of fewer than 192 rows on average stream each weight byte about once: 128x512 tiles with 8 waves,
  //    the tile height fitted to the expert, non-temporal weight loads.  When such a launch has too few tiles to
  //    fill the CUs, the time of one tile is what counts and it takes tiles of up to 256 rows and 32 columns per
  //    wave: each wave multiplies as little as the expert needs, and an expert of up to 256 rows streams its
  //    weights once.  Gate/up over a short K range (hidden < 4096) with experts of at most 32 rows on average takes
  //    the 128x256 tile with 4 waves, two blocks per CU: 2-10 % on the DeepSeek-style and Qwen2-style shapes up
  //    to 256 tokens (with a long K range the deeper weight ring of the 8-wave tile is worth more; with larger
  //    experts under skewed routing the non-temporal loads of several m-tiles per panel cost more than it gains).
  //  * Experts of 192 rows or more (a shared expert at a prefill batch, large routed experts) have several
  //    m-tiles that share their weight panel through L2: plain loads, and 128x256 tiles with 4 waves, two blocks
  //    per CU, so that one block's ring fill and epilogue overlap the other's main loop (4-14 % over the 8-wave
  //    tile on compute-bound launches).  The down projection keeps the 128x512 tile when its K range is short
  //    and its tiles are plenty (F < 4096: the stress and Qwen2 shapes, 1-2 % either way).
  const long m_tiles = (long)a.n_rows / 128 + std::min(d.n_experts, a.n_rows);
  const long tiles_down = m_tiles * ((d.hidden + 511) / 512);
  const bool few_gate_up = m_tiles * ((2 * d.ffn + 255) / 256) <= 128;
  const bool shared_panels = a.n_rows / d.n_experts >= 192;
  int v_gate_up = V_FIT, v_down = V_FIT;
  if (shared_panels) {
    v_gate_up = V_FIT4_PLAIN;
    v_down = tiles_down < 256 || d.ffn >= 4096 ? V_FIT4_PLAIN : V_FIT_PLAIN;
    // A layer whose routed experts make at least seven rounds of 224x256 tiles (a large batch) takes that tile with
    // one wave per SIMD, in blocks that walk through their tiles -- for both projections, and for the layer's shared
    // experts too (hmoe_cache_set_layer tells their launches which layer they run beside): stress shape -3.5 % per
    // layer, Qwen2 shape unchanged.  A block of these fills its CU, one of the other kernels half of one, and
    // launches of both kinds next to each other on two streams keep each other waiting (+2 %); alone, a dense
    // expert of a few rounds is 3-25 % slower with the large tile (its last, partly filled round).
    const hmoe_layer_desc& lay = a.beside ? *a.beside : d;
    const long lay_rows = a.beside ? (long)a.n_rows * lay.top_k : a.n_rows;
    const long m_tiles_224 = lay_rows / 224 + std::min((long)lay.n_experts, lay_rows);
    long min_rounds = 7;
    if (const char* env = getenv("HMOE_WALK_MIN_ROUNDS")) min_rounds = atol(env);  // tuning
    if (lay_rows / lay.n_experts >= 192 &&
        m_tiles_224 * ((2 * lay.ffn + 255) / 256) >= min_rounds * 256) v_gate_up = v_down = V_WALK_PLAIN;
  } else {
    if (few_gate_up) v_gate_up = V_FIT256;
    else if (d.hidden < 4096 && a.n_rows <= 32 * d.n_experts) v_gate_up = V_FIT4;
    // Experts of 96 to 191 rows on average: gate/up in walking blocks (non-temporal loads), whose weight stream does
    // not stop between tiles -- Mixtral shape at 512 tokens 405 -> 357 us, Qwen2 shape at 1024 tokens 480 -> 427 us,
    // DeepSeek-style at 1024 tokens 186 -> 181 us; below 96 rows the fitted tiles are faster (fewer padded rows).
    else if ((long)a.n_rows >= 96L * d.n_experts) v_gate_up = V_WALK;
    if (tiles_down < 256) v_down = V_FIT256;
  }
  if (const char* env = getenv("HMOE_TILED_VARIANT")) {
    // "<index>" for both projections or "<gate/up index>,<down index>"
    const int want_gate_up = atoi(env);
    const char* comma = strchr(env, ',');
    const int want_down = comma ? atoi(comma + 1) : want_gate_up;
    if (want_gate_up >= 0 && want_gate_up < kNumVariants) v_gate_up = want_gate_up;
    if (want_down >= 0 && want_down < kNumVariants) v_down = want_down;
  }
  probe_before(a.stream);
  kVariants[v_gate_up].gate_up(c, a.n_rows, x, h, a.stream);
  probe_after(a.stream);
  probe_before(a.stream);
  kVariants[v_down].down(c, a.n_rows, h, o, a.stream);
  probe_after(a.stream);
  HMOE_HIP(hipGetLastError());
  return HMOE_OK;
}

}  // namespace hmoe
