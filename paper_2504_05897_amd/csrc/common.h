// Internal declarations shared by the HIP sources of libhmoe (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <vector>

#include "hmoe.h"

namespace hmoe {

typedef uint16_t bf16_t;  // bfloat16 storage
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // 16 bytes = 8 bf16
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));  // MFMA operand
typedef float f32x16_t __attribute__((ext_vector_type(16)));  // 32x32 MFMA accumulator

// D = A(32x16) * B(16x32) + C.  Lane l supplies A[l%32][8*(l/32) .. +8] and B[8*(l/32) .. +8][l%32];
// accumulator register r of lane l is D[8*(r/4) + 4*(l/32) + r%4][l%32].
__device__ __forceinline__ f32x16_t mfma_32x32x16_bf16(u32x4 a, u32x4 b, f32x16_t c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c,
                                                 0, 0, 0);
}

// D = A(16x32) * B(32x16) + C.  Lane l supplies A[l%16][8*(l/16) .. +8] and B[8*(l/16) .. +8][l%16];
// accumulator register r of lane l is D[4*(l/16) + r][l%16].
typedef float f32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ f32x4_t mfma_16x16x32_bf16(u32x4 a, u32x4 b, f32x4_t c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c,
                                                 0, 0, 0);
}

__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }

// round to nearest, ties to even (inputs are finite on this path)
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

// two at once: the low half of the result is a, the high half b (same rounding; one instruction on gfx950)
typedef __bf16 bf16x2_hw_t __attribute__((ext_vector_type(2)));
typedef float f32x2_hw_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t f32_to_bf16_pair(float a, float b) {
  const f32x2_hw_t v = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_hw_t));
}

// source row of sorted row p (gather fused into the FFN's first GEMM when a row map is given)
__device__ __forceinline__ int mapped_row(const int32_t* __restrict__ row_map, int map_div, int p) {
  return row_map ? row_map[p] / map_div : p;
}

// silu(g) = g / (1 + exp(-g)) with the hardware reciprocal (1 ulp) in place of an IEEE division: the result is
// rounded to bf16 right away, and the division costs ten vector instructions per element in the epilogues.
__device__ __forceinline__ float silu_f32(float g) { return g * __builtin_amdgcn_rcpf(1.0f + __expf(-g)); }

// Experts taking part in one FFN call, one bit per expert id.
struct ActiveMask {
  uint64_t w[HMOE_MAX_EXPERTS / 64];
  __host__ __device__ bool test(int e) const { return (w[e >> 6] >> (e & 63)) & 1ull; }
};

// --- packed bf16 weight layout ---------------------------------------------------------
// A matrix W [N, K] (row = output feature, K contiguous) is cut into tiles of 32 rows x 16 k.
// A tile is 1 KiB, stored in the register order of one 32x32x16 bf16 MFMA operand: lane l of
// a wavefront owns the 8 consecutive k values  W[32*nb + l%32][16*kb + 8*(l/32) .. +8].
// Tiles are ordered [nb][kb] (kb fastest), so one 32-row group is one contiguous K stream.
// The gate/up matrix of an expert interleaves 32-row groups: packed group 2q is W_gate rows
// 32q..32q+31, group 2q+1 is W_up rows 32q..32q+31; the SwiGLU product then needs no data
// movement between lanes.  A slot holds [gate/up: 2F x H][down: H x F].
constexpr int TILE_N = 32;
constexpr int TILE_K = 16;
constexpr int TILE_ELEMS = TILE_N * TILE_K;  // 512 bf16 = 1 KiB

__host__ __device__ inline size_t packed_index(int n, int k, int k_tiles) {
  const int nb = n / TILE_N, kb = k / TILE_K;
  const int lane = (n % TILE_N) + TILE_N * ((k % TILE_K) / 8);
  return ((size_t)nb * k_tiles + kb) * TILE_ELEMS + (size_t)lane * 8 + (k % 8);
}

int set_hip_error(hipError_t err, const char* what);
int set_error_text(int status, const char* text);  // text for hmoe_last_error; returns status
int check_desc(const hmoe_layer_desc* d);
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

#define HMOE_HIP(call)                                                  \
  do {                                                                  \
    hipError_t hmoe_e_ = (call);                                        \
    if (hmoe_e_ != hipSuccess) return hmoe::set_hip_error(hmoe_e_, #call); \
  } while (0)

// probe (benchmark timing of the gate/up kernel)
void probe_before(hipStream_t s);
void probe_after(hipStream_t s);

// kernel launchers, one per source file ---------------------------------------------------
// --- 4-bit weight layout (HMOE_BF16_W4) -------------------------------------------------------
// A matrix W [N, K] is stored as a stream of 1 KiB units, each 16 rows x 128 k (one scale group),
// ordered [N/16][K/128] (k fastest), followed by its scales [N/16][K/128][16 rows] in bfloat16.
// Inside a unit lane l of a wavefront (row l % 16, k block l / 16) owns 16 bytes: dword t holds the 8
// codes of k = 128 unit + 32 t + 8 (l / 16) + j, code j at bit 16 (j & 1) + 4 (j >> 1) -- the operand
// order of v_mfma_f32_16x16x32_bf16 (B operand: column l % 16, k = 8 (l / 16) .. + 8), one k-step of 32
// per dword.  With that nibble order ((dword >> 4 i) & 0x000F000F) | 0x43004300 is register i of the
// operand holding the bfloat16 values 128 + q (bfloat16 0x4300 is 128 and its mantissa step there is 1).
// A slot is [gate/up units][gate/up scales][down units][down scales]; gate and up rows are interleaved
// in 16-row groups (packed group 2 q = gate rows 16 q .., 2 q + 1 = up rows 16 q ..).
constexpr int W4_GROUP = 128;
struct W4Offsets {
  size_t gate_up_scales, down_units, down_scales, total;  // byte offsets within a slot (gate/up units at 0)
};
__host__ __device__ inline W4Offsets w4_offsets(size_t hidden, size_t ffn) {
  W4Offsets o;
  const size_t hf = hidden * ffn;
  o.gate_up_scales = hf;                       // 2F x H codes, two per byte
  o.down_units = o.gate_up_scales + hf / 32;   // 2F x H/128 scales of 2 bytes
  o.down_scales = o.down_units + hf / 2;
  o.total = o.down_scales + hf / 64;
  return o;
}
// index of the dword that holds the code of W[n][k] (K columns), and the bit position of the code in it
__host__ __device__ inline size_t w4_dword_index(int n, int k, int K) {
  const int lane = ((k % 32) / 8) * 16 + n % 16;
  return (((size_t)(n / 16) * (K / W4_GROUP) + k / W4_GROUP) * 64 + lane) * 4 + (k % W4_GROUP) / 32;
}
__host__ __device__ inline int w4_code_shift(int k) { return 16 * (k & 1) + 4 * ((k % 8) >> 1); }
__host__ __device__ inline size_t w4_scale_index(int n, int group, int n_groups) {
  return ((size_t)(n / 16) * n_groups + group) * 16 + n % 16;
}

struct FfnArgs {
  const hmoe_layer_desc* desc = nullptr;
  const void* x_perm = nullptr;       // rows of the gate/up input; with row_map: the un-permuted x [T, H]
  const int32_t* row_map = nullptr;   // device [A] or NULL: input row of sorted row p is row_map[p] / map_div
  int32_t map_div = 1;
  const int32_t* offsets = nullptr;   // device [E+1]
  int32_t n_rows = 0;                 // A
  const int32_t* slot_of = nullptr;   // device [E]
  const char* slots = nullptr;        // device slot storage
  size_t slot_bytes = 0;
  ActiveMask active = {};
  void* o_perm = nullptr;
  void* h = nullptr;                  // workspace [A, F]
  hipStream_t stream = nullptr;
  const hmoe_layer_desc* beside = nullptr;  // a dense FFN over all tokens: the routed layer it runs next to, if known
};
// the sum of Eq. (1) computed inside the down projection's launch (decode batches)
struct CombineArgs {
  const int32_t* inv_perm = nullptr;
  const float* topk_w = nullptr;
  void* y = nullptr;
  unsigned int* tickets = nullptr;   // device counters, zero before and after the call
  int32_t n_tokens = 0;
};
int launch_ffn_reference(const FfnArgs& a);
int launch_ffn_skinny(const FfnArgs& a, const FfnArgs* dense = nullptr, const CombineArgs* combine = nullptr);
int launch_ffn_tiled(const FfnArgs& a);
int launch_ffn_skinny_w4(const FfnArgs& a);
int launch_ffn_tiled_w4(const FfnArgs& a);

}  // namespace hmoe

// The host-side cache object behind the opaque handle of the public header.
struct hmoe_cache {
  hmoe_layer_desc desc;
  char* slots;
  size_t slot_bytes;
  int32_t* d_slot_of;
  int device;
  std::vector<int32_t> slot_of;    // [E] host mirror
  std::vector<int32_t> expert_in;  // [S]
  std::vector<int64_t> tick;       // [E] LRU use ticks
  int policy;                      // HMOE_POLICY_*
  double alpha;                    // MRS averaging coefficient
  std::vector<double> score;       // [E] MRS priority estimate S
  int64_t clock;
  std::vector<uint8_t> pinned;     // [S]
  // read tracking: FFN calls record one event each; a slot remembers the sequence number of
  // the last call that may have read it.
  static const int RING = 16;
  hipEvent_t use_ev[RING];
  uint64_t use_seq;
  bool track_reads;
  bool reads_in_graphs;                  // an FFN call over this cache was captured into a HIP graph
  std::vector<uint64_t> slot_last_read;  // [S], 0 = never
  std::vector<hipEvent_t> ready_ev;      // [S]
  hipEvent_t fence_ev;
  hmoe_layer_desc beside;                // hmoe_cache_set_layer: the routed layer these (shared) experts belong to
  bool has_beside;
};
