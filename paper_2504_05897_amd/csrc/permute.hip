// hmoe_permute: stable counting sort of the A = T*K assignments by expert id, then row gather.
//
// Per-expert load is the quantity everything downstream consumes (Section IV-B uses it to order
// the queues); here it becomes expert_offsets.  The sort is stable and uses no order-dependent
// atomics, so the result is the same on every run:
//   1. histogram   every block counts its 1024-assignment chunk per expert in LDS
//   2. scan        one block turns the per-block counts into per-(block, expert) bases and the
//                  per-expert totals into expert_offsets
//   3. rank        every block re-reads its chunk; a wave ranks 64 assignments at a time with
//                  ballots (same-key mask), waves and steps are ordered by per-wave LDS bases
// For A <= 1024 (every decode shape) one block does all three in one launch.
//   4. gather      x_perm[p] = x[perm[p] / K], 16 bytes per lane
#include <mutex>

#include "route_body.h"
#include "router_body.h"

namespace hmoe {

constexpr int PB_THREADS = 256;
constexpr int PB_WAVES = PB_THREADS / 64;
constexpr int PB_CHUNK = 1024;               // assignments per block
constexpr int PB_STEPS = PB_CHUNK / PB_THREADS;  // 64-wide steps per wave

__device__ __forceinline__ int clamp_key(int key, int n_experts) {
  return key < 0 ? 0 : (key >= n_experts ? n_experts - 1 : key);
}

// lanes of this wavefront (among `valid` ones) that hold the same key as the caller
__device__ __forceinline__ uint64_t same_key_mask(int key, bool valid, int key_bits) {
  uint64_t m = __ballot(valid);
  for (int b = 0; b < key_bits; ++b) {
    const bool bit = (key >> b) & 1;
    const uint64_t bal = __ballot(bit);
    m &= bit ? bal : ~bal;
  }
  return m;
}

__global__ __launch_bounds__(PB_THREADS) void permute_hist_kernel(const int32_t* __restrict__ topk_idx, int n_assign,
                                                                  int n_experts, int32_t* __restrict__ block_counts) {
  __shared__ int hist[HMOE_MAX_EXPERTS];
  for (int e = threadIdx.x; e < n_experts; e += PB_THREADS) hist[e] = 0;
  __syncthreads();
  const long base = (long)blockIdx.x * PB_CHUNK;
  for (int i = threadIdx.x; i < PB_CHUNK; i += PB_THREADS) {
    const long a = base + i;
    if (a < n_assign) atomicAdd(&hist[clamp_key(topk_idx[a], n_experts)], 1);
  }
  __syncthreads();
  for (int e = threadIdx.x; e < n_experts; e += PB_THREADS) block_counts[(long)blockIdx.x * n_experts + e] = hist[e];
}

// one block: block_counts[b][e] -> exclusive base of (b, e) in the sorted order; expert_offsets
__global__ __launch_bounds__(PB_THREADS) void permute_scan_kernel(int32_t* __restrict__ block_counts, int n_blocks,
                                                                  int n_experts, int n_assign,
                                                                  int32_t* __restrict__ expert_offsets,
                                                                  int32_t* __restrict__ counts_out) {
  __shared__ int total[HMOE_MAX_EXPERTS];
  __shared__ int start[HMOE_MAX_EXPERTS];
  // (the counts are read 16 blocks at a time: one after the other, a read could not start before the store in
  // front of it, and 96 blocks of the largest workload cost 96 memory round trips)
  constexpr int AHEAD = 16;
  const int e = threadIdx.x;
  if (e < n_experts) {
    int run = 0;
    for (int b0 = 0; b0 < n_blocks; b0 += AHEAD) {
      int c[AHEAD];
#pragma unroll
      for (int i = 0; i < AHEAD; ++i) c[i] = b0 + i < n_blocks ? block_counts[(long)(b0 + i) * n_experts + e] : 0;
#pragma unroll
      for (int i = 0; i < AHEAD; ++i) {
        if (b0 + i < n_blocks) block_counts[(long)(b0 + i) * n_experts + e] = run;
        run += c[i];
      }
    }
    total[e] = run;
    if (counts_out) counts_out[e] = run;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    int run = 0;
    for (int i = 0; i < n_experts; ++i) { start[i] = run; expert_offsets[i] = run; run += total[i]; }
    expert_offsets[n_experts] = run;
  }
  __syncthreads();
  if (e < n_experts) {
    const int s = start[e];
    for (int b0 = 0; b0 < n_blocks; b0 += AHEAD) {
      int c[AHEAD];
#pragma unroll
      for (int i = 0; i < AHEAD; ++i) c[i] = b0 + i < n_blocks ? block_counts[(long)(b0 + i) * n_experts + e] : 0;
#pragma unroll
      for (int i = 0; i < AHEAD; ++i)
        if (b0 + i < n_blocks) block_counts[(long)(b0 + i) * n_experts + e] = c[i] + s;
    }
  }
}

// The whole permutation of at most 64 assignments (every decode batch) by one wavefront, without LDS and
// without barriers: lane a holds assignment a, learns every other key through readlane, and counts the
// keys that sort before its own (smaller key, or equal key in a lower lane: the stable order); lane l
// does the same counting for experts l, 64 + l, ... to produce the offsets.  Same integers as the general
// path.  Call with the first wavefront of a block.
__device__ __forceinline__ void permute_rank_one_wave(const int32_t* topk_idx, int n_assign, int n_experts,
                                                      int32_t* __restrict__ expert_offsets,
                                                      int32_t* __restrict__ counts_out, int32_t* __restrict__ perm,
                                                      int32_t* __restrict__ inv_perm) {
  constexpr int CH = HMOE_MAX_EXPERTS / 64;
  const int lane = threadIdx.x % 64;
  const bool valid = lane < n_assign;
  const int key = valid ? clamp_key(topk_idx[lane], n_experts) : n_experts;
  int before = 0, below[CH], equal[CH];
#pragma unroll
  for (int j = 0; j < CH; ++j) below[j] = equal[j] = 0;
  for (int i = 0; i < n_assign; ++i) {  // uniform
    const int ki = __builtin_amdgcn_readlane(key, i);
    before += (ki < key) | ((ki == key) & (i < lane));
#pragma unroll
    for (int j = 0; j < CH; ++j) {
      below[j] += ki < j * 64 + lane;
      equal[j] += ki == j * 64 + lane;
    }
  }
  if (valid) {
    perm[before] = lane;
    inv_perm[lane] = before;
  }
#pragma unroll
  for (int j = 0; j < CH; ++j) {
    const int e = j * 64 + lane;
    if (e < n_experts) {
      expert_offsets[e] = below[j];
      if (counts_out) counts_out[e] = equal[j];
    }
  }
  if (lane == 0) expert_offsets[n_experts] = n_assign;
}

// Ranks one chunk.  SINGLE: the chunk is the whole input and this block also builds the offsets.
template <bool SINGLE>
__device__ __forceinline__ void permute_rank_body(const int32_t* topk_idx, int n_assign, int n_experts, int key_bits,
                                                  const int32_t* __restrict__ block_bases,
                                                  int32_t* __restrict__ expert_offsets,
                                                  int32_t* __restrict__ counts_out, int32_t* __restrict__ perm,
                                                  int32_t* __restrict__ inv_perm) {
  __shared__ int wave_base[PB_WAVES][HMOE_MAX_EXPERTS];  // first counts, then running bases
  __shared__ int scan_tmp[HMOE_MAX_EXPERTS];
  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
  if (SINGLE && n_assign <= 64) {  // uniform over the block: nothing below runs, so no barrier is left unmatched
    if (wave == 0) permute_rank_one_wave(topk_idx, n_assign, n_experts, expert_offsets, counts_out, perm, inv_perm);
    return;
  }
  for (int i = threadIdx.x; i < PB_WAVES * HMOE_MAX_EXPERTS; i += PB_THREADS) (&wave_base[0][0])[i] = 0;
  __syncthreads();

  // each wave owns a contiguous quarter of the chunk, in PB_STEPS steps of 64
  const long wave_first = (long)blockIdx.x * PB_CHUNK + (long)wave * (PB_STEPS * 64);
  int keys[PB_STEPS];
#pragma unroll
  for (int s = 0; s < PB_STEPS; ++s) {
    const long a = wave_first + s * 64 + lane;
    keys[s] = a < n_assign ? clamp_key(topk_idx[a], n_experts) : -1;
    if (keys[s] >= 0) atomicAdd(&wave_base[wave][keys[s]], 1);
  }
  __syncthreads();

  // counts -> exclusive bases over (expert, wave)
  const int e = threadIdx.x;
  int cnt[PB_WAVES], tot = 0;
  if (e < n_experts) {
#pragma unroll
    for (int w = 0; w < PB_WAVES; ++w) { cnt[w] = wave_base[w][e]; tot += cnt[w]; }
  }
  int first;
  if (SINGLE) {
    // inclusive Hillis-Steele scan of the per-expert totals over the 256 threads
    scan_tmp[threadIdx.x] = e < n_experts ? tot : 0;
    __syncthreads();
    for (int off = 1; off < HMOE_MAX_EXPERTS; off <<= 1) {
      const int add = threadIdx.x >= off ? scan_tmp[threadIdx.x - off] : 0;
      __syncthreads();
      scan_tmp[threadIdx.x] += add;
      __syncthreads();
    }
    first = scan_tmp[threadIdx.x] - tot;
    if (e < n_experts) {
      expert_offsets[e] = first;
      if (counts_out) counts_out[e] = tot;
      if (e == n_experts - 1) expert_offsets[n_experts] = first + tot;
    }
  } else {
    first = e < n_experts ? block_bases[(long)blockIdx.x * n_experts + e] : 0;
  }
  if (e < n_experts) {
    int run = first;
#pragma unroll
    for (int w = 0; w < PB_WAVES; ++w) { wave_base[w][e] = run; run += cnt[w]; }
  }
  __syncthreads();

#pragma unroll
  for (int s = 0; s < PB_STEPS; ++s) {
    const int key = keys[s];
    const bool valid = key >= 0;
    const uint64_t same = same_key_mask(key, valid, key_bits);
    if (valid) {
      const uint64_t below = same & ((1ull << lane) - 1ull);
      const int pos = wave_base[wave][key] + __popcll(below);
      const int a = (int)(wave_first + s * 64 + lane);
      perm[pos] = a;
      inv_perm[a] = pos;
    }
    __syncthreads();  // everyone has read the bases of this step
    if (valid && (same >> lane) >> 1 == 0) wave_base[wave][key] += __popcll(same);  // highest lane of the group
    __syncthreads();
  }
}

template <bool SINGLE>
__global__ __launch_bounds__(PB_THREADS) void permute_rank_kernel(const int32_t* __restrict__ topk_idx, int n_assign,
                                                                  int n_experts, int key_bits,
                                                                  const int32_t* __restrict__ block_bases,
                                                                  int32_t* __restrict__ expert_offsets,
                                                                  int32_t* __restrict__ counts_out,
                                                                  int32_t* __restrict__ perm,
                                                                  int32_t* __restrict__ inv_perm) {
  permute_rank_body<SINGLE>(topk_idx, n_assign, n_experts, key_bits, block_bases, expert_offsets, counts_out, perm,
                            inv_perm);
}

// One block routes its tokens one lane group at a time, so beyond a few dozen tokens the many-block
// route kernel plus the one-block rank kernel are faster than the single launch (measured at 512
// tokens: 10 us against 25 us).
constexpr int ROUTE_PERMUTE_SMALL_T = 64;

// Small batches (T <= 64 and A <= 1024, every decode shape): routing and permutation in ONE block and one launch.
// The block first routes all tokens (lane groups as in hmoe_route), then ranks the assignments it has
// just written.
template <int G, int VPL>
__global__ __launch_bounds__(PB_THREADS) void route_permute_small_kernel(const float* __restrict__ logits, int n_tokens,
                                                                         int n_experts, int top_k, int key_bits,
                                                                         int32_t* topk_idx, float* __restrict__ topk_w,
                                                                         int32_t* __restrict__ expert_offsets,
                                                                         int32_t* __restrict__ counts_out,
                                                                         int32_t* __restrict__ perm,
                                                                         int32_t* __restrict__ inv_perm) {
  constexpr int TOKENS_PER_PASS = PB_THREADS / G;
  for (int t0 = 0; t0 < n_tokens; t0 += TOKENS_PER_PASS) {
    const long token = t0 + threadIdx.x / G;
    route_token<G, VPL>(logits, n_experts, top_k, token, token < n_tokens, threadIdx.x % G, topk_idx, topk_w);
  }
  __threadfence_block();
  __syncthreads();  // the ids written above are read back below by other lanes of this block
  permute_rank_body<true>(topk_idx, n_tokens * top_k, n_experts, key_bits, nullptr, expert_offsets, counts_out, perm,
                          inv_perm);
}

// Decode batches (T <= 8, bf16): router logits, routing and permutation in ONE block and one launch.
// The logits go to global memory (they are an output) and to LDS, from where the lane groups route.
template <int G, int VPL, int NF>
__global__ __launch_bounds__(PB_THREADS) void front_small_kernel(const bf16_t* __restrict__ x,
                                                                 const bf16_t* __restrict__ w_g, int hidden,
                                                                 float* __restrict__ logits, int n_tokens, int n_experts,
                                                                 int top_k, int key_bits, int32_t* topk_idx,
                                                                 float* __restrict__ topk_w,
                                                                 int32_t* __restrict__ expert_offsets,
                                                                 int32_t* __restrict__ counts_out,
                                                                 int32_t* __restrict__ perm,
                                                                 int32_t* __restrict__ inv_perm) {
  __shared__ float lds_logits[ROUTER_SMALL_T * HMOE_MAX_EXPERTS];
  router_logits_small<NF>(x, w_g, n_tokens, n_experts, hidden, logits, lds_logits);  // ends with a barrier
  constexpr int TOKENS_PER_PASS = PB_THREADS / G;
  for (int t0 = 0; t0 < n_tokens; t0 += TOKENS_PER_PASS) {
    const long token = t0 + threadIdx.x / G;
    route_token<G, VPL>(lds_logits, n_experts, top_k, token, token < n_tokens, threadIdx.x % G, topk_idx, topk_w);
  }
  __threadfence_block();
  __syncthreads();
  permute_rank_body<true>(topk_idx, n_tokens * top_k, n_experts, key_bits, nullptr, expert_offsets, counts_out, perm,
                          inv_perm);
}

// Larger bf16 batches: router logits and routing in one launch.  A block computes the logits of its tokens (global
// memory, they are an output, and LDS) and routes them from LDS, lane groups as in hmoe_route; the permutation,
// which needs every token's choice, stays a launch of its own.
template <int G, int VPL, int NF>
__global__ __launch_bounds__(PB_THREADS) void front_tokens_kernel(const bf16_t* __restrict__ x,
                                                                  const bf16_t* __restrict__ w_g, int hidden,
                                                                  float* __restrict__ logits, int n_tokens, int n_experts,
                                                                  int top_k, int tokens_per_block, int32_t* topk_idx,
                                                                  float* __restrict__ topk_w) {
  __shared__ float lds_logits[32 * NF * 32];
  router_logits_tokens<NF>(x, w_g, n_tokens, n_experts, hidden, logits, tokens_per_block, lds_logits);  // ends with a barrier
  constexpr int TOKENS_PER_PASS = PB_THREADS / G;
  const long t0 = (long)blockIdx.x * tokens_per_block;
  for (int l0 = 0; l0 < tokens_per_block; l0 += TOKENS_PER_PASS) {
    const int local = l0 + threadIdx.x / G;
    const bool valid = local < tokens_per_block && t0 + local < n_tokens;
    route_token<G, VPL>(lds_logits, n_experts, top_k, local, valid, threadIdx.x % G, topk_idx + t0 * top_k,
                        topk_w + t0 * top_k);
  }
}

// x_perm[p, :] = x[perm[p] / K, :], rows of row_bytes (multiple of 16)
__global__ __launch_bounds__(256) void gather_rows_kernel(const uint4* __restrict__ x, const int32_t* __restrict__ perm,
                                                          int top_k, int row_vec, int n_assign,
                                                          uint4* __restrict__ x_perm) {
  const int p = blockIdx.x;
  if (p >= n_assign) return;
  const long src = (long)(perm[p] / top_k) * row_vec, dst = (long)p * row_vec;
  for (int i = threadIdx.x; i < row_vec; i += blockDim.x) x_perm[dst + i] = x[src + i];
}

static inline int n_chunks(long n_assign) { return (int)((n_assign + PB_CHUNK - 1) / PB_CHUNK); }

}  // namespace hmoe

extern "C" size_t hmoe_permute_workspace_bytes(const hmoe_layer_desc* desc, int32_t T) {
  if (hmoe::check_desc(desc) != HMOE_OK || T < 0) return 0;
  const long A = (long)T * desc->top_k;
  // per-block counts + one row of counts for the pinned-host copy
  return ((size_t)hmoe::n_chunks(A) + 1) * desc->n_experts * sizeof(int32_t) + 256;
}

// hmoe_permute and hmoe_permute_static share this body; they differ in where the scratch memory comes from.
static int32_t permute_with_workspace(const hmoe_layer_desc* desc, const int32_t* topk_idx, int32_t T, const void* x,
                                      void* x_perm, int32_t* expert_offsets, int32_t* perm, int32_t* inv_perm,
                                      int32_t* h_counts_pinned, void* workspace, size_t workspace_bytes, void* stream) {
  using namespace hmoe;
  int rc = check_desc(desc);
  if (rc != HMOE_OK) return rc;
  if (T < 0 || !expert_offsets) return HMOE_ERR_INVALID_ARG;
  const long A = (long)T * desc->top_k;
  if (A > 0x7fffffffL - PB_CHUNK) return HMOE_ERR_UNSUPPORTED;
  if (A > 0 && (!topk_idx || !perm || !inv_perm)) return HMOE_ERR_INVALID_ARG;
  if ((x == nullptr) != (x_perm == nullptr)) return HMOE_ERR_INVALID_ARG;
  const size_t elem = desc->dtype == HMOE_F32 ? 4 : 2;
  const size_t row_bytes = (size_t)desc->hidden * elem;
  if (x && (row_bytes % 16 != 0)) return HMOE_ERR_UNSUPPORTED;
  if (x && (!aligned16(x) || !aligned16(x_perm))) return HMOE_ERR_INVALID_ARG;
  if (!workspace || workspace_bytes < hmoe_permute_workspace_bytes(desc, T)) return HMOE_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(workspace) & 3u) return HMOE_ERR_INVALID_ARG;
  hipStream_t s = (hipStream_t)stream;
  const int E = desc->n_experts;
  int key_bits = 0;
  while ((1 << key_bits) < E) ++key_bits;
  const int nblk = n_chunks(A);
  int32_t* block_counts = (int32_t*)workspace;
  int32_t* counts_dev = block_counts + (size_t)(nblk > 0 ? nblk : 0) * E;

  if (nblk <= 1) {
    hipLaunchKernelGGL((permute_rank_kernel<true>), dim3(1), dim3(PB_THREADS), 0, s, topk_idx, (int)A, E, key_bits,
                       (const int32_t*)nullptr, expert_offsets, counts_dev, perm, inv_perm);
  } else {
    hipLaunchKernelGGL(permute_hist_kernel, dim3(nblk), dim3(PB_THREADS), 0, s, topk_idx, (int)A, E, block_counts);
    hipLaunchKernelGGL(permute_scan_kernel, dim3(1), dim3(PB_THREADS), 0, s, block_counts, nblk, E, (int)A,
                       expert_offsets, counts_dev);
    hipLaunchKernelGGL((permute_rank_kernel<false>), dim3(nblk), dim3(PB_THREADS), 0, s, topk_idx, (int)A, E, key_bits,
                       (const int32_t*)block_counts, expert_offsets, (int32_t*)nullptr, perm, inv_perm);
  }
  HMOE_HIP(hipGetLastError());
  if (h_counts_pinned)
    HMOE_HIP(hipMemcpyAsync(h_counts_pinned, counts_dev, (size_t)E * sizeof(int32_t), hipMemcpyDeviceToHost, s));
  if (x && A > 0) {
    hipLaunchKernelGGL(gather_rows_kernel, dim3((unsigned)A), dim3(256), 0, s, (const uint4*)x, perm, desc->top_k,
                       (int)(row_bytes / 16), (int)A, (uint4*)x_perm);
    HMOE_HIP(hipGetLastError());
  }
  return HMOE_OK;
}

extern "C" int32_t hmoe_permute(const hmoe_layer_desc* desc, const int32_t* topk_idx, int32_t T, const void* x,
                                void* x_perm, int32_t* expert_offsets, int32_t* perm, int32_t* inv_perm,
                                int32_t* h_counts_pinned, void* workspace, size_t workspace_bytes, void* stream) {
  return permute_with_workspace(desc, topk_idx, T, x, x_perm, expert_offsets, perm, inv_perm, h_counts_pinned, workspace,
                                workspace_bytes, stream);
}

// ---- hmoe_permute without a workspace from the caller ------------------------------------------------------
// The per-block counts live in a file-scope device array instead.  In host code the array's name is only a
// stand-in: the address the kernels can use comes from hipGetSymbolAddress, once per device (each GPU holds its
// own copy of the array at its own address), and that pointer is what every launch and copy below is given.
static __device__ __align__(256) unsigned char scratch[HMOE_PERMUTE_STATIC_BYTES];

namespace hmoe {
constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices];  // device address of `scratch` per device, nullptr = not looked up yet
static std::mutex g_scratch_mutex;

// Device address of `scratch` on the current device (looked up on the first call on that device).
static int32_t static_scratch(void** out) {
  int dev = -1;
  HMOE_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return set_error_text(HMOE_ERR_UNSUPPORTED, "hmoe_permute_static: device index out of range");
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    HMOE_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (!ptr) return set_error_text(HMOE_ERR_HIP, "hmoe_permute_static: hipGetSymbolAddress returned a null address");
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return HMOE_OK;
}
}  // namespace hmoe

extern "C" int32_t hmoe_permute_static(const hmoe_layer_desc* desc, const int32_t* topk_idx, int32_t T, const void* x,
                                       void* x_perm, int32_t* expert_offsets, int32_t* perm, int32_t* inv_perm,
                                       int32_t* h_counts_pinned, void* stream) {
  using namespace hmoe;
  int rc = check_desc(desc);
  if (rc != HMOE_OK) return rc;
  if (T < 0) return HMOE_ERR_INVALID_ARG;
  const size_t need = hmoe_permute_workspace_bytes(desc, T);
  if (need == 0 || need > (size_t)HMOE_PERMUTE_STATIC_BYTES)
    return set_error_text(HMOE_ERR_WORKSPACE, "hmoe_permute_static: T * top_k assignments over n_experts experts need more than the "
                                              "library's static scratch array (HMOE_PERMUTE_STATIC_BYTES); use hmoe_permute");
  void* ws = nullptr;
  rc = static_scratch(&ws);
  if (rc != HMOE_OK) return rc;
  // Nothing in the scratch memory has to start at zero: the histogram kernel writes every per-block count before
  // the scan reads it, and the row of per-expert totals is written in full by the scan (or the one-block kernel).
  return permute_with_workspace(desc, topk_idx, T, x, x_perm, expert_offsets, perm, inv_perm, h_counts_pinned, ws,
                                (size_t)HMOE_PERMUTE_STATIC_BYTES, stream);
}

extern "C" int32_t hmoe_route_permute(const hmoe_layer_desc* desc, const float* logits, int32_t T, int32_t* topk_idx,
                                      float* topk_w, int32_t* expert_offsets, int32_t* perm, int32_t* inv_perm,
                                      int32_t* h_counts_pinned, void* workspace, size_t workspace_bytes, void* stream) {
  using namespace hmoe;
  int rc = check_desc(desc);
  if (rc != HMOE_OK) return rc;
  if (T < 0 || !expert_offsets) return HMOE_ERR_INVALID_ARG;
  const long A = (long)T * desc->top_k;
  if (A > PB_CHUNK || T > ROUTE_PERMUTE_SMALL_T || T == 0) {  // larger batches: the two separate calls
    rc = hmoe_route(desc, logits, T, topk_idx, topk_w, stream);
    if (rc != HMOE_OK) return rc;
    return hmoe_permute(desc, topk_idx, T, nullptr, nullptr, expert_offsets, perm, inv_perm, h_counts_pinned, workspace,
                        workspace_bytes, stream);
  }
  if (!logits || !topk_idx || !topk_w || !perm || !inv_perm) return HMOE_ERR_INVALID_ARG;
  if (!workspace || workspace_bytes < hmoe_permute_workspace_bytes(desc, T)) return HMOE_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(workspace) & 3u) return HMOE_ERR_INVALID_ARG;
  hipStream_t s = (hipStream_t)stream;
  const int E = desc->n_experts, K = desc->top_k;
  int key_bits = 0;
  while ((1 << key_bits) < E) ++key_bits;
  int32_t* counts_dev = (int32_t*)workspace + (size_t)n_chunks(A) * E;
#define HMOE_LAUNCH_SMALL(G, VPL)                                                                                   \
  hipLaunchKernelGGL((route_permute_small_kernel<G, VPL>), dim3(1), dim3(PB_THREADS), 0, s, logits, (int)T, E, K, key_bits, \
                     topk_idx, topk_w, expert_offsets, counts_dev, perm, inv_perm)
  if (E <= 8) HMOE_LAUNCH_SMALL(8, 1);
  else if (E <= 16) HMOE_LAUNCH_SMALL(16, 1);
  else if (E <= 32) HMOE_LAUNCH_SMALL(32, 1);
  else if (E <= 64) HMOE_LAUNCH_SMALL(64, 1);
  else if (E <= 128) HMOE_LAUNCH_SMALL(64, 2);
  else HMOE_LAUNCH_SMALL(64, 4);
#undef HMOE_LAUNCH_SMALL
  HMOE_HIP(hipGetLastError());
  if (h_counts_pinned)
    HMOE_HIP(hipMemcpyAsync(h_counts_pinned, counts_dev, (size_t)E * sizeof(int32_t), hipMemcpyDeviceToHost, s));
  return HMOE_OK;
}

extern "C" int32_t hmoe_router_route_permute(const hmoe_layer_desc* desc, const void* x, const void* w_g, int32_t T,
                                             float* logits, int32_t* topk_idx, float* topk_w, int32_t* expert_offsets,
                                             int32_t* perm, int32_t* inv_perm, int32_t* h_counts_pinned, void* workspace,
                                             size_t workspace_bytes, void* stream) {
  using namespace hmoe;
  int rc = check_desc(desc);
  if (rc != HMOE_OK) return rc;
  if (T < 0 || !expert_offsets) return HMOE_ERR_INVALID_ARG;
  const long A = (long)T * desc->top_k;
  if (T > ROUTER_SMALL_T && T <= 2048 && desc->dtype != HMOE_F32 && desc->hidden % 16 == 0 && x && w_g && logits &&
      topk_idx && topk_w && aligned16(x) && aligned16(w_g)) {
    // logits and routing in one launch, then the permutation (a launch saved; beyond a few thousand tokens the
    // separate routing kernel, with a block per few tokens, is the faster one)
    const int E = desc->n_experts, K = desc->top_k;
    int tpb = 32;  // tokens per block: fewer while the grid would leave more than half of the CUs without a block
    while (tpb > 4 && (T + tpb - 1) / tpb < 128) tpb /= 2;
    const dim3 grid((unsigned)((T + tpb - 1) / tpb));
#define HMOE_LAUNCH_FRONT_TOKENS(G, VPL, NF)                                                                        \
  hipLaunchKernelGGL((front_tokens_kernel<G, VPL, NF>), grid, dim3(PB_THREADS), 0, (hipStream_t)stream,             \
                     (const bf16_t*)x, (const bf16_t*)w_g, desc->hidden, logits, (int)T, E, K, tpb, topk_idx, topk_w)
    if (E <= 8) HMOE_LAUNCH_FRONT_TOKENS(8, 1, 1);
    else if (E <= 16) HMOE_LAUNCH_FRONT_TOKENS(16, 1, 1);
    else if (E <= 32) HMOE_LAUNCH_FRONT_TOKENS(32, 1, 1);
    else if (E <= 64) HMOE_LAUNCH_FRONT_TOKENS(64, 1, 2);
    else if (E <= 128) HMOE_LAUNCH_FRONT_TOKENS(64, 2, 4);
    else HMOE_LAUNCH_FRONT_TOKENS(64, 4, 8);
#undef HMOE_LAUNCH_FRONT_TOKENS
    HMOE_HIP(hipGetLastError());
    return hmoe_permute(desc, topk_idx, T, nullptr, nullptr, expert_offsets, perm, inv_perm, h_counts_pinned, workspace,
                        workspace_bytes, stream);
  }
  if (T == 0 || T > ROUTER_SMALL_T || A > PB_CHUNK || desc->dtype == HMOE_F32) {  // the separate calls
    rc = hmoe_router_logits(desc, x, w_g, T, logits, stream);
    if (rc != HMOE_OK) return rc;
    return hmoe_route_permute(desc, logits, T, topk_idx, topk_w, expert_offsets, perm, inv_perm, h_counts_pinned,
                              workspace, workspace_bytes, stream);
  }
  if (!x || !w_g || !logits || !topk_idx || !topk_w || !perm || !inv_perm) return HMOE_ERR_INVALID_ARG;
  if (desc->hidden % 16 != 0) return HMOE_ERR_UNSUPPORTED;
  if (!aligned16(x) || !aligned16(w_g)) return HMOE_ERR_INVALID_ARG;
  if (!workspace || workspace_bytes < hmoe_permute_workspace_bytes(desc, T)) return HMOE_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(workspace) & 3u) return HMOE_ERR_INVALID_ARG;
  hipStream_t s = (hipStream_t)stream;
  const int E = desc->n_experts, K = desc->top_k;
  int key_bits = 0;
  while ((1 << key_bits) < E) ++key_bits;
  int32_t* counts_dev = (int32_t*)workspace + (size_t)n_chunks(A) * E;
#define HMOE_LAUNCH_FRONT(G, VPL, NF)                                                                              \
  hipLaunchKernelGGL((front_small_kernel<G, VPL, NF>), dim3(1), dim3(PB_THREADS), 0, s, (const bf16_t*)x,          \
                     (const bf16_t*)w_g, desc->hidden, logits, (int)T, E, K, key_bits, topk_idx, topk_w, expert_offsets, \
                     counts_dev, perm, inv_perm)
  if (E <= 8) HMOE_LAUNCH_FRONT(8, 1, 1);
  else if (E <= 16) HMOE_LAUNCH_FRONT(16, 1, 1);
  else if (E <= 32) HMOE_LAUNCH_FRONT(32, 1, 1);
  else if (E <= 64) HMOE_LAUNCH_FRONT(64, 1, 2);
  else if (E <= 128) HMOE_LAUNCH_FRONT(64, 2, 4);
  else HMOE_LAUNCH_FRONT(64, 4, 8);
#undef HMOE_LAUNCH_FRONT
  HMOE_HIP(hipGetLastError());
  if (h_counts_pinned)
    HMOE_HIP(hipMemcpyAsync(h_counts_pinned, counts_dev, (size_t)E * sizeof(int32_t), hipMemcpyDeviceToHost, s));
  return HMOE_OK;
}
