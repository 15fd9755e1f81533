/*
 * hmoe.h -- C ABI of the MI355X (gfx950) MoE-layer forward over an HBM expert cache.
 *
 * The library evaluates the MoE layer of HybriMoE, Section II-A, Eq. (1)
 *
 *     y = sum_{i<N} Softmax(TopK(x . W_g))_i * E_i(x)          (N experts, K activated)
 *
 * plus the always-on shared experts of Section II-A, over experts that are resident in a
 * fixed number of GPU cache slots (the GPU expert cache of Sections I, IV-D and V), with
 * missing experts copied on demand from host memory (Section I, "on demand" loading over
 * PCIe).  One call per step:
 *
 *     hmoe_router_logits   x . W_g                       (helper)
 *     hmoe_route           Softmax(TopK(.))
 *     hmoe_permute         token-to-expert permutation (+ row gather)
 *     hmoe_cache_stage     make an expert resident in a slot
 *     hmoe_expert_ffn_grouped   E_i(.) for every expert with rows, from its slot
 *     hmoe_combine         the gate-weighted sum of Eq. (1) (+ shared experts)
 *
 * Conventions
 *   - Plain C.  Every call returns an int32 status (HMOE_OK = 0, negative = error), never
 *     throws and never allocates or frees device memory: the caller owns every buffer.
 *     The only library-owned objects are the small host-side hmoe_cache and its HIP events.
 *   - Pointers are DEVICE pointers unless the name starts with h_ (HOST).  Tensors are
 *     row-major with the innermost dimension contiguous and must be 16-byte aligned;
 *     slot storage must be 256-byte aligned.
 *   - `stream` arguments are hipStream_t passed as void* (NULL = the default stream).  All
 *     device work is enqueued on that stream; no call synchronises the device unless it
 *     says so.
 *   - T = tokens, H = hidden, F = expert FFN dim, E = routed experts, K = top_k,
 *     A = T*K assignments, S = cache slots.
 *   - dtype HMOE_BF16: activations/weights are bfloat16, accumulation fp32 (MFMA), the
 *     intermediate h = silu(g)*u and the per-assignment outputs are rounded to bf16.
 *     dtype HMOE_F32: everything fp32.
 *   - Errors detectable on the host are reported before anything is enqueued:
 *     NULL / negative / K > E / S > E / misaligned -> HMOE_ERR_INVALID_ARG; a shape or dtype
 *     the kernels are not built for -> HMOE_ERR_UNSUPPORTED; workspace too small ->
 *     HMOE_ERR_WORKSPACE; a failing HIP call -> HMOE_ERR_HIP (text via hmoe_last_error).
 */
#ifndef HMOE_H
#define HMOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  HMOE_OK = 0,
  HMOE_ERR_INVALID_ARG = -1,
  HMOE_ERR_UNSUPPORTED = -2,
  HMOE_ERR_WORKSPACE = -3,
  HMOE_ERR_NOT_RESIDENT = -4,
  HMOE_ERR_SLOT_BUSY = -5,
  HMOE_ERR_HIP = -6
};

enum { HMOE_F32 = 0, HMOE_BF16 = 1, HMOE_BF16_W4 = 2 };

/*
 * HMOE_BF16_W4: activations bfloat16 as for HMOE_BF16, expert weights stored in 4 bits (the paper runs
 * its experts in 4 bits, Section V, without defining a format; this one is group-wise symmetric):
 * a matrix W [N, K] is cut along K into groups of 128; scale of (row, group) s = bf16(max|W| / 7), the
 * maximum and the division in fp32; code q = clamp(rint(W / s), -8, 7) + 8 in fp32 (nearest even), a
 * group of zeros has s = 0 and codes 8; the value used in the FFN is (q - 8) * s.  hmoe_pack_expert
 * quantises bfloat16 weights into this format (4.125 bits per weight in the slot).  Needs
 * H % 128 == 0 and F % 128 == 0.  FFN paths: HMOE_FFN_SKINNY (AUTO up to 64 tokens), HMOE_FFN_TILED
 * (AUTO above) and HMOE_FFN_REFERENCE.  Everything else (router, route, permute, combine) behaves as for
 * HMOE_BF16.
 */

/* Which FFN kernels hmoe_expert_ffn_grouped uses.  AUTO picks by token count. */
enum {
  HMOE_FFN_AUTO = 0,
  HMOE_FFN_REFERENCE = 1, /* one wave per output element; any shape; fp32 and bf16          */
  HMOE_FFN_SKINNY = 2,    /* decode: weight-streaming MFMA GEMV, <= 32 rows per expert pass */
  HMOE_FFN_TILED = 3      /* prefill: LDS-tiled grouped MFMA GEMM                           */
};

/* Limits of this build. */
#define HMOE_MAX_EXPERTS 256
#define HMOE_MAX_TOP_K 32

/* Shape of one MoE layer (Table II of the paper lists such shapes per model). */
typedef struct hmoe_layer_desc {
  int32_t hidden;    /* H                                          */
  int32_t ffn;       /* F                                          */
  int32_t n_experts; /* E, 1..HMOE_MAX_EXPERTS                     */
  int32_t top_k;     /* K, 1..min(E, HMOE_MAX_TOP_K)               */
  int32_t n_slots;   /* S, 1..E                                    */
  int32_t dtype;     /* HMOE_F32, HMOE_BF16 or HMOE_BF16_W4        */
} hmoe_layer_desc;

/* Host-side cache object: slot table mirror, use ticks, events.  Opaque. */
typedef struct hmoe_cache hmoe_cache;

const char* hmoe_status_string(int32_t status);
/* Text of the last failing HIP call on this thread ("" if none). */
const char* hmoe_last_error(void);

/* ------------------------------------------------------------------------------------
 * Router logits, the x . W_g of Eq. (1).
 *   x      [T, H]  layer dtype
 *   w_g    [E, H]  layer dtype (row e is expert e's router vector)
 *   logits [T, E]  fp32 out; fp32 accumulation.
 * T = 0 is a no-op.  bf16 needs H % 16 == 0.
 */
int32_t hmoe_router_logits(const hmoe_layer_desc* desc, const void* x, const void* w_g, int32_t T,
                           float* logits, void* stream);

/* ------------------------------------------------------------------------------------
 * Softmax(TopK(.)) of Eq. (1).
 *   logits   [T, E] fp32, finite (NaN/inf: result unspecified, memory-safe)
 *   topk_idx [T, K] int32 out: the K largest logits' expert ids, by descending logit;
 *                              equal logits (+0 == -0) -> lower expert id first
 *   topk_w   [T, K] fp32 out: softmax over the K kept logits (sums to 1 per token)
 */
int32_t hmoe_route(const hmoe_layer_desc* desc, const float* logits, int32_t T, int32_t* topk_idx,
                   float* topk_w, void* stream);

/* ------------------------------------------------------------------------------------
 * Token-to-expert permutation: stable counting sort of the A = T*K flat assignments
 * a = t*K + j by expert id topk_idx[a] (per-expert load is what the paper's scheduler and
 * cache consume, Section IV-B; here it is expert_offsets).
 *   expert_offsets [E+1] int32 out: rows of expert e are [offsets[e], offsets[e+1])
 *   perm           [A]   int32 out: perm[p] = a (sorted position -> assignment)
 *   inv_perm       [A]   int32 out: inv_perm[a] = p
 *   x [T, H] / x_perm [A, H] (layer dtype): when both non-NULL, x_perm[p] = x[perm[p] / K]
 *   h_counts_pinned [E] int32, HOST pinned memory or NULL: when given, the per-expert row
 *       counts are also copied there asynchronously on `stream` (valid after the stream or
 *       an event recorded after this call has completed).
 *   workspace: hmoe_permute_workspace_bytes(desc, T) bytes of device scratch.
 * Expert ids outside [0, E) are a precondition violation (memory-safe: such assignments
 * are clamped to expert E-1).
 */
size_t hmoe_permute_workspace_bytes(const hmoe_layer_desc* desc, int32_t T);
int32_t hmoe_permute(const hmoe_layer_desc* desc, const int32_t* topk_idx, int32_t T, const void* x,
                     void* x_perm, int32_t* expert_offsets, int32_t* perm, int32_t* inv_perm,
                     int32_t* h_counts_pinned, void* workspace, size_t workspace_bytes, void* stream);

/*
 * hmoe_permute for callers that cannot allocate device memory and therefore have no workspace to hand over:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and the
 * same results, bit for bit, but the scratch memory (per-block expert counts) is a static device array of
 * HMOE_PERMUTE_STATIC_BYTES inside the library, which every GPU the library runs on holds until the process
 * ends.  The call allocates and frees nothing (its first call on a device looks the array's address up).
 *   Limit: hmoe_permute_workspace_bytes(desc, T) <= HMOE_PERMUTE_STATIC_BYTES, i.e. about
 *   (T * K / 1024 + 2) * E * 4 bytes; beyond it -> HMOE_ERR_WORKSPACE (text via hmoe_last_error), nothing enqueued.
 *   All calls on one GPU share the one array, which keeps the previous call's contents (nothing in it needs to
 *   start at zero): calls that may run at the same time on one GPU -- different streams without an ordering
 *   between them -- race and must use hmoe_permute with workspaces of their own.  The current device must be
 *   the device of `stream`.
 */
#define HMOE_PERMUTE_STATIC_BYTES (1 << 20)
int32_t hmoe_permute_static(const hmoe_layer_desc* desc, const int32_t* topk_idx, int32_t T, const void* x,
                            void* x_perm, int32_t* expert_offsets, int32_t* perm, int32_t* inv_perm,
                            int32_t* h_counts_pinned, void* stream);

/*
 * hmoe_route followed by hmoe_permute (without the row gather; see hmoe_expert_ffn_grouped_gather)
 * as one call.  For small batches (T <= 64 and T*K <= 1024: every decode shape) both run in a single
 * one-block launch; larger batches run the two calls above.  Arguments and results as in those calls.
 */
int32_t hmoe_route_permute(const hmoe_layer_desc* desc, const float* logits, int32_t T, int32_t* topk_idx,
                           float* topk_w, int32_t* expert_offsets, int32_t* perm, int32_t* inv_perm,
                           int32_t* h_counts_pinned, void* workspace, size_t workspace_bytes, void* stream);

/*
 * hmoe_router_logits followed by hmoe_route_permute as one call: the whole front end of Eq. (1)
 * (x . W_g, Softmax(TopK(.)), permutation).  For decode batches (bf16, T <= 8) it is a single
 * one-block launch; bf16 batches of up to 2048 tokens compute the logits and route in one launch and
 * permute in a second; anything else runs the two calls above.  `logits` [T, E] is an output (the same bits
 * hmoe_router_logits writes); the other arguments and results as in those calls.
 */
int32_t hmoe_router_route_permute(const hmoe_layer_desc* desc, const void* x, const void* w_g, int32_t T,
                                  float* logits, int32_t* topk_idx, float* topk_w, int32_t* expert_offsets,
                                  int32_t* perm, int32_t* inv_perm, int32_t* h_counts_pinned, void* workspace,
                                  size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------------------
 * Expert weights.  An expert is three bias-free matrices (SwiGLU; the paper gives only
 * the sizes, Table II): W_gate [F, H], W_up [F, H], W_down [H, F], row-major.
 * hmoe_pack_expert rewrites them (HOST to HOST) into the library-private slot layout of
 * hmoe_slot_bytes(desc) bytes; that blob is what lives in pinned host memory and in the
 * HBM slots.  bf16 needs H % 64 == 0 and F % 64 == 0 (MFMA tile packing); fp32 takes any.
 */
size_t hmoe_slot_bytes(const hmoe_layer_desc* desc);
int32_t hmoe_pack_expert(const hmoe_layer_desc* desc, const void* h_w_gate, const void* h_w_up,
                         const void* h_w_down, void* h_packed_out);

/* ------------------------------------------------------------------------------------
 * GPU expert cache: S slots of hmoe_slot_bytes each in `slot_storage` (device, 256-byte
 * aligned, S * slot_bytes) and the device table d_slot_of [E] int32 (expert -> slot,
 * -1 = not resident) that the FFN kernels read.  hmoe_cache_create fills d_slot_of with -1
 * (synchronously) and keeps a host mirror.  The cache must be used with ONE compute stream.
 */
int32_t hmoe_cache_create(const hmoe_layer_desc* desc, void* slot_storage, int32_t* d_slot_of,
                          hmoe_cache** out);
int32_t hmoe_cache_destroy(hmoe_cache* cache);
/* Host mirror: slot of an expert (-1 = not resident), expert in a slot (-1 = free). */
int32_t hmoe_cache_lookup(const hmoe_cache* cache, int32_t expert_id, int32_t* slot_out);
int32_t hmoe_cache_occupant(const hmoe_cache* cache, int32_t slot, int32_t* expert_out);
/* Drop an expert (no-op if not resident); the table changes in compute-stream order. */
int32_t hmoe_cache_evict(hmoe_cache* cache, int32_t expert_id, void* compute_stream);
/* Protect a slot from hmoe_cache_stage (pinned != 0) or release it. */
int32_t hmoe_cache_pin_slot(hmoe_cache* cache, int32_t slot, int32_t pinned);

/*
 * Make expert_id resident in `slot` (-1 = lowest-numbered free slot; none free ->
 * HMOE_ERR_SLOT_BUSY) from its packed blob in PINNED HOST memory (on-demand expert load,
 * Section I).  Enqueues, without blocking the host:
 *   copy_stream:    wait until the last FFN call that read this slot has finished,
 *                   hipMemcpyAsync host -> slot, record "ready"
 *   compute_stream: wait "ready", then update d_slot_of (new expert -> slot, previous
 *                   occupant -> -1)
 * so FFN calls enqueued on compute_stream afterwards see the new expert, and FFN calls
 * enqueued before are not disturbed; the copy overlaps whatever compute does not touch
 * the slot.  The previous occupant, if any, is evicted.  A pinned slot -> HMOE_ERR_SLOT_BUSY.
 * If the expert is already resident elsewhere it is first dropped from that slot.
 * h_packed_pinned must stay valid until the copy has completed.
 * h_packed_pinned == NULL marks the slot's current device contents as expert_id without
 * copying (for weights written into slot storage by the caller).
 * HIP graphs: hmoe_cache_stage itself must not be called on a capturing stream.  Once an FFN call over this cache
 * has been captured, the library cannot know when a replay reads a slot; every later copy into a slot therefore
 * waits for all work enqueued on compute_stream so far (replays included) instead of for the slot's last reader.
 */
int32_t hmoe_cache_stage(hmoe_cache* cache, int32_t expert_id, int32_t slot,
                         const void* h_packed_pinned, void* compute_stream, void* copy_stream);

/*
 * Host-only LRU planning for one call (LRU is the replacement policy the paper compares
 * against, Section IV-D).  h_counts [E]: rows per expert for this call (needed = count > 0).
 * Outputs, each [E]: h_wave[e] = wave in which e is computed (-1 = not needed; 0 = already
 * resident), h_slot[e] = slot e is computed from (-1 = not needed), h_victim[e] = expert it
 * replaces (-1 none).
 * *n_waves = 1 + the largest wave.  Rules: misses in ascending id; lowest free slot, else the
 * slot whose occupant has the oldest use tick (ties -> lowest slot); a miss that replaces an
 * expert needed by this call runs one wave after it.  Updates the use ticks and the clock;
 * the slot table itself changes only through hmoe_cache_stage.
 */
int32_t hmoe_cache_plan(hmoe_cache* cache, const int32_t* h_counts, int32_t* h_wave, int32_t* h_slot,
                        int32_t* h_victim, int32_t* n_waves);

/*
 * Shared experts (Section II-A) run as a dense FFN of their own, usually next to the routed experts' FFN on a second
 * stream.  hmoe_cache_set_layer tells the cache of such an FFN (one expert, one slot) which routed layer it belongs to
 * (`routed`: same hidden size and dtype; copied; NULL forgets it): prefill launches over that cache then choose their
 * kernels as the routed launches of a batch of the same tokens do, so that the two share the CUs well.  Host only;
 * results do not depend on it.  HMOE_ERR_INVALID_ARG for a cache of more than one expert or a layer that does not
 * match.
 */
int32_t hmoe_cache_set_layer(hmoe_cache* cache, const hmoe_layer_desc* routed);

/*
 * Score-aware replacement (Section IV-D, Eq. (3)): the Minus Recent Score policy keeps a priority
 * estimate S per expert, S <- alpha * TopP(s) + (1 - alpha) * S, where s are the routing scores of the
 * current iteration and only the p largest are accumulated (the paper uses p = 2K); the victim is the
 * candidate with the lowest S.  Where the paper is silent: S starts at 0; s is the batch mean of the
 * full softmax over all E experts (hmoe_route_scores); TopP keeps the p largest entries (ties: lower
 * id) and zeroes the rest; candidates are ordered as for LRU (experts this call does not need first,
 * then by wave), S replacing the use tick inside a class, ties -> lowest slot.
 *   hmoe_cache_set_policy    HMOE_POLICY_LRU (default) or HMOE_POLICY_MRS with 0 < alpha <= 1
 *   hmoe_cache_update_scores one update of Eq. (3) from HOST scores h_scores [E]; call once per
 *                            iteration, after the layer call
 *   hmoe_cache_get_scores    copies S [E] (double) to the host
 */
enum { HMOE_POLICY_LRU = 0, HMOE_POLICY_MRS = 1 };
int32_t hmoe_cache_set_policy(hmoe_cache* cache, int32_t policy, float alpha);
int32_t hmoe_cache_update_scores(hmoe_cache* cache, const float* h_scores, int32_t top_p);
int32_t hmoe_cache_get_scores(const hmoe_cache* cache, double* h_out);

/*
 * Routing scores of one iteration for Eq. (3): scores[e] = mean over the T tokens of
 * softmax(logits[t, :])[e] (full softmax over all E experts), fp32, summed in a fixed order.
 *   scores [E] device fp32 out; h_scores_pinned [E] HOST pinned or NULL (async copy on `stream`)
 *   workspace: hmoe_route_scores_workspace_bytes(desc, T) bytes of device scratch.
 */
size_t hmoe_route_scores_workspace_bytes(const hmoe_layer_desc* desc, int32_t T);
int32_t hmoe_route_scores(const hmoe_layer_desc* desc, const float* logits, int32_t T, float* scores,
                          float* h_scores_pinned, void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------------------
 * Grouped SwiGLU expert FFN over resident experts: for every expert e that is active,
 * has rows and sits in a slot,
 *     rows = x_perm[offsets[e] : offsets[e+1]]
 *     o_perm[rows] = (silu(rows . W_gate^T) * (rows . W_up^T)) . W_down^T
 *   x_perm [A, H], o_perm [A, H] layer dtype; expert_offsets [E+1] device int32
 *   h_active (HOST) / n_active: the experts of this call ("wave"); NULL = every resident
 *       expert.  An expert named here that is not resident (host mirror) ->
 *       HMOE_ERR_NOT_RESIDENT, nothing enqueued.  Rows of experts that are not active or not
 *       resident are left untouched.
 *   workspace: hmoe_ffn_workspace_bytes(desc, A) bytes of device scratch (holds h [A, F]).
 *   path: HMOE_FFN_*; AUTO = SKINNY when T = A/K <= 32 (4-bit weights: 64) else TILED, REFERENCE for fp32.
 * Shared experts (Section II-A) use the same call with a 1-expert layer (E = K = S = 1,
 * offsets {0, T}).
 */
size_t hmoe_ffn_workspace_bytes(const hmoe_layer_desc* desc, int32_t A);
int32_t hmoe_expert_ffn_grouped(const hmoe_layer_desc* desc, hmoe_cache* cache, const void* x_perm,
                                const int32_t* expert_offsets, int32_t A, const int32_t* h_active,
                                int32_t n_active, void* o_perm, void* workspace, size_t workspace_bytes,
                                int32_t path, void* stream);

/*
 * Same FFN with the row gather of hmoe_permute fused into its first GEMM: sorted row p of the
 * input is x[perm[p] / K] (x [T, H] un-permuted, perm [A] as written by hmoe_permute), so x_perm
 * need not be materialised.  Everything else as hmoe_expert_ffn_grouped.
 */
int32_t hmoe_expert_ffn_grouped_gather(const hmoe_layer_desc* desc, hmoe_cache* cache, const void* x,
                                       const int32_t* perm, const int32_t* expert_offsets, int32_t A,
                                       const int32_t* h_active, int32_t n_active, void* o_perm,
                                       void* workspace, size_t workspace_bytes, int32_t path, void* stream);

/*
 * hmoe_expert_ffn_grouped_gather for the routed experts and, on the same stream, the dense FFN of the
 * layer's shared experts (Section II-A: they see every token) over the same un-permuted x:
 *     o_perm   as hmoe_expert_ffn_grouped_gather(desc, cache, x, perm, expert_offsets, A, ...)
 *     o_shared as hmoe_expert_ffn_grouped(shared_desc, shared_cache, x, shared_offsets, T, NULL, 0, ...)
 * with the same bits as those two calls.  shared_desc is a 1-expert layer (E = K = S = 1) of the same
 * hidden size and dtype whose expert is resident in shared_cache; shared_offsets is the device array
 * {0, T}; o_shared [T, H]; shared_workspace holds hmoe_ffn_workspace_bytes(shared_desc, T) bytes.
 * When both parts are decode-sized bf16 calls (path resolves to HMOE_FFN_SKINNY for both), the shared
 * FFN is computed by extra blocks of the routed experts' two launches instead of two launches of its own,
 * which is what a layer of a few microseconds per kernel needs; in every other case the two calls run
 * one after the other.  Errors as in the two calls; nothing is enqueued when an argument is rejected.
 */
int32_t hmoe_expert_ffn_grouped_with_shared(
    const hmoe_layer_desc* desc, hmoe_cache* cache, const void* x, const int32_t* perm, const int32_t* expert_offsets,
    int32_t A, const int32_t* h_active, int32_t n_active, void* o_perm, void* workspace, size_t workspace_bytes,
    const hmoe_layer_desc* shared_desc, hmoe_cache* shared_cache, const int32_t* shared_offsets, int32_t T,
    void* o_shared, void* shared_workspace, size_t shared_workspace_bytes, int32_t path, void* stream);

/* ------------------------------------------------------------------------------------
 * The sum of Eq. (1) in gather form:
 *     y[t] = sum_{j<K} topk_w[t, j] * o_perm[inv_perm[t*K + j]]  (+ o_shared[t])
 * j in ascending order, then the shared term; fp32 accumulation, one rounding.
 *   o_perm [A, H], o_shared [T, H] or NULL, y [T, H]: layer dtype.
 */
int32_t hmoe_combine(const hmoe_layer_desc* desc, const void* o_perm, const int32_t* inv_perm,
                     const float* topk_w, const void* o_shared, int32_t T, void* y, void* stream);

/* ------------------------------------------------------------------------------------
 * Grouped expert FFN over a cache that holds fewer experts than the call needs (on-demand loading of the missing
 * experts over PCIe, Section I; transfer and compute overlapped on two streams, Section V): one call plans the
 * replacement (hmoe_cache_plan on h_counts_pinned), and then, wave by wave, stages the wave's missing experts
 * (hmoe_cache_stage from h_packed_pinned[e], on copy_stream) and runs the FFN of the wave's experts
 * (hmoe_expert_ffn_grouped_gather when perm is given, else hmoe_expert_ffn_grouped with x as x_perm) on
 * compute_stream.  A copy waits only for the last FFN call that read its slot, so the copies of wave w + 1 run under
 * the FFN of wave w wherever they do not replace an expert that wave computes.
 *   h_counts_pinned [E] HOST: per-expert rows as delivered by hmoe_permute / hmoe_route_permute on compute_stream;
 *       the call SYNCHRONISES compute_stream once before it reads them.
 *   h_packed_pinned [E] HOST array of HOST pointers: expert e's packed blob in pinned memory (may be NULL for
 *       experts that never have to be staged; a missing expert without a blob -> HMOE_ERR_INVALID_ARG).
 *   h_wave, h_slot, h_victim [E], n_waves: the plan, as written by hmoe_cache_plan.  staged_bytes (or NULL): bytes copied.
 * Other arguments, results and errors as in the calls named above.
 */
int32_t hmoe_expert_ffn_staged(const hmoe_layer_desc* desc, hmoe_cache* cache, const void* x, const int32_t* perm,
                               const int32_t* expert_offsets, int32_t A, const int32_t* h_counts_pinned,
                               const void* const* h_packed_pinned, void* o_perm, void* workspace, size_t workspace_bytes,
                               int32_t path, void* compute_stream, void* copy_stream, int32_t* h_wave, int32_t* h_slot,
                               int32_t* h_victim, int32_t* n_waves, uint64_t* staged_bytes);

/* ------------------------------------------------------------------------------------
 * Expert FFN and the sum of Eq. (1) as one call, for layers whose kernels take a few microseconds each:
 *     hmoe_expert_ffn_grouped_with_shared(desc, cache, x, perm, expert_offsets, T * K, NULL, 0, o_perm, ...,
 *                                         shared_desc, shared_cache, shared_offsets, T, o_shared, ...)
 *       (hmoe_expert_ffn_grouped_gather when shared_desc is NULL: a layer without shared experts)
 *     hmoe_combine(desc, o_perm, inv_perm, topk_w, o_shared, T, y)
 * with the same bits in o_perm, o_shared and y as those calls.  When the FFN runs as the decode kernel pair (bf16,
 * path resolves to HMOE_FFN_SKINNY for both parts) and every routed expert is resident, the sum is computed inside
 * the down projection's launch: a block that has stored its piece of o_perm / o_shared draws a ticket from the
 * counter of its column block in `sync`, and the block that draws the last ticket adds up those columns for every
 * token, in the order of hmoe_combine.  No block waits for another, and the result does not depend on which block is
 * last.  Otherwise the calls above run one after the other.
 *   sync: hmoe_ffn_combine_sync_bytes(desc) bytes of device memory that the CALLER ZEROES ONCE (before the first call
 *         that uses it); every call leaves it zero.  Calls that may run at the same time need buffers of their own.
 * Errors as in the calls above; nothing is enqueued when an argument is rejected.
 */
size_t hmoe_ffn_combine_sync_bytes(const hmoe_layer_desc* desc);
int32_t hmoe_expert_ffn_combine(
    const hmoe_layer_desc* desc, hmoe_cache* cache, const void* x, const int32_t* perm, const int32_t* inv_perm,
    const float* topk_w, const int32_t* expert_offsets, int32_t T, void* o_perm, void* workspace, size_t workspace_bytes,
    const hmoe_layer_desc* shared_desc, hmoe_cache* shared_cache, const int32_t* shared_offsets, void* o_shared,
    void* shared_workspace, size_t shared_workspace_bytes, void* y, void* sync, size_t sync_bytes, int32_t path, void* stream);

/* ------------------------------------------------------------------------------------
 * Hybrid CPU-GPU scheduling simulation (Section IV-B).  HOST ONLY: no device work, no stream.
 * The activated experts of a layer (load > 0) are placed on three timelines -- CPU compute, GPU
 * compute, host-to-GPU transfer -- by the paper's priority rules: the GPU takes experts whose weights
 * are on the GPU, highest load first; the CPU takes uncached experts, lowest load first, and with none
 * left the lowest-load cached expert; the link moves uncached experts, highest load first, and a moved
 * expert joins the GPU's list when it has arrived.  Whichever timeline is free first acts next (ties:
 * CPU, GPU, link; equal loads: lower id).  Cost model: an expert with L rows takes
 * gpu_base + gpu_per_token * L on the GPU, cpu_base + cpu_per_token * L on the CPU; a transfer takes
 * `transfer`; all in one unit of the caller's choice, >= 0.
 *   h_load [n] rows per expert (hmoe_permute's h_counts_pinned); h_cached [n] nonzero = weights in a slot
 *   h_device [n] out: HMOE_ON_* or -1 (not activated); h_start / h_end [n] out: compute interval (-1 if
 *   not activated); h_transfer_start [n] out: -1 if not transferred; *makespan out.
 * hmoe_schedule_simulate runs one rule set (`rules`: which of the three optional operations exist);
 * HMOE_ERR_UNSUPPORTED if the rules leave an activated expert that nothing may compute.
 * hmoe_schedule_plan simulates four rule sets -- all rules; without the CPU taking cached experts; the two
 * fixed mappings the paper compares against (uncached experts on the CPU, no transfers; no CPU, every
 * uncached expert loaded) -- and returns the first with the smallest makespan (*rules_out, may be NULL).
 */
typedef struct hmoe_sched_cost {
  double gpu_base, gpu_per_token, cpu_base, cpu_per_token, transfer;
} hmoe_sched_cost;
enum { HMOE_ON_GPU_CACHED = 0, HMOE_ON_GPU_LOADED = 1, HMOE_ON_CPU = 2 };
enum { HMOE_SCHED_CPU_UNCACHED = 1, HMOE_SCHED_CPU_CACHED = 2, HMOE_SCHED_TRANSFERS = 4, HMOE_SCHED_ALL = 7 };
int32_t hmoe_schedule_simulate(int32_t n_experts, const int32_t* h_load, const int32_t* h_cached,
                               const hmoe_sched_cost* cost, int32_t rules, int32_t* h_device, double* h_start,
                               double* h_end, double* h_transfer_start, double* makespan);
int32_t hmoe_schedule_plan(int32_t n_experts, const int32_t* h_load, const int32_t* h_cached,
                           const hmoe_sched_cost* cost, int32_t* h_device, double* h_start, double* h_end,
                           double* h_transfer_start, double* makespan, int32_t* rules_out);

/* ------------------------------------------------------------------------------------
 * Timing probe for benchmarks: while armed, every grouped-FFN call brackets each of its two
 * kernel launches with a pair of HIP events on the call's stream: first the gate/up launch
 * (h = silu(x W_gate^T) * (x W_up^T)), then the down projection, so a call records two pairs.
 * hmoe_probe_arm(max_pairs) creates the events; hmoe_probe_read synchronises them and
 * writes the elapsed milliseconds of each recorded pair to h_ms (up to max), returns the
 * count in *n, and disarms.  Not for use under stream capture.
 */
int32_t hmoe_probe_arm(int32_t max_pairs);
int32_t hmoe_probe_read(float* h_ms, int32_t max, int32_t* n);

#ifdef __cplusplus
}
#endif
#endif /* HMOE_H */
