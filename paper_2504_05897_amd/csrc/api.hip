// Host side of libhmoe: argument checks, weight packing, the expert cache (slot table, LRU
// planning, staging streams and events) and the FFN dispatcher.
#include <string.h>

#include <algorithm>
#include <cmath>
#include <new>
#include <string>

#include "common.h"

namespace hmoe {

static thread_local std::string g_last_error;

int set_hip_error(hipError_t err, const char* what) {
  g_last_error = std::string(what) + ": " + hipGetErrorString(err);
  (void)hipGetLastError();  // clear the sticky error state
  return HMOE_ERR_HIP;
}

int set_error_text(int status, const char* text) {
  g_last_error = text;
  return status;
}

int check_desc(const hmoe_layer_desc* d) {
  if (!d) return HMOE_ERR_INVALID_ARG;
  if (d->hidden <= 0 || d->ffn <= 0 || d->n_experts <= 0 || d->top_k <= 0 || d->n_slots <= 0)
    return HMOE_ERR_INVALID_ARG;
  if (d->top_k > d->n_experts || d->n_slots > d->n_experts) return HMOE_ERR_INVALID_ARG;
  if (d->dtype != HMOE_F32 && d->dtype != HMOE_BF16 && d->dtype != HMOE_BF16_W4) return HMOE_ERR_INVALID_ARG;
  if (d->n_experts > HMOE_MAX_EXPERTS || d->top_k > HMOE_MAX_TOP_K) return HMOE_ERR_UNSUPPORTED;
  return HMOE_OK;
}

static int check_ffn_shape(const hmoe_layer_desc* d) {
  int rc = check_desc(d);
  if (rc != HMOE_OK) return rc;
  if (d->dtype == HMOE_BF16 && (d->hidden % 64 != 0 || d->ffn % 64 != 0)) return HMOE_ERR_UNSUPPORTED;
  if (d->dtype == HMOE_BF16_W4 && (d->hidden % W4_GROUP != 0 || d->ffn % W4_GROUP != 0)) return HMOE_ERR_UNSUPPORTED;
  return HMOE_OK;
}

// ---- timing probe ----------------------------------------------------------------------
static std::vector<hipEvent_t> g_probe_ev;  // pairs
static int g_probe_used = 0;
static bool g_probe_armed = false;

void probe_before(hipStream_t s) {
  if (g_probe_armed && 2 * g_probe_used + 1 < (int)g_probe_ev.size()) (void)hipEventRecord(g_probe_ev[2 * g_probe_used], s);
}
void probe_after(hipStream_t s) {
  if (g_probe_armed && 2 * g_probe_used + 1 < (int)g_probe_ev.size()) {
    (void)hipEventRecord(g_probe_ev[2 * g_probe_used + 1], s);
    ++g_probe_used;
  }
}

__global__ void set_slot_kernel(int32_t* slot_of, int e_new, int slot, int e_old) {
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    if (e_old >= 0) slot_of[e_old] = -1;
    if (e_new >= 0) slot_of[e_new] = slot;
  }
}

}  // namespace hmoe

using namespace hmoe;

extern "C" const char* hmoe_status_string(int32_t status) {
  switch (status) {
    case HMOE_OK: return "ok";
    case HMOE_ERR_INVALID_ARG: return "invalid argument";
    case HMOE_ERR_UNSUPPORTED: return "shape or dtype not supported by this build";
    case HMOE_ERR_WORKSPACE: return "workspace too small";
    case HMOE_ERR_NOT_RESIDENT: return "expert not resident in the cache";
    case HMOE_ERR_SLOT_BUSY: return "no usable cache slot";
    case HMOE_ERR_HIP: return "HIP runtime error";
    default: return "unknown status";
  }
}

extern "C" const char* hmoe_last_error(void) { return g_last_error.c_str(); }

extern "C" int32_t hmoe_probe_arm(int32_t max_pairs) {
  if (max_pairs <= 0) return HMOE_ERR_INVALID_ARG;
  for (hipEvent_t e : g_probe_ev) (void)hipEventDestroy(e);
  g_probe_ev.clear();
  g_probe_ev.resize(2 * (size_t)max_pairs);
  for (auto& e : g_probe_ev) HMOE_HIP(hipEventCreate(&e));
  g_probe_used = 0;
  g_probe_armed = true;
  return HMOE_OK;
}

extern "C" int32_t hmoe_probe_read(float* h_ms, int32_t max, int32_t* n) {
  if (!h_ms || !n || max < 0) return HMOE_ERR_INVALID_ARG;
  g_probe_armed = false;
  const int cnt = std::min<int>(g_probe_used, max);
  for (int i = 0; i < cnt; ++i) {
    HMOE_HIP(hipEventSynchronize(g_probe_ev[2 * i + 1]));
    HMOE_HIP(hipEventElapsedTime(&h_ms[i], g_probe_ev[2 * i], g_probe_ev[2 * i + 1]));
  }
  *n = cnt;
  for (hipEvent_t e : g_probe_ev) (void)hipEventDestroy(e);
  g_probe_ev.clear();
  g_probe_used = 0;
  return HMOE_OK;
}

// ---- weights ---------------------------------------------------------------------------
extern "C" size_t hmoe_slot_bytes(const hmoe_layer_desc* desc) {
  if (check_desc(desc) != HMOE_OK) return 0;
  if (desc->dtype == HMOE_BF16_W4) {
    if (check_ffn_shape(desc) != HMOE_OK) return 0;
    return w4_offsets((size_t)desc->hidden, (size_t)desc->ffn).total;  // a multiple of 256 for valid shapes
  }
  const size_t elem = desc->dtype == HMOE_BF16 ? 2 : 4;
  const size_t raw = 3 * (size_t)desc->hidden * desc->ffn * elem;
  return (raw + 255) & ~(size_t)255;
}

// ---- 4-bit quantisation (host) ------------------------------------------------------------
static float bf16_bits_to_f32(bf16_t b) {
  const uint32_t u = (uint32_t)b << 16;
  float f;
  memcpy(&f, &u, 4);
  return f;
}
static bf16_t f32_to_bf16_bits_rne(float f) {
  uint32_t u;
  memcpy(&u, &f, 4);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}
// Quantises src [N, K] (bfloat16, row-major) into the unit stream `units` and the scale array `scales`
// of a matrix whose packed 16-row group index of source rows [16 q, 16 q + 16) is q * stride + first.
static void quantize_matrix_w4(const bf16_t* src, int N, int K, uint32_t* units, bf16_t* scales, int stride, int first) {
  const int n_groups = K / W4_GROUP;
  for (int n = 0; n < N; ++n) {
    const int packed_n = ((n / 16) * stride + first) * 16 + n % 16;
    for (int g = 0; g < n_groups; ++g) {
      const bf16_t* w = src + (size_t)n * K + (size_t)g * W4_GROUP;
      float amax = 0.0f;
      for (int k = 0; k < W4_GROUP; ++k) amax = std::max(amax, std::fabs(bf16_bits_to_f32(w[k])));
      const bf16_t sb = f32_to_bf16_bits_rne(amax / 7.0f);
      const float s = bf16_bits_to_f32(sb);
      scales[w4_scale_index(packed_n, g, n_groups)] = sb;
      for (int k = 0; k < W4_GROUP; ++k) {
        int q = 8;
        if (s != 0.0f) {
          float r = std::nearbyintf(bf16_bits_to_f32(w[k]) / s);  // nearest even (default rounding mode)
          r = std::min(7.0f, std::max(-8.0f, r));
          q = (int)r + 8;
        }
        const int kk = g * W4_GROUP + k;
        units[w4_dword_index(packed_n, kk, K)] |= (uint32_t)q << w4_code_shift(kk);
      }
    }
  }
}

// rows [n0, n0+32) of src [*, K] -> one 32-row group of tiles at dst
static void pack_row_group(const bf16_t* src, int n0, int K, bf16_t* dst) {
  const int kt = K / TILE_K;
  for (int kb = 0; kb < kt; ++kb) {
    bf16_t* tile = dst + (size_t)kb * TILE_ELEMS;
    for (int lane = 0; lane < 64; ++lane) {
      const bf16_t* s = src + (size_t)(n0 + lane % TILE_N) * K + kb * TILE_K + 8 * (lane / TILE_N);
      memcpy(tile + lane * 8, s, 16);
    }
  }
}

extern "C" int32_t hmoe_pack_expert(const hmoe_layer_desc* desc, const void* h_w_gate, const void* h_w_up,
                                    const void* h_w_down, void* h_packed_out) {
  int rc = check_ffn_shape(desc);
  if (rc != HMOE_OK) return rc;
  if (!h_w_gate || !h_w_up || !h_w_down || !h_packed_out) return HMOE_ERR_INVALID_ARG;
  const size_t H = desc->hidden, F = desc->ffn;
  if (desc->dtype == HMOE_F32) {
    float* out = (float*)h_packed_out;
    memcpy(out, h_w_gate, F * H * 4);
    memcpy(out + F * H, h_w_up, F * H * 4);
    memcpy(out + 2 * F * H, h_w_down, F * H * 4);
    return HMOE_OK;
  }
  if (desc->dtype == HMOE_BF16_W4) {
    const W4Offsets off = w4_offsets(H, F);
    char* base = (char*)h_packed_out;
    memset(base, 0, off.total);
    quantize_matrix_w4((const bf16_t*)h_w_gate, (int)F, (int)H, (uint32_t*)base, (bf16_t*)(base + off.gate_up_scales), 2, 0);
    quantize_matrix_w4((const bf16_t*)h_w_up, (int)F, (int)H, (uint32_t*)base, (bf16_t*)(base + off.gate_up_scales), 2, 1);
    quantize_matrix_w4((const bf16_t*)h_w_down, (int)H, (int)F, (uint32_t*)(base + off.down_units),
                       (bf16_t*)(base + off.down_scales), 1, 0);
    return HMOE_OK;
  }
  bf16_t* out = (bf16_t*)h_packed_out;
  const size_t group = (size_t)TILE_N * H;  // elements of one packed 32-row group of the gate/up matrix
  for (size_t q = 0; q < F / TILE_N; ++q) {
    pack_row_group((const bf16_t*)h_w_gate, (int)(q * TILE_N), (int)H, out + (2 * q) * group);
    pack_row_group((const bf16_t*)h_w_up, (int)(q * TILE_N), (int)H, out + (2 * q + 1) * group);
  }
  bf16_t* down = out + 2 * F * H;
  for (size_t nb = 0; nb < H / TILE_N; ++nb)
    pack_row_group((const bf16_t*)h_w_down, (int)(nb * TILE_N), (int)F, down + nb * (size_t)TILE_N * F);
  return HMOE_OK;
}

// ---- cache -----------------------------------------------------------------------------
extern "C" int32_t hmoe_cache_create(const hmoe_layer_desc* desc, void* slot_storage, int32_t* d_slot_of,
                                     hmoe_cache** out) {
  int rc = check_desc(desc);
  if (rc != HMOE_OK) return rc;
  if (!slot_storage || !d_slot_of || !out) return HMOE_ERR_INVALID_ARG;
  if (reinterpret_cast<uintptr_t>(slot_storage) & 255u) return HMOE_ERR_INVALID_ARG;
  hmoe_cache* c = new (std::nothrow) hmoe_cache();
  if (!c) return HMOE_ERR_INVALID_ARG;
  c->desc = *desc;
  c->slots = (char*)slot_storage;
  c->slot_bytes = hmoe_slot_bytes(desc);
  c->d_slot_of = d_slot_of;
  c->slot_of.assign(desc->n_experts, -1);
  c->expert_in.assign(desc->n_slots, -1);
  c->tick.assign(desc->n_experts, 0);
  c->clock = 1;
  c->policy = HMOE_POLICY_LRU;
  c->alpha = 0.5;
  c->score.assign(desc->n_experts, 0.0);
  c->pinned.assign(desc->n_slots, 0);
  c->use_seq = 0;
  c->track_reads = desc->n_slots < desc->n_experts;
  c->reads_in_graphs = false;
  c->has_beside = false;
  c->slot_last_read.assign(desc->n_slots, 0);
  c->ready_ev.assign(desc->n_slots, nullptr);
  for (auto& e : c->use_ev) e = nullptr;
  c->fence_ev = nullptr;
  hipError_t err = hipGetDevice(&c->device);
  for (int i = 0; err == hipSuccess && i < hmoe_cache::RING; ++i)
    err = hipEventCreateWithFlags(&c->use_ev[i], hipEventDisableTiming);
  for (int i = 0; err == hipSuccess && i < desc->n_slots; ++i)
    err = hipEventCreateWithFlags(&c->ready_ev[i], hipEventDisableTiming);
  if (err == hipSuccess) err = hipEventCreateWithFlags(&c->fence_ev, hipEventDisableTiming);
  if (err == hipSuccess)
    err = hipMemcpy(d_slot_of, c->slot_of.data(), sizeof(int32_t) * desc->n_experts, hipMemcpyHostToDevice);
  if (err != hipSuccess) {
    hmoe_cache_destroy(c);
    return set_hip_error(err, "hmoe_cache_create");
  }
  *out = c;
  return HMOE_OK;
}

extern "C" int32_t hmoe_cache_destroy(hmoe_cache* c) {
  if (!c) return HMOE_ERR_INVALID_ARG;
  for (auto e : c->use_ev)
    if (e) (void)hipEventDestroy(e);
  for (auto e : c->ready_ev)
    if (e) (void)hipEventDestroy(e);
  if (c->fence_ev) (void)hipEventDestroy(c->fence_ev);
  delete c;
  return HMOE_OK;
}

extern "C" int32_t hmoe_cache_lookup(const hmoe_cache* c, int32_t expert_id, int32_t* slot_out) {
  if (!c || !slot_out || expert_id < 0 || expert_id >= c->desc.n_experts) return HMOE_ERR_INVALID_ARG;
  *slot_out = c->slot_of[expert_id];
  return HMOE_OK;
}

extern "C" int32_t hmoe_cache_occupant(const hmoe_cache* c, int32_t slot, int32_t* expert_out) {
  if (!c || !expert_out || slot < 0 || slot >= c->desc.n_slots) return HMOE_ERR_INVALID_ARG;
  *expert_out = c->expert_in[slot];
  return HMOE_OK;
}

extern "C" int32_t hmoe_cache_pin_slot(hmoe_cache* c, int32_t slot, int32_t pinned) {
  if (!c || slot < 0 || slot >= c->desc.n_slots) return HMOE_ERR_INVALID_ARG;
  c->pinned[slot] = pinned ? 1 : 0;
  return HMOE_OK;
}

extern "C" int32_t hmoe_cache_evict(hmoe_cache* c, int32_t expert_id, void* compute_stream) {
  if (!c || expert_id < 0 || expert_id >= c->desc.n_experts) return HMOE_ERR_INVALID_ARG;
  const int s = c->slot_of[expert_id];
  if (s < 0) return HMOE_OK;
  hipLaunchKernelGGL(set_slot_kernel, dim3(1), dim3(64), 0, (hipStream_t)compute_stream, c->d_slot_of, -1, -1,
                     expert_id);
  HMOE_HIP(hipGetLastError());
  c->slot_of[expert_id] = -1;
  c->expert_in[s] = -1;
  return HMOE_OK;
}

extern "C" int32_t hmoe_cache_stage(hmoe_cache* c, int32_t expert_id, int32_t slot, const void* h_packed_pinned,
                                    void* compute_stream, void* copy_stream) {
  if (!c || expert_id < 0 || expert_id >= c->desc.n_experts || slot < -1 || slot >= c->desc.n_slots)
    return HMOE_ERR_INVALID_ARG;
  hipStream_t comp = (hipStream_t)compute_stream, copy = (hipStream_t)copy_stream;
  if (slot < 0) {
    for (int s = 0; s < c->desc.n_slots && slot < 0; ++s)
      if (c->expert_in[s] < 0 && !c->pinned[s]) slot = s;
    if (slot < 0) return HMOE_ERR_SLOT_BUSY;
  }
  if (c->pinned[slot]) return HMOE_ERR_SLOT_BUSY;
  const int prev_slot = c->slot_of[expert_id];
  if (prev_slot >= 0 && prev_slot != slot) {  // resident elsewhere: drop that copy first
    int rc = hmoe_cache_evict(c, expert_id, compute_stream);
    if (rc != HMOE_OK) return rc;
  }
  const int e_old = c->expert_in[slot] == expert_id ? -1 : c->expert_in[slot];
  if (h_packed_pinned) {
    // the copy may overwrite the slot only after the last FFN call that could read it
    if (!c->track_reads || c->reads_in_graphs) {
      // reads were not tracked so far, or some of them sit in captured graphs whose replays are not tracked: order the
      // copy after everything enqueued on compute
      HMOE_HIP(hipEventRecord(c->fence_ev, comp));
      HMOE_HIP(hipStreamWaitEvent(copy, c->fence_ev, 0));
      c->track_reads = true;
    } else if (c->slot_last_read[slot] != 0) {
      HMOE_HIP(hipStreamWaitEvent(copy, c->use_ev[c->slot_last_read[slot] % hmoe_cache::RING], 0));
    }
    HMOE_HIP(hipMemcpyAsync(c->slots + (size_t)slot * c->slot_bytes, h_packed_pinned, c->slot_bytes,
                            hipMemcpyHostToDevice, copy));
    HMOE_HIP(hipEventRecord(c->ready_ev[slot], copy));
    HMOE_HIP(hipStreamWaitEvent(comp, c->ready_ev[slot], 0));
  }
  hipLaunchKernelGGL(set_slot_kernel, dim3(1), dim3(64), 0, comp, c->d_slot_of, expert_id, slot, e_old);
  HMOE_HIP(hipGetLastError());
  if (e_old >= 0) c->slot_of[e_old] = -1;
  c->slot_of[expert_id] = slot;
  c->expert_in[slot] = expert_id;
  return HMOE_OK;
}

extern "C" int32_t hmoe_cache_plan(hmoe_cache* c, const int32_t* h_counts, int32_t* h_wave, int32_t* h_slot,
                                   int32_t* h_victim, int32_t* n_waves) {
  if (!c || !h_counts || !h_wave || !h_slot || !h_victim || !n_waves) return HMOE_ERR_INVALID_ARG;
  const int E = c->desc.n_experts, S = c->desc.n_slots;
  std::vector<int32_t> occ(c->expert_in);  // planned occupant per slot
  const int64_t base = c->clock;
  int last_wave = 0;
  for (int e = 0; e < E; ++e) {
    h_wave[e] = -1;
    h_slot[e] = -1;
    h_victim[e] = -1;
    if (h_counts[e] > 0 && c->slot_of[e] >= 0) {
      h_wave[e] = 0;
      h_slot[e] = c->slot_of[e];
      c->tick[e] = base;
    }
  }
  for (int e = 0; e < E; ++e) {
    if (h_counts[e] <= 0 || h_wave[e] == 0) continue;
    int target = -1;
    for (int s = 0; s < S && target < 0; ++s)
      if (occ[s] < 0 && !c->pinned[s]) target = s;
    int wave = 1;
    if (target < 0) {
      for (int s = 0; s < S; ++s) {
        if (c->pinned[s]) continue;
        if (target < 0) { target = s; continue; }
        const int a = occ[s], b = occ[target];
        bool better;
        if (c->policy == HMOE_POLICY_MRS) {
          // class: not needed by this call first, then by the wave in which it is computed; lowest S inside a class
          const int ca = h_wave[a] >= 0 ? 1 + h_wave[a] : 0, cb = h_wave[b] >= 0 ? 1 + h_wave[b] : 0;
          better = ca < cb || (ca == cb && c->score[a] < c->score[b]);
        } else {
          better = c->tick[a] < c->tick[b];
        }
        if (better) target = s;
      }
      if (target < 0) return HMOE_ERR_SLOT_BUSY;
      const int victim = occ[target];
      h_victim[e] = victim;
      if (h_wave[victim] >= 0) wave = h_wave[victim] + 1;
    }
    occ[target] = e;
    h_slot[e] = target;
    h_wave[e] = wave;
    c->tick[e] = base + wave;
    last_wave = std::max(last_wave, wave);
  }
  c->clock = base + last_wave + 1;
  *n_waves = last_wave + 1;
  return HMOE_OK;
}

extern "C" int32_t hmoe_cache_set_policy(hmoe_cache* c, int32_t policy, float alpha) {
  if (!c || (policy != HMOE_POLICY_LRU && policy != HMOE_POLICY_MRS)) return HMOE_ERR_INVALID_ARG;
  if (policy == HMOE_POLICY_MRS && !(alpha > 0.0f && alpha <= 1.0f)) return HMOE_ERR_INVALID_ARG;
  c->policy = policy;
  if (policy == HMOE_POLICY_MRS) c->alpha = alpha;
  return HMOE_OK;
}

extern "C" int32_t hmoe_cache_set_layer(hmoe_cache* c, const hmoe_layer_desc* routed) {
  if (!c) return HMOE_ERR_INVALID_ARG;
  if (!routed) {
    c->has_beside = false;
    return HMOE_OK;
  }
  int rc = check_desc(routed);
  if (rc != HMOE_OK) return rc;
  if (c->desc.n_experts != 1 || routed->hidden != c->desc.hidden || routed->dtype != c->desc.dtype) return HMOE_ERR_INVALID_ARG;
  c->beside = *routed;
  c->has_beside = true;
  return HMOE_OK;
}

extern "C" int32_t hmoe_cache_update_scores(hmoe_cache* c, const float* h_scores, int32_t top_p) {
  if (!c || !h_scores || top_p < 1) return HMOE_ERR_INVALID_ARG;
  const int E = c->desc.n_experts;
  // TopP: the top_p largest scores (ties: lower id) are accumulated, the others count as 0
  std::vector<int> order(E);
  for (int e = 0; e < E; ++e) order[e] = e;
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return h_scores[a] > h_scores[b]; });
  std::vector<uint8_t> keep(E, 0);
  for (int i = 0; i < E && i < top_p; ++i) keep[order[i]] = 1;
  for (int e = 0; e < E; ++e)
    c->score[e] = c->alpha * (keep[e] ? (double)h_scores[e] : 0.0) + (1.0 - c->alpha) * c->score[e];
  return HMOE_OK;
}

extern "C" int32_t hmoe_cache_get_scores(const hmoe_cache* c, double* h_out) {
  if (!c || !h_out) return HMOE_ERR_INVALID_ARG;
  for (int e = 0; e < c->desc.n_experts; ++e) h_out[e] = c->score[e];
  return HMOE_OK;
}

// ---- FFN dispatch ------------------------------------------------------------------------
extern "C" size_t hmoe_ffn_workspace_bytes(const hmoe_layer_desc* desc, int32_t A) {
  if (check_desc(desc) != HMOE_OK || A < 0) return 0;
  const size_t elem = desc->dtype == HMOE_F32 ? 4 : 2;
  return (((size_t)A * desc->ffn * elem) + 255) & ~(size_t)255;
}

// Checks the arguments of one grouped-FFN call, fills the launch arguments and resolves HMOE_FFN_AUTO.
// *skip is set when there is nothing to compute (A == 0).
static int32_t ffn_prepare(const hmoe_layer_desc* desc, hmoe_cache* cache, const void* x_perm, const int32_t* row_map,
                           const int32_t* expert_offsets, int32_t A, const int32_t* h_active, int32_t n_active,
                           void* o_perm, void* workspace, size_t workspace_bytes, int32_t* path, void* stream, FfnArgs* out,
                           bool* skip) {
  int rc = check_ffn_shape(desc);
  if (rc != HMOE_OK) return rc;
  if (!cache || A < 0 || !expert_offsets) return HMOE_ERR_INVALID_ARG;
  if (memcmp(desc, &cache->desc, sizeof(*desc)) != 0) return HMOE_ERR_INVALID_ARG;
  if (*path < HMOE_FFN_AUTO || *path > HMOE_FFN_TILED) return HMOE_ERR_INVALID_ARG;
  *skip = A == 0;
  if (A == 0) return HMOE_OK;
  if (!x_perm || !o_perm) return HMOE_ERR_INVALID_ARG;
  if (!aligned16(x_perm) || !aligned16(o_perm) || !aligned16(workspace)) return HMOE_ERR_INVALID_ARG;
  if (!workspace || workspace_bytes < hmoe_ffn_workspace_bytes(desc, A)) return HMOE_ERR_WORKSPACE;
  if (h_active && n_active < 0) return HMOE_ERR_INVALID_ARG;

  FfnArgs& a = *out;
  a.desc = desc;
  a.x_perm = x_perm;
  a.row_map = row_map;
  a.map_div = desc->top_k;
  a.offsets = expert_offsets;
  a.n_rows = A;
  a.slot_of = cache->d_slot_of;
  a.slots = cache->slots;
  a.slot_bytes = cache->slot_bytes;
  a.o_perm = o_perm;
  a.h = workspace;
  a.stream = (hipStream_t)stream;
  a.beside = cache->has_beside ? &cache->beside : nullptr;
  memset(&a.active, 0, sizeof(a.active));
  if (h_active) {
    for (int i = 0; i < n_active; ++i) {
      const int e = h_active[i];
      if (e < 0 || e >= desc->n_experts) return HMOE_ERR_INVALID_ARG;
      if (cache->slot_of[e] < 0) return HMOE_ERR_NOT_RESIDENT;
      a.active.w[e >> 6] |= 1ull << (e & 63);
    }
  } else {
    for (int e = 0; e < desc->n_experts; ++e) a.active.w[e >> 6] |= 1ull << (e & 63);
  }

  if (*path == HMOE_FFN_AUTO) {
    if (desc->dtype == HMOE_F32) *path = HMOE_FFN_REFERENCE;
    else if (desc->dtype == HMOE_BF16_W4) *path = (A / desc->top_k <= 64) ? HMOE_FFN_SKINNY : HMOE_FFN_TILED;
    else *path = (A / desc->top_k <= 32) ? HMOE_FFN_SKINNY : HMOE_FFN_TILED;
  }
  if (desc->dtype == HMOE_F32 && *path != HMOE_FFN_REFERENCE) return HMOE_ERR_UNSUPPORTED;
  return HMOE_OK;
}

static int32_t ffn_launch(const FfnArgs& a, int32_t path) {
  if (path == HMOE_FFN_REFERENCE) return launch_ffn_reference(a);
  if (path == HMOE_FFN_SKINNY) return a.desc->dtype == HMOE_BF16_W4 ? launch_ffn_skinny_w4(a) : launch_ffn_skinny(a);
  return a.desc->dtype == HMOE_BF16_W4 ? launch_ffn_tiled_w4(a) : launch_ffn_tiled(a);
}

// remembers, per slot, the last call that read it, so that a later copy into the slot can wait for it
static int32_t ffn_record_reads(hmoe_cache* cache, const FfnArgs& a) {
  if (!cache->track_reads) return HMOE_OK;
  // Under stream capture an event record becomes a node of the graph: it says nothing about when a replay reads the
  // slots.  From then on a copy into a slot is ordered after everything enqueued on the compute stream instead.
  hipStreamCaptureStatus capturing = hipStreamCaptureStatusNone;
  HMOE_HIP(hipStreamIsCapturing(a.stream, &capturing));
  if (capturing != hipStreamCaptureStatusNone) {
    cache->reads_in_graphs = true;
    return HMOE_OK;
  }
  const uint64_t seq = ++cache->use_seq;
  HMOE_HIP(hipEventRecord(cache->use_ev[seq % hmoe_cache::RING], a.stream));
  for (int e = 0; e < cache->desc.n_experts; ++e)
    if (a.active.test(e) && cache->slot_of[e] >= 0) cache->slot_last_read[cache->slot_of[e]] = seq;
  return HMOE_OK;
}

static int32_t ffn_grouped(const hmoe_layer_desc* desc, hmoe_cache* cache, const void* x_perm, const int32_t* row_map,
                           const int32_t* expert_offsets, int32_t A, const int32_t* h_active, int32_t n_active,
                           void* o_perm, void* workspace, size_t workspace_bytes, int32_t path, void* stream) {
  FfnArgs a;
  bool skip = false;
  int rc = ffn_prepare(desc, cache, x_perm, row_map, expert_offsets, A, h_active, n_active, o_perm, workspace,
                       workspace_bytes, &path, stream, &a, &skip);
  if (rc != HMOE_OK || skip) return rc;
  rc = ffn_launch(a, path);
  if (rc != HMOE_OK) return rc;
  return ffn_record_reads(cache, a);
}

extern "C" int32_t hmoe_expert_ffn_grouped(const hmoe_layer_desc* desc, hmoe_cache* cache, const void* x_perm,
                                           const int32_t* expert_offsets, int32_t A, const int32_t* h_active,
                                           int32_t n_active, void* o_perm, void* workspace, size_t workspace_bytes,
                                           int32_t path, void* stream) {
  return ffn_grouped(desc, cache, x_perm, nullptr, expert_offsets, A, h_active, n_active, o_perm, workspace,
                     workspace_bytes, path, stream);
}

extern "C" int32_t hmoe_expert_ffn_grouped_gather(const hmoe_layer_desc* desc, hmoe_cache* cache, const void* x,
                                                  const int32_t* perm, const int32_t* expert_offsets, int32_t A,
                                                  const int32_t* h_active, int32_t n_active, void* o_perm,
                                                  void* workspace, size_t workspace_bytes, int32_t path, void* stream) {
  if (A > 0 && !perm) return HMOE_ERR_INVALID_ARG;
  return ffn_grouped(desc, cache, x, perm, expert_offsets, A, h_active, n_active, o_perm, workspace, workspace_bytes,
                     path, stream);
}

extern "C" int32_t hmoe_expert_ffn_grouped_with_shared(
    const hmoe_layer_desc* desc, hmoe_cache* cache, const void* x, const int32_t* perm, const int32_t* expert_offsets,
    int32_t A, const int32_t* h_active, int32_t n_active, void* o_perm, void* workspace, size_t workspace_bytes,
    const hmoe_layer_desc* shared_desc, hmoe_cache* shared_cache, const int32_t* shared_offsets, int32_t T, void* o_shared,
    void* shared_workspace, size_t shared_workspace_bytes, int32_t path, void* stream) {
  if (A > 0 && !perm) return HMOE_ERR_INVALID_ARG;
  if (!shared_desc || T < 0) return HMOE_ERR_INVALID_ARG;
  if (shared_desc->n_experts != 1 || shared_desc->n_slots != 1 || shared_desc->top_k != 1) return HMOE_ERR_INVALID_ARG;
  FfnArgs routed, dense;
  bool skip_routed = false, skip_dense = false;
  int32_t path_routed = path, path_dense = path;
  int rc = ffn_prepare(desc, cache, x, perm, expert_offsets, A, h_active, n_active, o_perm, workspace, workspace_bytes,
                       &path_routed, stream, &routed, &skip_routed);
  if (rc != HMOE_OK) return rc;
  rc = ffn_prepare(shared_desc, shared_cache, x, nullptr, shared_offsets, T, nullptr, 0, o_shared, shared_workspace,
                   shared_workspace_bytes, &path_dense, stream, &dense, &skip_dense);
  if (rc != HMOE_OK) return rc;
  if (desc->hidden != shared_desc->hidden || desc->dtype != shared_desc->dtype) return HMOE_ERR_INVALID_ARG;
  // One pair of launches for both when both are decode-sized bf16 calls; otherwise the two calls one after the other.
  const bool together = !skip_routed && !skip_dense && desc->dtype == HMOE_BF16 && path_routed == HMOE_FFN_SKINNY &&
                        path_dense == HMOE_FFN_SKINNY && shared_cache->slot_of[0] >= 0;
  if (together) {
    dense.slots = shared_cache->slots + (size_t)shared_cache->slot_of[0] * shared_cache->slot_bytes;
    rc = launch_ffn_skinny(routed, &dense);
    if (rc != HMOE_OK) return rc;
  } else {
    if (!skip_routed && (rc = ffn_launch(routed, path_routed)) != HMOE_OK) return rc;
    if (!skip_dense && (rc = ffn_launch(dense, path_dense)) != HMOE_OK) return rc;
  }
  if (!skip_routed && (rc = ffn_record_reads(cache, routed)) != HMOE_OK) return rc;
  if (!skip_dense && (rc = ffn_record_reads(shared_cache, dense)) != HMOE_OK) return rc;
  return HMOE_OK;
}

extern "C" size_t hmoe_ffn_combine_sync_bytes(const hmoe_layer_desc* desc) {
  if (check_desc(desc) != HMOE_OK) return 0;
  return (((size_t)desc->hidden / TILE_N + 1) * sizeof(unsigned int) + 255) & ~(size_t)255;
}

extern "C" int32_t hmoe_expert_ffn_combine(
    const hmoe_layer_desc* desc, hmoe_cache* cache, const void* x, const int32_t* perm, const int32_t* inv_perm,
    const float* topk_w, const int32_t* expert_offsets, int32_t T, void* o_perm, void* workspace, size_t workspace_bytes,
    const hmoe_layer_desc* shared_desc, hmoe_cache* shared_cache, const int32_t* shared_offsets, void* o_shared,
    void* shared_workspace, size_t shared_workspace_bytes, void* y, void* sync, size_t sync_bytes, int32_t path, void* stream) {
  int rc = check_desc(desc);
  if (rc != HMOE_OK) return rc;
  if (T < 0) return HMOE_ERR_INVALID_ARG;
  if (T == 0) return HMOE_OK;
  const int32_t A = T * desc->top_k;
  if (!perm || !inv_perm || !topk_w || !y || !aligned16(y)) return HMOE_ERR_INVALID_ARG;
  if (shared_desc && (shared_desc->n_experts != 1 || shared_desc->n_slots != 1 || shared_desc->top_k != 1 ||
                      shared_desc->hidden != desc->hidden || shared_desc->dtype != desc->dtype || !o_shared))
    return HMOE_ERR_INVALID_ARG;
  if (!sync || sync_bytes < hmoe_ffn_combine_sync_bytes(desc) || (reinterpret_cast<uintptr_t>(sync) & 3u)) return HMOE_ERR_WORKSPACE;
  FfnArgs routed, dense;
  bool skip_routed = false, skip_dense = true;
  int32_t path_routed = path, path_dense = path;
  rc = ffn_prepare(desc, cache, x, perm, expert_offsets, A, nullptr, 0, o_perm, workspace, workspace_bytes, &path_routed, stream,
                   &routed, &skip_routed);
  if (rc != HMOE_OK) return rc;
  if (shared_desc) {
    rc = ffn_prepare(shared_desc, shared_cache, x, nullptr, shared_offsets, T, nullptr, 0, o_shared, shared_workspace,
                     shared_workspace_bytes, &path_dense, stream, &dense, &skip_dense);
    if (rc != HMOE_OK) return rc;
    if (shared_cache->slot_of[0] < 0) return HMOE_ERR_NOT_RESIDENT;
  }
  // The sum runs inside the down projection's launch when the FFN is the decode kernel pair and every routed expert
  // is resident (each expert with rows then stores its rows in this call, and at least one block draws every ticket).
  bool all_resident = true;
  for (int e = 0; e < desc->n_experts; ++e) all_resident = all_resident && cache->slot_of[e] >= 0;
  const bool fused = desc->dtype == HMOE_BF16 && path_routed == HMOE_FFN_SKINNY && (!shared_desc || path_dense == HMOE_FFN_SKINNY) &&
                     all_resident && desc->hidden % 8 == 0;
  if (!fused) {  // the calls this one stands for, one after the other
    rc = shared_desc ? hmoe_expert_ffn_grouped_with_shared(desc, cache, x, perm, expert_offsets, A, nullptr, 0, o_perm, workspace,
                                                           workspace_bytes, shared_desc, shared_cache, shared_offsets, T, o_shared,
                                                           shared_workspace, shared_workspace_bytes, path, stream)
                     : hmoe_expert_ffn_grouped_gather(desc, cache, x, perm, expert_offsets, A, nullptr, 0, o_perm, workspace,
                                                      workspace_bytes, path, stream);
    if (rc != HMOE_OK) return rc;
    return hmoe_combine(desc, o_perm, inv_perm, topk_w, shared_desc ? o_shared : nullptr, T, y, stream);
  }
  CombineArgs cb;
  cb.inv_perm = inv_perm;
  cb.topk_w = topk_w;
  cb.y = y;
  cb.tickets = (unsigned int*)sync;
  cb.n_tokens = T;
  if (shared_desc) dense.slots = shared_cache->slots + (size_t)shared_cache->slot_of[0] * shared_cache->slot_bytes;
  rc = launch_ffn_skinny(routed, shared_desc ? &dense : nullptr, &cb);
  if (rc != HMOE_OK) return rc;
  if ((rc = ffn_record_reads(cache, routed)) != HMOE_OK) return rc;
  if (shared_desc && (rc = ffn_record_reads(shared_cache, dense)) != HMOE_OK) return rc;
  return HMOE_OK;
}

extern "C" int32_t hmoe_expert_ffn_staged(const hmoe_layer_desc* desc, hmoe_cache* cache, const void* x, const int32_t* perm,
                                          const int32_t* expert_offsets, int32_t A, const int32_t* h_counts_pinned,
                                          const void* const* h_packed_pinned, void* o_perm, void* workspace,
                                          size_t workspace_bytes, int32_t path, void* compute_stream, void* copy_stream,
                                          int32_t* h_wave, int32_t* h_slot, int32_t* h_victim, int32_t* n_waves,
                                          uint64_t* staged_bytes) {
  int rc = check_ffn_shape(desc);
  if (rc != HMOE_OK) return rc;
  if (!cache || !h_counts_pinned || !h_packed_pinned || !h_wave || !h_slot || !h_victim || !n_waves) return HMOE_ERR_INVALID_ARG;
  if (memcmp(desc, &cache->desc, sizeof(*desc)) != 0 || A < 0) return HMOE_ERR_INVALID_ARG;
  // the plan needs the per-expert loads on the host: wait for whatever delivers them
  HMOE_HIP(hipStreamSynchronize((hipStream_t)compute_stream));
  rc = hmoe_cache_plan(cache, h_counts_pinned, h_wave, h_slot, h_victim, n_waves);
  if (rc != HMOE_OK) return rc;
  const int E = desc->n_experts;
  for (int e = 0; e < E; ++e)
    if (h_wave[e] > 0 && !h_packed_pinned[e]) return HMOE_ERR_INVALID_ARG;
  std::vector<int32_t> members;
  uint64_t staged = 0;
  for (int w = 0; w < *n_waves; ++w) {
    members.clear();
    for (int e = 0; e < E; ++e)
      if (h_wave[e] == w) members.push_back(e);
    if (w > 0) {
      // the copies of a wave go out before its FFN call: each waits on the copy stream for the last call that read its
      // slot only, so it runs under the FFN of earlier waves wherever the slot is not one they read
      for (int e : members) {
        rc = hmoe_cache_stage(cache, e, h_slot[e], h_packed_pinned[e], compute_stream, copy_stream);
        if (rc != HMOE_OK) return rc;
        staged += cache->slot_bytes;
      }
    }
    if (!members.empty()) {
      rc = ffn_grouped(desc, cache, x, perm, expert_offsets, A, members.data(), (int32_t)members.size(), o_perm, workspace,
                       workspace_bytes, path, compute_stream);
      if (rc != HMOE_OK) return rc;
    }
  }
  if (staged_bytes) *staged_bytes = staged;
  return HMOE_OK;
}
