"""Python binding of libhmoe, the MI355X (gfx950) MoE-layer forward over an HBM expert cache.

The functions named ``hmoe_*`` mirror the C ABI of ``include/hmoe.h`` one to one and only
marshal arguments (torch tensors -> device pointers, torch stream -> hipStream_t); every step
of the layer runs in the library's HIP kernels.  PyTorch is used for device memory and streams
only.  There is no CPU or PyTorch fallback: if ``libhmoe.so`` has not been built, importing this
package raises.

``MoELayer`` strings the calls together for one layer (router logits -> route -> permute ->
cache staging -> grouped expert FFN -> combine); it owns the buffers a caller would own.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libhmoe.so")

HMOE_OK = 0
HMOE_ERR_INVALID_ARG = -1
HMOE_ERR_UNSUPPORTED = -2
HMOE_ERR_WORKSPACE = -3
HMOE_ERR_NOT_RESIDENT = -4
HMOE_ERR_SLOT_BUSY = -5
HMOE_ERR_HIP = -6
HMOE_F32 = 0
HMOE_BF16 = 1
HMOE_BF16_W4 = 2      # bf16 activations, 4-bit group-wise expert weights
HMOE_FFN_AUTO, HMOE_FFN_REFERENCE, HMOE_FFN_SKINNY, HMOE_FFN_TILED = 0, 1, 2, 3

# every symbol include/hmoe.h declares
EXPORTS = [
    "hmoe_status_string", "hmoe_last_error", "hmoe_router_logits", "hmoe_route",
    "hmoe_permute_workspace_bytes", "hmoe_permute", "hmoe_permute_static", "hmoe_slot_bytes", "hmoe_pack_expert",
    "hmoe_cache_create", "hmoe_cache_destroy", "hmoe_cache_lookup", "hmoe_cache_occupant",
    "hmoe_cache_evict", "hmoe_cache_pin_slot", "hmoe_cache_stage", "hmoe_cache_plan",
    "hmoe_ffn_workspace_bytes", "hmoe_expert_ffn_grouped", "hmoe_expert_ffn_grouped_gather", "hmoe_route_permute",
    "hmoe_router_route_permute", "hmoe_expert_ffn_grouped_with_shared", "hmoe_ffn_combine_sync_bytes", "hmoe_expert_ffn_combine",
    "hmoe_expert_ffn_staged",
    "hmoe_combine",
    "hmoe_cache_set_policy", "hmoe_cache_update_scores", "hmoe_cache_get_scores", "hmoe_cache_set_layer",
    "hmoe_route_scores_workspace_bytes", "hmoe_route_scores",
    "hmoe_schedule_simulate", "hmoe_schedule_plan",
    "hmoe_probe_arm", "hmoe_probe_read",
]
HMOE_POLICY_LRU, HMOE_POLICY_MRS = 0, 1


class HmoeError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = _lib.hmoe_status_string(status).decode()
        detail = _lib.hmoe_last_error().decode() if status == HMOE_ERR_HIP else ""
        super().__init__("%s: %s (%d) %s" % (where, msg, status, detail))


class SchedCost(ctypes.Structure):
    """Cost model of the scheduling simulation (Section IV-B): time = base + per_token * load."""
    _fields_ = [("gpu_base", ctypes.c_double), ("gpu_per_token", ctypes.c_double), ("cpu_base", ctypes.c_double),
                ("cpu_per_token", ctypes.c_double), ("transfer", ctypes.c_double)]


class LayerDesc(ctypes.Structure):
    _fields_ = [("hidden", ctypes.c_int32), ("ffn", ctypes.c_int32), ("n_experts", ctypes.c_int32),
                ("top_k", ctypes.c_int32), ("n_slots", ctypes.c_int32), ("dtype", ctypes.c_int32)]

    def __repr__(self):
        return "LayerDesc(H=%d, F=%d, E=%d, K=%d, S=%d, %s)" % (
            self.hidden, self.ffn, self.n_experts, self.top_k, self.n_slots, "bf16" if self.dtype else "f32")


def _load() -> ctypes.CDLL:
    if not os.path.exists(_LIB_PATH):
        raise ImportError("libhmoe.so is not built: run `python paper_2504_05897_amd/build.py` "
                          "(needs hipcc; there is no fallback path)")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
    dp = ctypes.POINTER(LayerDesc)
    lib.hmoe_status_string.restype = ctypes.c_char_p
    lib.hmoe_status_string.argtypes = [i32]
    lib.hmoe_last_error.restype = ctypes.c_char_p
    lib.hmoe_last_error.argtypes = []
    lib.hmoe_router_logits.argtypes = [dp, vp, vp, i32, vp, vp]
    lib.hmoe_route.argtypes = [dp, vp, i32, vp, vp, vp]
    lib.hmoe_permute_workspace_bytes.restype = sz
    lib.hmoe_permute_workspace_bytes.argtypes = [dp, i32]
    lib.hmoe_permute.argtypes = [dp, vp, i32, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.hmoe_permute_static.argtypes = [dp, vp, i32, vp, vp, vp, vp, vp, vp, vp]
    lib.hmoe_slot_bytes.restype = sz
    lib.hmoe_slot_bytes.argtypes = [dp]
    lib.hmoe_pack_expert.argtypes = [dp, vp, vp, vp, vp]
    lib.hmoe_cache_create.argtypes = [dp, vp, vp, ctypes.POINTER(vp)]
    lib.hmoe_cache_destroy.argtypes = [vp]
    lib.hmoe_cache_lookup.argtypes = [vp, i32, ctypes.POINTER(i32)]
    lib.hmoe_cache_occupant.argtypes = [vp, i32, ctypes.POINTER(i32)]
    lib.hmoe_cache_evict.argtypes = [vp, i32, vp]
    lib.hmoe_cache_pin_slot.argtypes = [vp, i32, i32]
    lib.hmoe_cache_stage.argtypes = [vp, i32, i32, vp, vp, vp]
    lib.hmoe_cache_plan.argtypes = [vp, vp, vp, vp, vp, ctypes.POINTER(i32)]
    lib.hmoe_ffn_workspace_bytes.restype = sz
    lib.hmoe_ffn_workspace_bytes.argtypes = [dp, i32]
    lib.hmoe_expert_ffn_grouped.argtypes = [dp, vp, vp, vp, i32, vp, i32, vp, vp, sz, i32, vp]
    lib.hmoe_expert_ffn_grouped_gather.argtypes = [dp, vp, vp, vp, vp, i32, vp, i32, vp, vp, sz, i32, vp]
    lib.hmoe_expert_ffn_grouped_with_shared.argtypes = [dp, vp, vp, vp, vp, i32, vp, i32, vp, vp, sz,
                                                        dp, vp, vp, i32, vp, vp, sz, i32, vp]
    lib.hmoe_ffn_combine_sync_bytes.restype = sz
    lib.hmoe_ffn_combine_sync_bytes.argtypes = [dp]
    lib.hmoe_expert_ffn_combine.argtypes = [dp, vp, vp, vp, vp, vp, vp, i32, vp, vp, sz, dp, vp, vp, vp, vp, sz, vp, vp, sz, i32, vp]
    lib.hmoe_expert_ffn_staged.argtypes = [dp, vp, vp, vp, vp, i32, vp, vp, vp, vp, sz, i32, vp, vp, vp, vp, vp,
                                           ctypes.POINTER(i32), ctypes.POINTER(ctypes.c_uint64)]
    lib.hmoe_route_permute.argtypes = [dp, vp, i32, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.hmoe_router_route_permute.argtypes = [dp, vp, vp, i32, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.hmoe_combine.argtypes = [dp, vp, vp, vp, vp, i32, vp, vp]
    lib.hmoe_cache_set_policy.argtypes = [vp, i32, ctypes.c_float]
    lib.hmoe_cache_set_layer.argtypes = [vp, dp]
    lib.hmoe_cache_update_scores.argtypes = [vp, vp, i32]
    lib.hmoe_cache_get_scores.argtypes = [vp, vp]
    lib.hmoe_route_scores_workspace_bytes.restype = sz
    lib.hmoe_route_scores_workspace_bytes.argtypes = [dp, i32]
    lib.hmoe_route_scores.argtypes = [dp, vp, i32, vp, vp, vp, sz, vp]
    lib.hmoe_schedule_simulate.argtypes = [i32, vp, vp, ctypes.POINTER(SchedCost), i32, vp, vp, vp, vp,
                                           ctypes.POINTER(ctypes.c_double)]
    lib.hmoe_schedule_plan.argtypes = [i32, vp, vp, ctypes.POINTER(SchedCost), vp, vp, vp, vp,
                                       ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i32)]
    lib.hmoe_probe_arm.argtypes = [i32]
    lib.hmoe_probe_read.argtypes = [vp, i32, ctypes.POINTER(i32)]
    for name in EXPORTS:
        fn = getattr(lib, name)
        if fn.restype is ctypes.c_int:      # default: the status-returning calls
            fn.restype = i32
    return lib


_lib = _load()


def _check(status: int, where: str) -> None:
    if status != HMOE_OK:
        raise HmoeError(status, where)


def _ptr(t) -> Optional[int]:
    """Device/host address of a tensor or numpy array (None -> NULL)."""
    if t is None:
        return None
    if isinstance(t, torch.Tensor):
        return t.data_ptr()
    if isinstance(t, np.ndarray):
        return t.ctypes.data
    return int(t)


def _stream(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    if isinstance(stream, torch.cuda.Stream):
        return stream.cuda_stream
    return int(stream)


def make_desc(hidden: int, ffn: int, n_experts: int, top_k: int, n_slots: int, dtype: int) -> LayerDesc:
    return LayerDesc(hidden, ffn, n_experts, top_k, n_slots, dtype)


def torch_dtype(desc: LayerDesc):
    return torch.float32 if desc.dtype == HMOE_F32 else torch.bfloat16


# ---------------------------------------------------------------------------------------------
# one-to-one wrappers of the C ABI
# ---------------------------------------------------------------------------------------------
def hmoe_router_logits(desc, x, w_g, T, logits, stream=None):
    _check(_lib.hmoe_router_logits(ctypes.byref(desc), _ptr(x), _ptr(w_g), T, _ptr(logits), _stream(stream)),
           "hmoe_router_logits")


def hmoe_route(desc, logits, T, topk_idx, topk_w, stream=None):
    _check(_lib.hmoe_route(ctypes.byref(desc), _ptr(logits), T, _ptr(topk_idx), _ptr(topk_w), _stream(stream)),
           "hmoe_route")


def hmoe_permute_workspace_bytes(desc, T) -> int:
    return int(_lib.hmoe_permute_workspace_bytes(ctypes.byref(desc), T))


def hmoe_permute(desc, topk_idx, T, x, x_perm, expert_offsets, perm, inv_perm, h_counts_pinned, workspace,
                 workspace_bytes, stream=None):
    _check(_lib.hmoe_permute(ctypes.byref(desc), _ptr(topk_idx), T, _ptr(x), _ptr(x_perm), _ptr(expert_offsets),
                             _ptr(perm), _ptr(inv_perm), _ptr(h_counts_pinned), _ptr(workspace), workspace_bytes,
                             _stream(stream)), "hmoe_permute")


HMOE_PERMUTE_STATIC_BYTES = 1 << 20


def hmoe_permute_static(desc, topk_idx, T, x, x_perm, expert_offsets, perm, inv_perm, h_counts_pinned, stream=None):
    """hmoe_permute without a caller workspace (the library's static scratch array); allocates nothing."""
    status = _lib.hmoe_permute_static(ctypes.byref(desc), _ptr(topk_idx), T, _ptr(x), _ptr(x_perm), _ptr(expert_offsets),
                                      _ptr(perm), _ptr(inv_perm), _ptr(h_counts_pinned), _stream(stream))
    if status == HMOE_ERR_WORKSPACE:
        raise HmoeError(status, "hmoe_permute_static: " + _lib.hmoe_last_error().decode())
    _check(status, "hmoe_permute_static")


def hmoe_slot_bytes(desc) -> int:
    return int(_lib.hmoe_slot_bytes(ctypes.byref(desc)))


def hmoe_pack_expert(desc, h_w_gate, h_w_up, h_w_down, h_packed_out):
    _check(_lib.hmoe_pack_expert(ctypes.byref(desc), _ptr(h_w_gate), _ptr(h_w_up), _ptr(h_w_down),
                                 _ptr(h_packed_out)), "hmoe_pack_expert")


def hmoe_cache_create(desc, slot_storage, d_slot_of) -> int:
    handle = ctypes.c_void_p()
    _check(_lib.hmoe_cache_create(ctypes.byref(desc), _ptr(slot_storage), _ptr(d_slot_of), ctypes.byref(handle)),
           "hmoe_cache_create")
    return handle.value


def hmoe_cache_destroy(cache):
    _check(_lib.hmoe_cache_destroy(cache), "hmoe_cache_destroy")


def hmoe_cache_lookup(cache, expert_id) -> int:
    out = ctypes.c_int32()
    _check(_lib.hmoe_cache_lookup(cache, expert_id, ctypes.byref(out)), "hmoe_cache_lookup")
    return out.value


def hmoe_cache_occupant(cache, slot) -> int:
    out = ctypes.c_int32()
    _check(_lib.hmoe_cache_occupant(cache, slot, ctypes.byref(out)), "hmoe_cache_occupant")
    return out.value


def hmoe_cache_evict(cache, expert_id, compute_stream=None):
    _check(_lib.hmoe_cache_evict(cache, expert_id, _stream(compute_stream)), "hmoe_cache_evict")


def hmoe_cache_pin_slot(cache, slot, pinned):
    _check(_lib.hmoe_cache_pin_slot(cache, slot, int(pinned)), "hmoe_cache_pin_slot")


def hmoe_cache_stage(cache, expert_id, slot, h_packed_pinned, compute_stream=None, copy_stream=None):
    _check(_lib.hmoe_cache_stage(cache, expert_id, slot, _ptr(h_packed_pinned), _stream(compute_stream),
                                 _stream(copy_stream)), "hmoe_cache_stage")


def hmoe_cache_plan(cache, h_counts: np.ndarray):
    """Returns (wave[E], slot[E], victim[E], n_waves) as numpy int32 arrays / int."""
    n = h_counts.shape[0]
    counts = np.ascontiguousarray(h_counts, dtype=np.int32)
    wave = np.empty(n, np.int32)
    slot = np.empty(n, np.int32)
    victim = np.empty(n, np.int32)
    n_waves = ctypes.c_int32()
    _check(_lib.hmoe_cache_plan(cache, _ptr(counts), _ptr(wave), _ptr(slot), _ptr(victim), ctypes.byref(n_waves)),
           "hmoe_cache_plan")
    return wave, slot, victim, n_waves.value


def hmoe_ffn_workspace_bytes(desc, A) -> int:
    return int(_lib.hmoe_ffn_workspace_bytes(ctypes.byref(desc), A))


def hmoe_expert_ffn_grouped(desc, cache, x_perm, expert_offsets, A, h_active, o_perm, workspace, workspace_bytes,
                            path=HMOE_FFN_AUTO, stream=None):
    act = None if h_active is None else np.ascontiguousarray(h_active, dtype=np.int32)
    _check(_lib.hmoe_expert_ffn_grouped(ctypes.byref(desc), cache, _ptr(x_perm), _ptr(expert_offsets), A, _ptr(act),
                                        0 if act is None else int(act.shape[0]), _ptr(o_perm), _ptr(workspace),
                                        workspace_bytes, path, _stream(stream)), "hmoe_expert_ffn_grouped")


def hmoe_expert_ffn_grouped_gather(desc, cache, x, perm, expert_offsets, A, h_active, o_perm, workspace,
                                   workspace_bytes, path=HMOE_FFN_AUTO, stream=None):
    act = None if h_active is None else np.ascontiguousarray(h_active, dtype=np.int32)
    _check(_lib.hmoe_expert_ffn_grouped_gather(ctypes.byref(desc), cache, _ptr(x), _ptr(perm), _ptr(expert_offsets), A,
                                               _ptr(act), 0 if act is None else int(act.shape[0]), _ptr(o_perm),
                                               _ptr(workspace), workspace_bytes, path, _stream(stream)),
           "hmoe_expert_ffn_grouped_gather")


def hmoe_expert_ffn_grouped_with_shared(desc, cache, x, perm, expert_offsets, A, h_active, o_perm, workspace,
                                        workspace_bytes, shared_desc, shared_cache, shared_offsets, T, o_shared,
                                        shared_workspace, shared_workspace_bytes, path=HMOE_FFN_AUTO, stream=None):
    act = None if h_active is None else np.ascontiguousarray(h_active, dtype=np.int32)
    _check(_lib.hmoe_expert_ffn_grouped_with_shared(
        ctypes.byref(desc), cache, _ptr(x), _ptr(perm), _ptr(expert_offsets), A, _ptr(act),
        0 if act is None else int(act.shape[0]), _ptr(o_perm), _ptr(workspace), workspace_bytes,
        ctypes.byref(shared_desc), shared_cache, _ptr(shared_offsets), T, _ptr(o_shared), _ptr(shared_workspace),
        shared_workspace_bytes, path, _stream(stream)), "hmoe_expert_ffn_grouped_with_shared")


def hmoe_expert_ffn_staged(desc, cache, x, perm, expert_offsets, A, h_counts_pinned, h_packed_ptrs, o_perm, workspace,
                           workspace_bytes, path=HMOE_FFN_AUTO, compute_stream=None, copy_stream=None):
    """h_packed_ptrs: ctypes array of E host pointers (c_void_p).  -> (wave[E], slot[E], victim[E], n_waves, staged bytes)"""
    n = desc.n_experts
    wave, slot, victim = (np.empty(n, np.int32) for _ in range(3))
    n_waves, staged = ctypes.c_int32(), ctypes.c_uint64()
    _check(_lib.hmoe_expert_ffn_staged(ctypes.byref(desc), cache, _ptr(x), _ptr(perm), _ptr(expert_offsets), A,
                                       _ptr(h_counts_pinned), ctypes.cast(h_packed_ptrs, ctypes.c_void_p), _ptr(o_perm),
                                       _ptr(workspace), workspace_bytes, path, _stream(compute_stream), _stream(copy_stream),
                                       _ptr(wave), _ptr(slot), _ptr(victim), ctypes.byref(n_waves), ctypes.byref(staged)),
           "hmoe_expert_ffn_staged")
    return wave, slot, victim, n_waves.value, int(staged.value)


def hmoe_ffn_combine_sync_bytes(desc) -> int:
    return int(_lib.hmoe_ffn_combine_sync_bytes(ctypes.byref(desc)))


def hmoe_expert_ffn_combine(desc, cache, x, perm, inv_perm, topk_w, expert_offsets, T, o_perm, workspace, workspace_bytes,
                            shared_desc, shared_cache, shared_offsets, o_shared, shared_workspace, shared_workspace_bytes,
                            y, sync, sync_bytes, path=HMOE_FFN_AUTO, stream=None):
    _check(_lib.hmoe_expert_ffn_combine(
        ctypes.byref(desc), cache, _ptr(x), _ptr(perm), _ptr(inv_perm), _ptr(topk_w), _ptr(expert_offsets), T, _ptr(o_perm),
        _ptr(workspace), workspace_bytes, None if shared_desc is None else ctypes.byref(shared_desc), shared_cache,
        _ptr(shared_offsets), _ptr(o_shared), _ptr(shared_workspace), shared_workspace_bytes, _ptr(y), _ptr(sync), sync_bytes,
        path, _stream(stream)), "hmoe_expert_ffn_combine")


def hmoe_route_permute(desc, logits, T, topk_idx, topk_w, expert_offsets, perm, inv_perm, h_counts_pinned, workspace,
                       workspace_bytes, stream=None):
    _check(_lib.hmoe_route_permute(ctypes.byref(desc), _ptr(logits), T, _ptr(topk_idx), _ptr(topk_w),
                                   _ptr(expert_offsets), _ptr(perm), _ptr(inv_perm), _ptr(h_counts_pinned),
                                   _ptr(workspace), workspace_bytes, _stream(stream)), "hmoe_route_permute")


def hmoe_router_route_permute(desc, x, w_g, T, logits, topk_idx, topk_w, expert_offsets, perm, inv_perm, h_counts_pinned,
                              workspace, workspace_bytes, stream=None):
    _check(_lib.hmoe_router_route_permute(ctypes.byref(desc), _ptr(x), _ptr(w_g), T, _ptr(logits), _ptr(topk_idx),
                                          _ptr(topk_w), _ptr(expert_offsets), _ptr(perm), _ptr(inv_perm),
                                          _ptr(h_counts_pinned), _ptr(workspace), workspace_bytes, _stream(stream)),
           "hmoe_router_route_permute")


def hmoe_combine(desc, o_perm, inv_perm, topk_w, o_shared, T, y, stream=None):
    _check(_lib.hmoe_combine(ctypes.byref(desc), _ptr(o_perm), _ptr(inv_perm), _ptr(topk_w), _ptr(o_shared), T,
                             _ptr(y), _stream(stream)), "hmoe_combine")


def hmoe_cache_set_layer(cache, routed_desc):
    _check(_lib.hmoe_cache_set_layer(cache, None if routed_desc is None else ctypes.byref(routed_desc)), "hmoe_cache_set_layer")


def hmoe_cache_set_policy(cache, policy: int, alpha: float = 0.5):
    _check(_lib.hmoe_cache_set_policy(cache, policy, alpha), "hmoe_cache_set_policy")


def hmoe_cache_update_scores(cache, h_scores, top_p: int):
    s = h_scores.numpy() if isinstance(h_scores, torch.Tensor) else np.ascontiguousarray(h_scores, dtype=np.float32)
    _check(_lib.hmoe_cache_update_scores(cache, _ptr(s), top_p), "hmoe_cache_update_scores")


def hmoe_cache_get_scores(cache, n_experts: int) -> np.ndarray:
    out = np.zeros(n_experts, np.float64)
    _check(_lib.hmoe_cache_get_scores(cache, _ptr(out)), "hmoe_cache_get_scores")
    return out


def hmoe_route_scores_workspace_bytes(desc, T) -> int:
    return int(_lib.hmoe_route_scores_workspace_bytes(ctypes.byref(desc), T))


def hmoe_route_scores(desc, logits, T, scores, h_scores_pinned, workspace, workspace_bytes, stream=None):
    _check(_lib.hmoe_route_scores(ctypes.byref(desc), _ptr(logits), T, _ptr(scores), _ptr(h_scores_pinned),
                                  _ptr(workspace), workspace_bytes, _stream(stream)), "hmoe_route_scores")


HMOE_ON_GPU_CACHED, HMOE_ON_GPU_LOADED, HMOE_ON_CPU = 0, 1, 2
HMOE_SCHED_CPU_UNCACHED, HMOE_SCHED_CPU_CACHED, HMOE_SCHED_TRANSFERS, HMOE_SCHED_ALL = 1, 2, 4, 7


def _sched_call(fn_name, load, cached, cost, rules):
    load = np.ascontiguousarray(load, dtype=np.int32)
    cached = np.ascontiguousarray(cached, dtype=np.int32)
    n = int(load.shape[0])
    device = np.zeros(max(n, 1), np.int32)
    start, end, xfer = (np.zeros(max(n, 1), np.float64) for _ in range(3))
    makespan = ctypes.c_double(0.0)
    if rules is None:
        chosen = ctypes.c_int32(0)
        _check(_lib.hmoe_schedule_plan(n, _ptr(load), _ptr(cached), ctypes.byref(cost), _ptr(device), _ptr(start),
                                       _ptr(end), _ptr(xfer), ctypes.byref(makespan), ctypes.byref(chosen)), fn_name)
        return device[:n], start[:n], end[:n], xfer[:n], makespan.value, chosen.value
    _check(_lib.hmoe_schedule_simulate(n, _ptr(load), _ptr(cached), ctypes.byref(cost), rules, _ptr(device), _ptr(start),
                                       _ptr(end), _ptr(xfer), ctypes.byref(makespan)), fn_name)
    return device[:n], start[:n], end[:n], xfer[:n], makespan.value


def hmoe_schedule_simulate(load, cached, cost: SchedCost, rules: int = HMOE_SCHED_ALL):
    """-> (device [n], start [n], end [n], transfer_start [n], makespan); host only."""
    return _sched_call("hmoe_schedule_simulate", load, cached, cost, rules)


def hmoe_schedule_plan(load, cached, cost: SchedCost):
    """-> (device, start, end, transfer_start, makespan, rules of the winning strategy); host only."""
    return _sched_call("hmoe_schedule_plan", load, cached, cost, None)


def hmoe_probe_arm(max_pairs: int):
    _check(_lib.hmoe_probe_arm(max_pairs), "hmoe_probe_arm")


def hmoe_probe_read(max_pairs: int) -> np.ndarray:
    ms = np.zeros(max_pairs, np.float32)
    n = ctypes.c_int32()
    _check(_lib.hmoe_probe_read(_ptr(ms), max_pairs, ctypes.byref(n)), "hmoe_probe_read")
    return ms[: n.value].copy()


# ---------------------------------------------------------------------------------------------
# buffers of one layer + the call sequence
# ---------------------------------------------------------------------------------------------
def _storage_tensor(a: np.ndarray) -> torch.Tensor:
    """numpy storage array (float32 values or uint16 bf16 bit patterns) -> CPU torch tensor."""
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).view(torch.bfloat16)
    return torch.from_numpy(a)


class MoELayer:
    """One MoE layer on the GPU: slot storage + expert cache + pinned host copies of every
    packed expert + the work buffers for up to ``max_tokens`` tokens.

    ``experts[e]`` / ``shared[i]`` are (W_gate [F,H], W_up [F,H], W_down [H,F]) numpy arrays in
    storage form (float32, or uint16 bf16 bit patterns).  Shared experts are packed as one
    always-resident expert whose FFN dim is the sum of theirs.
    """

    def __init__(self, desc: LayerDesc, experts: Sequence, shared: Sequence = (), w_router=None,
                 max_tokens: int = 1, device: str = "cuda:0", resident: Optional[Sequence[int]] = None,
                 fused: bool = True, host_copies: bool = True):
        self.desc = desc
        self.fused = fused          # route+permute in one call, gather fused into the FFN
        self.overlap_shared = fused  # shared-expert FFN on a side stream, next to the routed path
        self.merge_shared = fused    # decode-sized batches: shared-expert FFN inside the routed experts' launches
        # ... and, on request, the weighted sum inside the down projection's launch (hmoe_expert_ffn_combine): the same
        # bits, one launch fewer, but measured no faster than the separate combine launch (43.2 against 42.8 us on the
        # DeepSeek-V2-Lite-style decode step, 129.6 against 132.3 us Mixtral-style, 307 against 297 us Qwen2-style)
        self.merge_combine = False
        self.dev = torch.device(device)
        self.dt = torch_dtype(desc)
        E, S, K, H, F = desc.n_experts, desc.n_slots, desc.top_k, desc.hidden, desc.ffn
        self.slot_bytes = hmoe_slot_bytes(desc)
        self.slots = torch.empty(S * self.slot_bytes, dtype=torch.uint8, device=self.dev)
        self.slot_of = torch.empty(E, dtype=torch.int32, device=self.dev)
        self.cache = hmoe_cache_create(desc, self.slots, self.slot_of)
        # pinned host copies of the packed experts: what misses are staged from.  A layer whose cache holds every
        # expert never stages; with host_copies=False it packs each expert once and writes it into its slot.
        if not host_copies:
            assert S == E and resident is None and len(experts) == E, "host_copies=False needs every expert resident"
        self.h_packed: List[torch.Tensor] = [torch.empty(self.slot_bytes, dtype=torch.uint8, pin_memory=True)
                                             for _ in experts] if host_copies else []

        def pack_one(i):
            wg, wu, wd = experts[i]
            out = self.h_packed[i] if host_copies else torch.empty(self.slot_bytes, dtype=torch.uint8)
            hmoe_pack_expert(desc, np.ascontiguousarray(wg), np.ascontiguousarray(wu), np.ascontiguousarray(wd), out)
            if not host_copies:
                self.slots[i * self.slot_bytes:(i + 1) * self.slot_bytes].copy_(out)

        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(max_workers=min(16, max(1, len(experts)))) as pool:   # packing is host-side memcpy work
            list(pool.map(pack_one, range(len(experts))))
        self.copy_stream = torch.cuda.Stream(device=self.dev)
        self.side_stream = torch.cuda.Stream(device=self.dev)
        self.ev_fork = torch.cuda.Event()
        self.ev_join = torch.cuda.Event()
        self.w_router = None if w_router is None else _storage_tensor(w_router).to(self.dev)
        # shared experts: one always-resident expert
        self.shared_desc = None
        if len(shared):
            fs = sum(int(s[0].shape[0]) for s in shared)
            self.shared_desc = make_desc(H, fs, 1, 1, 1, desc.dtype)
            wg = np.concatenate([s[0] for s in shared], axis=0)
            wu = np.concatenate([s[1] for s in shared], axis=0)
            wd = np.concatenate([s[2] for s in shared], axis=1)
            sb = hmoe_slot_bytes(self.shared_desc)
            hbuf = torch.empty(sb, dtype=torch.uint8)
            hmoe_pack_expert(self.shared_desc, np.ascontiguousarray(wg), np.ascontiguousarray(wu),
                             np.ascontiguousarray(wd), hbuf)
            self.shared_slots = hbuf.to(self.dev)
            self.shared_slot_of = torch.empty(1, dtype=torch.int32, device=self.dev)
            self.shared_cache = hmoe_cache_create(self.shared_desc, self.shared_slots, self.shared_slot_of)
            hmoe_cache_stage(self.shared_cache, 0, 0, None)
            hmoe_cache_set_layer(self.shared_cache, desc)
        self.h_packed_ptrs = (ctypes.c_void_p * E)(*[t.data_ptr() for t in self.h_packed]) if host_copies else None
        self._alloc(max_tokens)
        for s, e in enumerate(range(S) if resident is None else resident):
            hmoe_cache_stage(self.cache, int(e), s, self.h_packed[int(e)] if host_copies else None, None, self.copy_stream)
        torch.cuda.synchronize(self.dev)
        self.last_plan = None
        self.staged_bytes = 0

    def _alloc(self, max_tokens: int):
        d, dev = self.desc, self.dev
        T, K, E, H = max_tokens, d.top_k, d.n_experts, d.hidden
        A = T * K
        self.max_tokens = T
        self.logits = torch.empty(T, E, dtype=torch.float32, device=dev)
        self.topk_idx = torch.empty(T, K, dtype=torch.int32, device=dev)
        self.topk_w = torch.empty(T, K, dtype=torch.float32, device=dev)
        self.offsets = torch.empty(E + 1, dtype=torch.int32, device=dev)
        self.perm = torch.empty(A, dtype=torch.int32, device=dev)
        self.inv_perm = torch.empty(A, dtype=torch.int32, device=dev)
        self.x_perm = torch.empty(A, H, dtype=self.dt, device=dev)
        self.o_perm = torch.empty(A, H, dtype=self.dt, device=dev)
        self.y = torch.empty(T, H, dtype=self.dt, device=dev)
        self.perm_ws_bytes = hmoe_permute_workspace_bytes(d, T)
        self.perm_ws = torch.empty(self.perm_ws_bytes, dtype=torch.uint8, device=dev)
        self.ffn_ws_bytes = hmoe_ffn_workspace_bytes(d, A)
        self.ffn_ws = torch.empty(max(self.ffn_ws_bytes, 256), dtype=torch.uint8, device=dev)
        self.h_counts = torch.zeros(E, dtype=torch.int32, pin_memory=True)
        self.sync_bytes = hmoe_ffn_combine_sync_bytes(d)
        self.sync = torch.zeros(self.sync_bytes, dtype=torch.uint8, device=dev)   # zeroed once; the calls leave it zero
        if self.shared_desc is not None:
            self.o_shared = torch.empty(T, H, dtype=self.dt, device=dev)
            self.shared_offsets = torch.zeros(2, dtype=torch.int32, device=dev)
            self.shared_ws_bytes = hmoe_ffn_workspace_bytes(self.shared_desc, T)
            self.shared_ws = torch.empty(max(self.shared_ws_bytes, 256), dtype=torch.uint8, device=dev)
            self._shared_T = -1

    def close(self):
        if getattr(self, "cache", None):
            torch.cuda.synchronize(self.dev)
            hmoe_cache_destroy(self.cache)
            self.cache = None
            if self.shared_desc is not None:
                hmoe_cache_destroy(self.shared_cache)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- the hot path --------------------------------------------------------------------
    def forward(self, x: torch.Tensor, logits: Optional[torch.Tensor] = None, path: int = HMOE_FFN_AUTO,
                all_resident: Optional[bool] = None) -> torch.Tensor:
        """x [T, H] on the device (layer dtype); logits [T, E] fp32 or None (then x . W_g).
        Returns y [T, H] (a view of an internal buffer, valid until the next call)."""
        d = self.desc
        T = int(x.shape[0])
        assert T <= self.max_tokens and x.dtype == self.dt and x.is_contiguous()
        K, E = d.top_k, d.n_experts
        A = T * K
        if all_resident is None:
            all_resident = d.n_slots == d.n_experts
        counts = None if all_resident else self.h_counts
        cur = torch.cuda.current_stream()
        o_shared = None
        # one call for routed and shared experts when the kernels are a few microseconds each (the library
        # merges the launches for T <= 32 in bfloat16) and the routed experts need a single call
        merged = (self.shared_desc is not None and self.fused and self.merge_shared and all_resident and T <= 32
                  and d.dtype == HMOE_BF16)
        if self.shared_desc is not None:
            # shared experts (Section II-A) see every token and do not depend on the routing: with
            # `fused` they run on a side stream next to the routed path
            if self._shared_T != T:
                self.shared_offsets.copy_(torch.tensor([0, T], dtype=torch.int32))
                self._shared_T = T
            o_shared = self.o_shared
            if self.overlap_shared and not merged:
                self.ev_fork.record(cur)
                self.side_stream.wait_event(self.ev_fork)
                with torch.cuda.stream(self.side_stream):
                    hmoe_expert_ffn_grouped(self.shared_desc, self.shared_cache, x, self.shared_offsets, T, None,
                                            self.o_shared, self.shared_ws, self.shared_ws_bytes, path)
                    self.ev_join.record(self.side_stream)
        if logits is None and self.fused:
            hmoe_router_route_permute(d, x, self.w_router, T, self.logits, self.topk_idx, self.topk_w, self.offsets,
                                      self.perm, self.inv_perm, counts, self.perm_ws, self.perm_ws_bytes)
            logits = self.logits
        elif logits is None:
            hmoe_router_logits(d, x, self.w_router, T, self.logits)
            logits = self.logits
            hmoe_route(d, logits, T, self.topk_idx, self.topk_w)
            hmoe_permute(d, self.topk_idx, T, x, self.x_perm, self.offsets, self.perm, self.inv_perm, counts,
                         self.perm_ws, self.perm_ws_bytes)
        elif self.fused:
            hmoe_route_permute(d, logits, T, self.topk_idx, self.topk_w, self.offsets, self.perm, self.inv_perm, counts,
                               self.perm_ws, self.perm_ws_bytes)
        else:
            hmoe_route(d, logits, T, self.topk_idx, self.topk_w)
            hmoe_permute(d, self.topk_idx, T, x, self.x_perm, self.offsets, self.perm, self.inv_perm, counts,
                         self.perm_ws, self.perm_ws_bytes)

        def routed_ffn(active):
            if self.fused:
                hmoe_expert_ffn_grouped_gather(d, self.cache, x, self.perm, self.offsets, A, active, self.o_perm,
                                               self.ffn_ws, self.ffn_ws_bytes, path)
            else:
                hmoe_expert_ffn_grouped(d, self.cache, self.x_perm, self.offsets, A, active, self.o_perm, self.ffn_ws,
                                        self.ffn_ws_bytes, path)

        # decode-sized batches with every expert resident: FFN (routed and shared) and the sum in two launches
        with_sum = (self.fused and self.merge_combine and all_resident and T <= 32 and d.dtype == HMOE_BF16 and d.n_slots == E
                    and path in (HMOE_FFN_AUTO, HMOE_FFN_SKINNY) and (self.shared_desc is None or merged))
        if with_sum:
            sd = self.shared_desc
            hmoe_expert_ffn_combine(d, self.cache, x, self.perm, self.inv_perm, self.topk_w, self.offsets, T, self.o_perm,
                                    self.ffn_ws, self.ffn_ws_bytes, sd, None if sd is None else self.shared_cache,
                                    None if sd is None else self.shared_offsets, None if sd is None else self.o_shared,
                                    None if sd is None else self.shared_ws, 0 if sd is None else self.shared_ws_bytes,
                                    self.y, self.sync, self.sync_bytes, path)
            return self.y[:T]
        if merged:
            hmoe_expert_ffn_grouped_with_shared(d, self.cache, x, self.perm, self.offsets, A, None, self.o_perm,
                                                self.ffn_ws, self.ffn_ws_bytes, self.shared_desc, self.shared_cache,
                                                self.shared_offsets, T, self.o_shared, self.shared_ws,
                                                self.shared_ws_bytes, path)
        elif all_resident:
            routed_ffn(None)
        else:
            # plan, staging of the missing experts and the FFN wave by wave, in one library call (it synchronises the
            # stream once: the host needs the per-expert loads)
            wave, slot, victim, n_waves, staged = hmoe_expert_ffn_staged(
                d, self.cache, x if self.fused else self.x_perm, self.perm if self.fused else None, self.offsets, A,
                self.h_counts, self.h_packed_ptrs, self.o_perm, self.ffn_ws, self.ffn_ws_bytes, path, None, self.copy_stream)
            self.last_plan = (wave, slot, victim, n_waves)
            self.staged_bytes += staged
        if self.shared_desc is not None and not merged:
            if self.overlap_shared:
                cur.wait_event(self.ev_join)
            else:
                hmoe_expert_ffn_grouped(self.shared_desc, self.shared_cache, x, self.shared_offsets, T, None,
                                        self.o_shared, self.shared_ws, self.shared_ws_bytes, path)
        hmoe_combine(d, self.o_perm, self.inv_perm, self.topk_w, o_shared, T, self.y)
        return self.y[:T]

    # -- score-aware replacement (Section IV-D) -------------------------------------------
    def set_policy(self, policy: int, alpha: float = 0.5):
        hmoe_cache_set_policy(self.cache, policy, alpha)

    def update_scores(self, logits: torch.Tensor, top_p: Optional[int] = None) -> np.ndarray:
        """One Eq. (3) update from this iteration's logits [T, E]; returns the routing scores used."""
        d = self.desc
        T = int(logits.shape[0])
        if not hasattr(self, "_scores_dev"):
            self._scores_dev = torch.empty(d.n_experts, dtype=torch.float32, device=self.dev)
            self._scores_host = torch.zeros(d.n_experts, dtype=torch.float32, pin_memory=True)
        ws_bytes = hmoe_route_scores_workspace_bytes(d, T)
        if getattr(self, "_scores_ws", None) is None or self._scores_ws.numel() < ws_bytes:
            self._scores_ws = torch.empty(ws_bytes, dtype=torch.uint8, device=self.dev)
        hmoe_route_scores(d, logits, T, self._scores_dev, self._scores_host, self._scores_ws, ws_bytes)
        torch.cuda.current_stream().synchronize()
        hmoe_cache_update_scores(self.cache, self._scores_host, 2 * d.top_k if top_p is None else top_p)
        return self._scores_host.numpy().copy()

    def slot_map(self) -> List[int]:
        return [hmoe_cache_lookup(self.cache, e) for e in range(self.desc.n_experts)]
