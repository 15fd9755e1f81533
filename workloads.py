"""Seeded synthetic inputs for the MoE-layer hot path.

This module holds no arithmetic of the method (no routing, no FFN, no combine):
it only draws random tensors of the stated shapes and distributions and rounds
them to the storage dtype.  Both the CPU oracle's tests and the HIP path's
tests / benchmark take their inputs from here, so the two sides see the same
bits.  Neither the oracle nor the HIP binding imports it.

Storage convention
------------------
* fp32 workloads: ``numpy.float32`` arrays.
* bf16 workloads: ``numpy.uint16`` arrays holding the bf16 bit pattern
  (round-to-nearest-even of the fp32 draw).  ``as_f32`` / ``as_f64`` decode
  either storage form to real numbers for the oracle.

Random streams: ``numpy.random.Generator(Philox(key=seed))``; every tensor gets
its own sub-stream ``Philox(key=seed).jumped(i)`` with a fixed index ``i`` so a
tensor's bits do not depend on which other tensors were drawn.
"""
from __future__ import annotations

import dataclasses
from concurrent.futures import ThreadPoolExecutor
from typing import List, Optional

import numpy as np

F32 = "f32"
BF16 = "bf16"

# sub-stream indices (fixed order: x, router, logits noise, then experts, shared)
_STREAM_X = 0
_STREAM_WG = 1
_STREAM_LOGITS = 2
_STREAM_EXPERT0 = 16          # expert e uses 16 + 3e .. 16 + 3e + 2
_STREAM_SHARED0 = 16 + 3 * 4096


@dataclasses.dataclass(frozen=True)
class LayerShape:
    """Shape of one MoE layer workload (names follow the layer equation:
    N experts -> ``n_experts``, K activated -> ``top_k``)."""
    name: str
    dtype: str                 # F32 or BF16
    hidden: int                # H
    ffn: int                   # F, routed expert FFN dim
    n_experts: int             # E
    top_k: int                 # k
    n_slots: int               # S, experts the HBM cache holds
    shared_ffn: tuple = ()     # FFN dim of each always-on shared expert
    logits_mode: str = "router"  # "router" | "zipf" | "hot0"
    weight_std: float = 0.02
    x_mode: str = "normal"     # "normal" (N(0, x_std^2)) | "rmsnorm"
    x_std: float = 0.02
    router_std: Optional[float] = None   # None -> weight_std


# The five workload shapes.  Token counts are chosen by the caller.
TOY = LayerShape("toy", F32, 256, 512, 8, 2, 8, (), "router",
                 weight_std=0.02, x_mode="normal", x_std=0.02, router_std=1.0 / 16.0)
MIXTRAL = LayerShape("mixtral", BF16, 4096, 14336, 8, 2, 4, (), "router",
                     x_mode="rmsnorm")
DSV2LITE = LayerShape("dsv2lite", BF16, 2048, 1408, 64, 6, 32, (1408, 1408), "zipf",
                      x_mode="rmsnorm")
QWEN2MOE = LayerShape("qwen2moe", BF16, 3584, 2560, 64, 8, 48, (20480,), "hot0",
                      x_mode="rmsnorm")
STRESS = LayerShape("stress", BF16, 2048, 1408, 64, 6, 64, (1408, 1408), "router",
                    x_mode="rmsnorm", router_std=1.0 / np.sqrt(2048.0))

SHAPES = {s.name: s for s in (TOY, MIXTRAL, DSV2LITE, QWEN2MOE, STRESS)}


# ---------------------------------------------------------------------------
# storage helpers (format conversion only)
# ---------------------------------------------------------------------------
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest, ties to even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def as_f32(a: np.ndarray) -> np.ndarray:
    """Decode a stored tensor (fp32 array or bf16 bit patterns) to fp32 values."""
    if a.dtype == np.uint16:
        return bf16_bits_to_f32(a)
    return np.asarray(a, dtype=np.float32)


def as_f64(a: np.ndarray) -> np.ndarray:
    return as_f32(a).astype(np.float64)


def store(a_f32: np.ndarray, dtype: str) -> np.ndarray:
    """Round an fp32 draw to the storage dtype."""
    if dtype == BF16:
        return f32_to_bf16_bits(a_f32)
    return np.ascontiguousarray(a_f32, dtype=np.float32)


def _gen(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=seed).jumped(stream))


def _normal(seed: int, stream: int, shape, std: float) -> np.ndarray:
    a = _gen(seed, stream).standard_normal(size=shape, dtype=np.float32)
    a *= np.float32(std)
    return a


# ---------------------------------------------------------------------------
# tensors
# ---------------------------------------------------------------------------
def make_x(shape: LayerShape, seed: int, n_tokens: int) -> np.ndarray:
    """Token activations [T, H] in storage dtype."""
    if shape.x_mode == "rmsnorm":
        z = _normal(seed, _STREAM_X, (n_tokens, shape.hidden), 1.0)
        ms = np.mean(z.astype(np.float64) ** 2, axis=1, keepdims=True)
        z = (z / np.sqrt(ms + 1e-5)).astype(np.float32)
        return store(z, shape.dtype)
    return store(_normal(seed, _STREAM_X, (n_tokens, shape.hidden), shape.x_std), shape.dtype)


def make_router_weight(shape: LayerShape, seed: int) -> np.ndarray:
    """Router matrix W_g [E, H] in storage dtype."""
    std = shape.weight_std if shape.router_std is None else shape.router_std
    return store(_normal(seed, _STREAM_WG, (shape.n_experts, shape.hidden), std), shape.dtype)


def zipf_bias(n_experts: int, s: float = 1.1) -> np.ndarray:
    """Per-expert additive logit bias ln(E * p_e), p_e proportional to (e+1)^-s."""
    r = np.arange(1, n_experts + 1, dtype=np.float64)
    p = r ** (-s)
    p /= p.sum()
    return np.log(n_experts * p).astype(np.float32)


def make_logits(shape: LayerShape, seed: int, n_tokens: int) -> Optional[np.ndarray]:
    """fp32 router logits [T, E] for the workloads that draw them directly
    ("zipf": N(0,1) plus a Zipf(1.1) per-expert bias; "hot0": N(0,1) with every
    tenth token forced onto expert 0).  Returns None for "router" workloads,
    whose logits come from x and W_g."""
    if shape.logits_mode == "router":
        return None
    lg = _normal(seed, _STREAM_LOGITS, (n_tokens, shape.n_experts), 1.0)
    if shape.logits_mode == "zipf":
        lg = lg + zipf_bias(shape.n_experts)[None, :]
    elif shape.logits_mode == "hot0":
        hot = np.arange(n_tokens) % 10 == 0
        lg[hot, 0] = lg[hot].max(axis=1) + np.float32(1.0)
    else:
        raise ValueError(shape.logits_mode)
    return np.ascontiguousarray(lg, dtype=np.float32)


def make_logit_sequence(shape: LayerShape, seed: int, n_tokens: int, n_steps: int, rho: float = 0.9) -> np.ndarray:
    """fp32 router logits [n_steps, T, E] of consecutive decode steps with temporal locality: an AR(1)
    process per (token slot, expert), l_s = rho * l_(s-1) + sqrt(1 - rho^2) * N(0,1), started from N(0,1),
    plus the workload's per-expert bias ("zipf") or forcing ("hot0").  The stationary distribution per step is
    that of make_logits; rho = 0 gives independent steps.  Stands in for the step-to-step similarity of
    routing scores in real decoding traces, which is what a score-aware replacement policy exploits."""
    e = shape.n_experts
    noise = _normal(seed, _STREAM_LOGITS, (n_steps, n_tokens, e), 1.0)
    out = np.empty_like(noise)
    cur = noise[0]
    for s in range(n_steps):
        if s:
            cur = np.float32(rho) * cur + np.float32(np.sqrt(1.0 - rho * rho)) * noise[s]
        out[s] = cur
    if shape.logits_mode == "zipf":
        out = out + zipf_bias(e)[None, None, :]
    elif shape.logits_mode == "hot0":
        hot = np.arange(n_tokens) % 10 == 0
        out[:, hot, 0] = out[:, hot].max(axis=2) + np.float32(1.0)
    return np.ascontiguousarray(out, dtype=np.float32)


def make_expert(shape: LayerShape, seed: int, e: int, ffn: Optional[int] = None, shared: bool = False):
    """One expert's three matrices in logical form and storage dtype:
    W_gate [F, H], W_up [F, H], W_down [H, F]."""
    f = shape.ffn if ffn is None else ffn
    base = (_STREAM_SHARED0 if shared else _STREAM_EXPERT0) + 3 * e
    wg = store(_normal(seed, base + 0, (f, shape.hidden), shape.weight_std), shape.dtype)
    wu = store(_normal(seed, base + 1, (f, shape.hidden), shape.weight_std), shape.dtype)
    wd = store(_normal(seed, base + 2, (shape.hidden, f), shape.weight_std), shape.dtype)
    return wg, wu, wd


@dataclasses.dataclass
class LayerInputs:
    shape: LayerShape
    seed: int
    n_tokens: int
    x: np.ndarray                       # [T, H] storage dtype
    w_router: Optional[np.ndarray]      # [E, H] storage dtype, or None
    logits: Optional[np.ndarray]        # [T, E] fp32 when drawn directly, else None
    experts: List[tuple]                # E x (W_gate, W_up, W_down)
    shared: List[tuple]                 # per shared expert (W_gate, W_up, W_down)


def make_layer(shape: LayerShape, seed: int, n_tokens: int, *, with_weights: bool = True,
               threads: int = 8) -> LayerInputs:
    """Draw every tensor of one layer workload."""
    x = make_x(shape, seed, n_tokens)
    logits = make_logits(shape, seed, n_tokens)
    w_router = make_router_weight(shape, seed) if logits is None else None
    experts: List[tuple] = []
    shared: List[tuple] = []
    if with_weights:
        with ThreadPoolExecutor(max_workers=max(1, threads)) as pool:
            experts = list(pool.map(lambda e: make_expert(shape, seed, e), range(shape.n_experts)))
            shared = list(pool.map(lambda i: make_expert(shape, seed, i, shape.shared_ffn[i], True),
                                   range(len(shape.shared_ffn))))
    return LayerInputs(shape, seed, n_tokens, x, w_router, logits, experts, shared)


def small_shape(name: str = "tiny", dtype: str = F32, hidden: int = 64, ffn: int = 96,
                n_experts: int = 8, top_k: int = 2, n_slots: Optional[int] = None,
                shared_ffn: tuple = (), logits_mode: str = "router", x_mode: str = "normal",
                x_std: float = 1.0, weight_std: float = 0.1) -> LayerShape:
    """A reduced shape with O(1) activations, for tests that the oracle finishes in seconds."""
    return LayerShape(name, dtype, hidden, ffn, n_experts, top_k,
                      n_experts if n_slots is None else n_slots, tuple(shared_ffn), logits_mode,
                      weight_std=weight_std, x_mode=x_mode, x_std=x_std,
                      router_std=1.0 / np.sqrt(hidden))
