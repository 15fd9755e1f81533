"""CPU oracle for the MoE-layer forward over an expert cache.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
HIP path is checked against.  It shares no code with the HIP path and is
imported only by tests, the smoke check and the benchmark's CPU-baseline leg;
the product never routes through it.

What it computes (HybriMoE, Section II-A, Eq. (1)):

    y = sum_{i<N} Softmax(TopK(x . W_g))_i * E_i(x)

with N routed experts of which K are activated per token, plus the shared
experts of Section II-A that are active for every token.  Every dot product and
sum is accumulated in float64 from the already-rounded input values, so this
side is the more exact one in every comparison.

Readings where the paper is silent (each also listed in the design notes):
  * TopK ties: the lowest expert index wins; the K outputs are ordered by
    descending logit, ties by ascending index.
  * Softmax is taken over the K kept logits (Eq. (1) as written); non-selected
    experts have gate 0.
  * The expert FFN form is not given in the paper (Table II lists sizes only);
    the workload definition fixes it as a bias-free SwiGLU:
    E(x) = W_down (silu(W_gate x) * (W_up x)), silu(z) = z / (1 + exp(-z)).
  * Shared experts have weight exactly 1 and are added after the routed sum.
  * Token-to-expert permutation: stable sort of the flat assignments
    a = t*K + j by expert id.
  * Expert cache (Section I, Section IV-D context): S slots, LRU victim choice
    (the paper's comparator policy), deterministic tie-breaks, see ExpertCacheModel.

Pins (tests/test_oracle_*.py): brute-force dense evaluation of every expert
masked by the gate, stable full arg-sort for TopK, closed-form softmax values,
a hand-computed SwiGLU example, permutation invariants, hand-traced LRU
sequences.  No function here is "parity unpinned".
"""
from __future__ import annotations

import math
from typing import List, Optional, Sequence, Tuple

import numpy as np

f64 = np.float64


# ---------------------------------------------------------------------------
# Eq. (1), x . W_g
# ---------------------------------------------------------------------------
def router_logits(x: np.ndarray, w_g: np.ndarray) -> np.ndarray:
    """logits[t, e] = sum_h x[t, h] * W_g[e, h]; float64 accumulation, float32 result
    (the logits cross the library boundary as float32)."""
    return (np.asarray(x, f64) @ np.asarray(w_g, f64).T).astype(np.float32)


# ---------------------------------------------------------------------------
# Eq. (1), Softmax(TopK(.))
# ---------------------------------------------------------------------------
def route_f64(logits: np.ndarray, top_k: int) -> Tuple[np.ndarray, np.ndarray]:
    """TopK by repeated arg-max, then softmax over the K kept logits.

    logits: [T, E] float32, finite.  Returns (topk_idx [T, K] int32,
    topk_w [T, K] float64).  Arg-max takes the first (lowest-index) maximum.
    """
    lg = np.asarray(logits, dtype=np.float32)
    assert lg.ndim == 2 and np.all(np.isfinite(lg)), "logits must be finite"
    n_tokens, n_experts = lg.shape
    assert 1 <= top_k <= n_experts
    work = lg.astype(f64).copy()
    idx = np.empty((n_tokens, top_k), dtype=np.int32)
    val = np.empty((n_tokens, top_k), dtype=f64)
    rows = np.arange(n_tokens)
    for j in range(top_k):
        best = np.argmax(work, axis=1)          # first occurrence of the maximum
        idx[:, j] = best
        val[:, j] = work[rows, best]
        work[rows, best] = -np.inf
    z = np.exp(val - val[:, :1])                # val[:, 0] is the row maximum
    w = z / z.sum(axis=1, keepdims=True)
    return idx, w


def route(logits: np.ndarray, top_k: int) -> Tuple[np.ndarray, np.ndarray]:
    """route_f64 with the gate weights rounded to float32, the type in which they
    cross the library boundary."""
    idx, w = route_f64(logits, top_k)
    return idx, w.astype(np.float32)


# ---------------------------------------------------------------------------
# token-to-expert permutation
# ---------------------------------------------------------------------------
def permute(topk_idx: np.ndarray, n_experts: int):
    """Stable sort of the A = T*K assignments by expert id.

    Returns (expert_offsets [E+1], perm [A], inv_perm [A]), all int32:
    perm[p] = flat assignment index a = t*K + j that lands at sorted position p,
    inv_perm[a] = p, rows of expert e occupy [expert_offsets[e], expert_offsets[e+1]).
    """
    keys = np.asarray(topk_idx, dtype=np.int64).reshape(-1)
    assert keys.size == 0 or (keys.min() >= 0 and keys.max() < n_experts)
    perm = np.argsort(keys, kind="stable").astype(np.int32)
    inv_perm = np.empty_like(perm)
    inv_perm[perm] = np.arange(perm.size, dtype=np.int32)
    counts = np.bincount(keys, minlength=n_experts)
    offsets = np.zeros(n_experts + 1, dtype=np.int32)
    offsets[1:] = np.cumsum(counts)
    return offsets, perm, inv_perm


def gather_rows(x: np.ndarray, perm: np.ndarray, top_k: int) -> np.ndarray:
    """x_perm[p, :] = x[perm[p] // K, :]."""
    return np.asarray(x)[np.asarray(perm) // top_k]


# ---------------------------------------------------------------------------
# E_i(x): SwiGLU expert
# ---------------------------------------------------------------------------
def silu(z: np.ndarray) -> np.ndarray:
    return z / (1.0 + np.exp(-z))


def expert_ffn(x_rows: np.ndarray, w_gate: np.ndarray, w_up: np.ndarray, w_down: np.ndarray) -> np.ndarray:
    """Rows [M, H] through one expert: W_gate, W_up are [F, H]; W_down is [H, F].
    float64 throughout, no intermediate rounding."""
    xr = np.asarray(x_rows, f64)
    g = xr @ np.asarray(w_gate, f64).T
    u = xr @ np.asarray(w_up, f64).T
    h = silu(g) * u
    return h @ np.asarray(w_down, f64).T


# ---------------------------------------------------------------------------
# the whole layer, in the order of the hot path
# ---------------------------------------------------------------------------
def moe_layer(x: np.ndarray, logits: np.ndarray, top_k: int, experts: Sequence, shared: Sequence = (),
              token_subset: Optional[np.ndarray] = None, to_f64=None) -> np.ndarray:
    """route -> permute -> per-expert FFN on the permuted rows -> weighted combine
    (+ shared experts).  `experts[e]` / `shared[i]` are (W_gate, W_up, W_down);
    `to_f64` decodes a stored matrix to float64 (identity by default).
    `token_subset` restricts the evaluation to some tokens (tokens are
    independent in Eq. (1)); the result then has one row per listed token.
    Returns y in float64 (the caller rounds once to the output dtype).
    """
    dec = (lambda a: np.asarray(a, f64)) if to_f64 is None else to_f64
    xs = np.asarray(x, f64)
    lg = np.asarray(logits, np.float32)
    if token_subset is not None:
        xs = xs[token_subset]
        lg = lg[token_subset]
    n_tokens, hidden = xs.shape
    n_experts = lg.shape[1]
    idx, w = route_f64(lg, top_k)
    offsets, perm, inv_perm = permute(idx, n_experts)
    x_perm = gather_rows(xs, perm, top_k)
    o_perm = np.zeros((n_tokens * top_k, hidden), dtype=f64)
    for e in range(n_experts):
        lo, hi = int(offsets[e]), int(offsets[e + 1])
        if hi > lo:
            wg, wu, wd = experts[e]
            o_perm[lo:hi] = expert_ffn(x_perm[lo:hi], dec(wg), dec(wu), dec(wd))
    y = np.zeros((n_tokens, hidden), dtype=f64)
    for j in range(top_k):                       # fixed order j = 0..K-1
        y += w[:, j][:, None] * o_perm[inv_perm[np.arange(n_tokens) * top_k + j]]
    for (wg, wu, wd) in shared:                  # shared experts: weight 1, all tokens
        y += expert_ffn(xs, dec(wg), dec(wu), dec(wd))
    return y


def dense_masked(x: np.ndarray, logits: np.ndarray, top_k: int, experts: Sequence,
                 shared: Sequence = ()) -> np.ndarray:
    """Brute force of Eq. (1): every expert evaluated for every token, scaled by a
    dense gate matrix G[t, e] that is zero outside the token's K selected experts.
    Written with scalar loops and without the permutation so that it shares no
    structure with moe_layer; only for tiny inputs."""
    xs = np.asarray(x, f64)
    lg = np.asarray(logits, np.float32)
    n_tokens, hidden = xs.shape
    n_experts = lg.shape[1]
    # gate matrix from a full stable arg-sort (value descending, index ascending)
    gate = [[0.0] * n_experts for _ in range(n_tokens)]
    for t in range(n_tokens):
        order = sorted(range(n_experts), key=lambda e: (-float(lg[t, e]), e))[:top_k]
        m = max(float(lg[t, e]) for e in order)
        den = sum(math.exp(float(lg[t, e]) - m) for e in order)
        for e in order:
            gate[t][e] = math.exp(float(lg[t, e]) - m) / den
    y = np.zeros((n_tokens, hidden), dtype=f64)

    def one_expert(vec, mats):
        w_gate, w_up, w_down = (np.asarray(a, f64) for a in mats)
        ffn = w_gate.shape[0]
        hvec = np.zeros(ffn, dtype=f64)
        for f in range(ffn):
            g = float(np.dot(w_gate[f], vec))
            u = float(np.dot(w_up[f], vec))
            hvec[f] = g / (1.0 + math.exp(-g)) * u
        return np.array([float(np.dot(w_down[r], hvec)) for r in range(w_down.shape[0])])

    for t in range(n_tokens):
        for e in range(n_experts):
            y[t] += gate[t][e] * one_expert(xs[t], experts[e])
        for mats in shared:
            y[t] += one_expert(xs[t], mats)
    return y


# ---------------------------------------------------------------------------
# expert cache state machine (host integers only)
# ---------------------------------------------------------------------------
class ExpertCacheModel:
    """S cache slots over E experts with least-recently-used replacement.

    The paper keeps a fixed fraction of the experts in GPU memory and loads the
    others on demand (Section I; cache ratios of Section V); LRU is the
    replacement policy it compares against (Section IV-D).  Rules, all
    deterministic so that slot maps can be compared exactly:

      * Initially expert i sits in slot i for i < S; every use tick is 0.
      * One call names the set of needed experts.  It is served in waves:
        wave 0 computes the needed experts that are resident.  Each missing
        expert, in ascending id, takes the lowest-numbered free slot, else the
        slot whose occupant has the smallest use tick (ties: lowest slot).  Its
        wave is 1 if the victim was not needed by this call (or the slot was
        free), else the victim's wave + 1.
      * Experts computed in wave w of a call get use tick base + w, where base
        is the value of the clock at the start of the call; the clock then
        advances past the last wave.  Needed residents are never chosen while
        an unneeded resident exists because their tick is already >= base.
    """

    def __init__(self, n_experts: int, n_slots: int):
        assert 1 <= n_slots <= n_experts
        self.n_experts, self.n_slots = n_experts, n_slots
        self.slot_of = [-1] * n_experts
        self.expert_in = [-1] * n_slots
        self.tick = [0] * n_experts
        self.clock = 1
        for i in range(n_slots):
            self.slot_of[i] = i
            self.expert_in[i] = i

    def serve(self, needed: Sequence[int]) -> List[Tuple[int, int, int, int]]:
        """Serve one call.  Returns the plan as a list of
        (expert, slot, wave, evicted_expert_or_-1), hits first (ascending id, wave 0,
        evicted = -1), then misses in ascending id."""
        need = sorted(set(int(e) for e in needed))
        base = self.clock
        wave = {}
        plan = []
        for e in need:
            if self.slot_of[e] >= 0:
                wave[e] = 0
                self.tick[e] = base
                plan.append((e, self.slot_of[e], 0, -1))
        misses = [e for e in need if e not in wave]
        for e in misses:
            free = [s for s in range(self.n_slots) if self.expert_in[s] < 0]
            if free:
                s, victim, w = free[0], -1, 1
            else:
                s = min(range(self.n_slots), key=lambda q: (self.tick[self.expert_in[q]], q))
                victim = self.expert_in[s]
                w = wave[victim] + 1 if victim in wave else 1
                self.slot_of[victim] = -1
            self.expert_in[s] = e
            self.slot_of[e] = s
            wave[e] = w
            self.tick[e] = base + w
            plan.append((e, s, w, victim))
        self.clock = base + (max(wave.values()) if wave else 0) + 1
        return plan

    def evict(self, expert: int) -> None:
        s = self.slot_of[expert]
        if s >= 0:
            self.slot_of[expert] = -1
            self.expert_in[s] = -1


# ---------------------------------------------------------------------------
# score-aware replacement (Section IV-D, Eq. (3))
# ---------------------------------------------------------------------------
def route_scores(logits: np.ndarray) -> np.ndarray:
    """Routing scores s of one iteration: the batch mean of the full softmax over all experts."""
    lg = np.asarray(logits, f64)
    z = np.exp(lg - lg.max(axis=1, keepdims=True))
    return (z / z.sum(axis=1, keepdims=True)).mean(axis=0)


def mrs_update(score: Sequence[float], s: Sequence[float], alpha: float, top_p: int) -> List[float]:
    """One step of Eq. (3), S <- alpha * TopP(s) + (1 - alpha) * S: only the top_p largest routing
    scores are accumulated (ties: lower id), the others count as zero."""
    n = len(s)
    keep = set(sorted(range(n), key=lambda e: (-float(s[e]), e))[:top_p])
    return [alpha * (float(s[e]) if e in keep else 0.0) + (1.0 - alpha) * float(score[e]) for e in range(n)]


class MRSCacheModel(ExpertCacheModel):
    """ExpertCacheModel with the Minus Recent Score victim choice: candidates are ordered by class
    (occupants this call does not need first, then by the wave in which they are computed), inside a
    class the lowest priority estimate S loses, ties -> lowest slot.  S starts at 0 and is updated once
    per iteration with `update` (the paper sets p to twice the number of activated experts)."""

    def __init__(self, n_experts: int, n_slots: int, alpha: float):
        super().__init__(n_experts, n_slots)
        self.alpha = alpha
        self.score = [0.0] * n_experts

    def update(self, s: Sequence[float], top_p: int) -> None:
        self.score = mrs_update(self.score, s, self.alpha, top_p)

    def serve(self, needed: Sequence[int]) -> List[Tuple[int, int, int, int]]:
        need = sorted(set(int(e) for e in needed))
        wave = {}
        plan = []
        for e in need:
            if self.slot_of[e] >= 0:
                wave[e] = 0
                plan.append((e, self.slot_of[e], 0, -1))
        for e in [x for x in need if x not in wave]:
            free = [s for s in range(self.n_slots) if self.expert_in[s] < 0]
            if free:
                s, victim, w = free[0], -1, 1
            else:
                def key(q):
                    occ = self.expert_in[q]
                    return (1 + wave[occ] if occ in wave else 0, self.score[occ], q)
                s = min(range(self.n_slots), key=key)
                victim = self.expert_in[s]
                w = wave[victim] + 1 if victim in wave else 1
                self.slot_of[victim] = -1
            self.expert_in[s] = e
            self.slot_of[e] = s
            wave[e] = w
            plan.append((e, s, w, victim))
        return plan
