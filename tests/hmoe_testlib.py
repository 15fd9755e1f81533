"""Helpers shared by the GPU parity tests: build a device layer from seeded inputs, run the HIP
path through the C ABI, and evaluate the oracle on the same bits."""
from __future__ import annotations

import numpy as np
import torch

import workloads as wl
from oracle import moe_oracle as orc

TOL = {wl.BF16: 2e-2, wl.F32: 1e-4}      # max|y - y_ref| / max|y_ref| per workload dtype


def desc_of(hm, shape: wl.LayerShape, n_slots=None):
    return hm.make_desc(shape.hidden, shape.ffn, shape.n_experts, shape.top_k,
                        shape.n_slots if n_slots is None else n_slots,
                        hm.HMOE_BF16 if shape.dtype == wl.BF16 else hm.HMOE_F32)


def to_device(a: np.ndarray, dev="cuda:0") -> torch.Tensor:
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).view(torch.bfloat16).to(dev)
    return torch.from_numpy(a).to(dev)


def to_host_f32(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float32).cpu().numpy()


def build_layer(hm, lay: wl.LayerInputs, max_tokens=None, n_slots=None):
    d = desc_of(hm, lay.shape, n_slots)
    return hm.MoELayer(d, lay.experts, lay.shared, lay.w_router,
                       max_tokens=lay.n_tokens if max_tokens is None else max_tokens)


def max_rel_err(y: np.ndarray, y_ref: np.ndarray) -> float:
    return float(np.abs(y.astype(np.float64) - y_ref).max() / np.abs(y_ref).max())


def oracle_layer(lay: wl.LayerInputs, logits: np.ndarray, token_subset=None) -> np.ndarray:
    return orc.moe_layer(wl.as_f64(lay.x), logits, lay.shape.top_k, lay.experts, lay.shared,
                         token_subset=token_subset, to_f64=wl.as_f64)
