"""4-bit expert weights (HMOE_BF16_W4) on the GPU: the weight-streaming decode kernel, the prefill tile kernel and
the reference kernel against the oracle, which evaluates the FFN with every weight replaced by the value its 4-bit code stands for."""
import sys

import numpy as np
import pytest
import torch

import workloads as wl
from oracle import moe_oracle as orc
from oracle import w4_oracle as w4
from hmoe_testlib import TOL, max_rel_err, to_device, to_host_f32

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def hm():
    import paper_2504_05897_amd as hm
    return hm


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def as_quantised(m):
    return w4.dequantize_w4(*w4.quantize_w4(wl.as_f32(m)))


@pytest.mark.parametrize("path", [1, 2, 3])
@pytest.mark.parametrize("hidden,ffn,counts", [
    (256, 128, [3, 0, 7, 1, 40, 0, 9, 2]),       # decode-sized groups and one of 40 rows (two passes of 32)
    (128, 384, [33, 1, 0, 0, 70, 5, 8, 32]),     # one scale group in gate/up, three in down; half-filled column tile in down
    (1024, 256, [0, 0, 0, 1, 0, 0, 0, 0]),       # as many scale groups as waves
    (2048, 128, [8, 9]),                         # more scale groups than waves: two per wave
    (640, 512, [130, 0, 64, 257]),               # several row tiles with ragged ends; 5 and 4 scale groups (not a multiple of the ring)
])
def test_ffn_w4_paths(hm, path, hidden, ffn, counts):
    say("ffn w4 path", path, hidden, ffn, counts)
    shape = wl.small_shape(dtype=wl.BF16, hidden=hidden, ffn=ffn, n_experts=len(counts), top_k=2)
    E = shape.n_experts
    lay = wl.make_layer(shape, hidden + path, n_tokens=1)
    d = hm.make_desc(hidden, ffn, E, 2, E, hm.HMOE_BF16_W4)
    offsets = np.zeros(E + 1, np.int32)
    offsets[1:] = np.cumsum(counts)
    A = int(offsets[-1])
    xp = wl.store(np.random.default_rng(5).standard_normal((A, hidden)).astype(np.float32), wl.BF16)
    layer = hm.MoELayer(d, lay.experts, (), None, max_tokens=A)
    o = torch.zeros(A, hidden, dtype=torch.bfloat16, device=DEV)
    ws_bytes = hm.hmoe_ffn_workspace_bytes(d, A)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=DEV)
    hm.hmoe_expert_ffn_grouped(d, layer.cache, to_device(xp), to_device(offsets), A, None, o, ws, ws_bytes, path)
    torch.cuda.synchronize()
    ref = np.zeros((A, hidden))
    for e in range(E):
        lo, hi = offsets[e], offsets[e + 1]
        if hi > lo:
            ref[lo:hi] = orc.expert_ffn(wl.as_f64(xp[lo:hi]), *(as_quantised(m) for m in lay.experts[e]))
    assert max_rel_err(to_host_f32(o), ref) < TOL[wl.BF16]
    assert np.abs(ref).max() > 1e-3
    layer.close()


@pytest.mark.parametrize("T", [1, 5, 40, 200])
def test_w4_layer_with_shared_experts_and_partial_cache(hm, T):
    say("w4 layer", T)
    shape = wl.small_shape(dtype=wl.BF16, hidden=256, ffn=128, n_experts=8, top_k=2, n_slots=5, shared_ffn=(128, 128),
                           x_mode="rmsnorm")
    lay = wl.make_layer(shape, 40 + T, T)
    d = hm.make_desc(256, 128, 8, 2, 5, hm.HMOE_BF16_W4)
    layer = hm.MoELayer(d, lay.experts, lay.shared, lay.w_router, max_tokens=T)
    y = layer.forward(to_device(lay.x))
    torch.cuda.synchronize()
    logits = layer.logits[:T].cpu().numpy()
    ref = orc.moe_layer(wl.as_f64(lay.x), logits, 2, lay.experts, lay.shared, to_f64=as_quantised)
    assert max_rel_err(to_host_f32(y), ref) < TOL[wl.BF16]
    layer.close()


@pytest.mark.parametrize("T", [1, 8, 512])
def test_mixtral_w4_full_size(hm, T):
    """The Mixtral-style shape at full size with 4-bit experts, all resident, as the benchmark runs it: the decode
    kernel (1 and 8 tokens) and the prefill tile kernel (512 tokens)."""
    say("mixtral w4", T)
    shape = wl.SHAPES["mixtral"]
    lay = wl.make_layer(shape, 1, T, threads=16)
    d = hm.make_desc(shape.hidden, shape.ffn, shape.n_experts, shape.top_k, shape.n_experts, hm.HMOE_BF16_W4)
    layer = hm.MoELayer(d, lay.experts, (), lay.w_router, max_tokens=T)
    y = layer.forward(to_device(lay.x))
    torch.cuda.synchronize()
    logits = layer.logits[:T].cpu().numpy()
    ridx, _ = orc.route(logits, shape.top_k)
    assert np.array_equal(layer.topk_idx[:T].cpu().numpy(), ridx)
    sub = np.arange(T) if T == 1 else np.array([0, T - 1])      # the oracle quantises every expert its tokens touch
    ref = orc.moe_layer(wl.as_f64(lay.x), logits, shape.top_k, lay.experts, (), token_subset=sub, to_f64=as_quantised)
    assert max_rel_err(to_host_f32(y)[sub], ref) < TOL[wl.BF16]
    layer.close()
