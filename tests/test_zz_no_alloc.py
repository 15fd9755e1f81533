"""hmoe_permute_static -- the permutation for callers that cannot allocate (it takes no workspace: its scratch
memory is a static device array inside the library) -- against hmoe_permute, bit for bit, through the C ABI:
two calls in a row on the same GPU, the second with a smaller input, so that what the first call left in the
shared array must not leak into the second; then the size limit."""
import sys

import numpy as np
import pytest
import torch

import workloads as wl
from oracle import moe_oracle as orc
from hmoe_testlib import to_device

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def hm():
    import paper_2504_05897_amd as hm
    return hm


def _run(hm, static, T, E, K, H, seed):
    """One permutation (+ row gather) through hmoe_permute_static or hmoe_permute; returns host copies."""
    rng = np.random.default_rng(seed)
    lg = rng.standard_normal((T, E)).astype(np.float32) + wl.zipf_bias(E)[None]
    idx, _ = orc.route(lg, K)
    A = T * K
    d = hm.make_desc(H, 64, E, K, E, hm.HMOE_BF16)
    xb = wl.f32_to_bf16_bits((rng.standard_normal((T, H)) * 4).astype(np.float32))
    xd, idx_d = to_device(xb), to_device(idx)
    offs = torch.full((E + 1,), -7, dtype=torch.int32, device=DEV)
    perm = torch.full((A,), -7, dtype=torch.int32, device=DEV)
    inv = torch.full((A,), -7, dtype=torch.int32, device=DEV)
    xp = torch.zeros(A, H, dtype=torch.bfloat16, device=DEV)
    counts = torch.full((E,), -1, dtype=torch.int32).pin_memory()
    if static:
        hm.hmoe_permute_static(d, idx_d, T, xd, xp, offs, perm, inv, counts)
    else:
        ws_bytes = hm.hmoe_permute_workspace_bytes(d, T)
        ws = torch.empty(ws_bytes, dtype=torch.uint8, device=DEV)
        hm.hmoe_permute(d, idx_d, T, xd, xp, offs, perm, inv, counts, ws, ws_bytes)
    torch.cuda.synchronize()
    return (idx, offs.cpu().numpy(), perm.cpu().numpy(), inv.cpu().numpy(), counts.numpy().copy(),
            xp.view(torch.int16).cpu().numpy())


# each case: a larger input first, then a smaller one, through the same static array
@pytest.mark.parametrize("first,second", [((16384, 64, 6), (171, 64, 6)), ((3000, 200, 5), (1000, 200, 5)),
                                          ((2048, 64, 8), (4, 64, 8)), ((300, 8, 2), (1, 8, 2))])
def test_permute_static_equals_permute_twice_in_a_row(hm, first, second):
    for n, (T, E, K) in enumerate((first, second)):
        print("permute_static", T, E, K, flush=True)
        sys.stdout.flush()
        got = _run(hm, True, T, E, K, 64, 100 + n)
        want = _run(hm, False, T, E, K, 64, 100 + n)
        for g, w, what in zip(got[1:], want[1:], ("offsets", "perm", "inv_perm", "counts", "x_perm")):
            assert np.array_equal(g, w), (what, T, E, K)
        ro, rp, ri = orc.permute(got[0], E)          # and the oracle's integers
        assert np.array_equal(got[1], ro) and np.array_equal(got[2], rp) and np.array_equal(got[3], ri)


def test_permute_static_rejects_what_does_not_fit(hm):
    d = hm.make_desc(64, 64, 256, 32, 256, hm.HMOE_BF16)
    T = 40000                                            # 1.28 M assignments x 256 experts: beyond the static array
    assert hm.hmoe_permute_workspace_bytes(d, T) > hm.HMOE_PERMUTE_STATIC_BYTES
    t = torch.zeros(8, dtype=torch.int32, device=DEV)
    with pytest.raises(hm.HmoeError) as ei:
        hm.hmoe_permute_static(d, t, T, None, None, t, t, t, None)
    assert ei.value.status == hm.HMOE_ERR_WORKSPACE and "HMOE_PERMUTE_STATIC_BYTES" in str(ei.value)
