"""Parity of the HIP path (through the C ABI) with the CPU oracle, step by step and end to end,
on seeded inputs small enough for the oracle yet spanning several tiles and a ragged tail.
Integer results (top-k ids, permutation, offsets, slot maps) must match bit for bit; floating
point within the stated tolerance."""
import sys

import ctypes

import numpy as np
import pytest
import torch

import workloads as wl
from oracle import moe_oracle as orc
from hmoe_testlib import TOL, build_layer, desc_of, max_rel_err, oracle_layer, to_device, to_host_f32

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def hm():
    import paper_2504_05897_amd as hm
    return hm


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


# ----------------------------------------------------------------------------------------- route
@pytest.mark.parametrize("T,E,K", [(16, 8, 2), (1, 8, 2), (1, 64, 6), (1000, 64, 8), (333, 60, 4), (77, 200, 9),
                                   (5, 5, 5), (4097, 16, 3), (64, 256, 32), (9, 1, 1)])
def test_route_bit_exact(hm, T, E, K):
    say("route", T, E, K)
    rng = np.random.default_rng(T * 1000 + E)
    lg = rng.standard_normal((T, E)).astype(np.float32)
    lg[::3] = np.round(lg[::3] * 2) / 2              # exact ties
    if T > 4:
        lg[1] = 0.0                                   # a whole row of ties
        lg[2, ::2] = -0.0
        lg[2, 1::2] = 0.0
    d = hm.make_desc(64, 64, E, K, E, hm.HMOE_BF16)
    idx = torch.empty(T, K, dtype=torch.int32, device=DEV)
    w = torch.empty(T, K, dtype=torch.float32, device=DEV)
    hm.hmoe_route(d, to_device(lg), T, idx, w)
    ridx, rw = orc.route(lg, K)
    assert np.array_equal(idx.cpu().numpy(), ridx)
    np.testing.assert_allclose(w.cpu().numpy(), rw, rtol=2e-6, atol=1e-7)
    np.testing.assert_allclose(w.cpu().numpy().astype(np.float64).sum(axis=1), 1.0, atol=1e-6)


# ----------------------------------------------------------------------------------------- permute
@pytest.mark.parametrize("T,E,K", [(1, 8, 2), (16, 8, 2), (1, 64, 6), (4, 64, 8), (512, 8, 2), (171, 64, 6),
                                   (1024, 64, 1), (1025, 64, 1), (16384, 64, 6), (3000, 200, 5), (0, 8, 2),
                                   (2048, 64, 8), (32, 8, 2), (13, 64, 5), (2, 256, 32), (1, 256, 32), (64, 3, 1)])
def test_permute_bit_exact(hm, T, E, K):
    say("permute", T, E, K)
    rng = np.random.default_rng(T + 17 * E)
    if T:
        lg = rng.standard_normal((T, E)).astype(np.float32) + wl.zipf_bias(E)[None]
        idx, _ = orc.route(lg, K)
    else:
        idx = np.zeros((0, K), np.int32)
    H = 64
    d = hm.make_desc(H, 64, E, K, E, hm.HMOE_BF16)
    A = T * K
    x = (rng.standard_normal((T, H)) * 4).astype(np.float32)
    xb = wl.f32_to_bf16_bits(x)
    xd = to_device(xb) if T else torch.empty(0, H, dtype=torch.bfloat16, device=DEV)
    offs = torch.full((E + 1,), -7, dtype=torch.int32, device=DEV)
    perm = torch.full((max(A, 1),), -7, dtype=torch.int32, device=DEV)
    inv = torch.full((max(A, 1),), -7, dtype=torch.int32, device=DEV)
    xp = torch.zeros(max(A, 1), H, dtype=torch.bfloat16, device=DEV)
    counts = torch.zeros(E, dtype=torch.int32, pin_memory=True)
    ws_bytes = hm.hmoe_permute_workspace_bytes(d, T)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=DEV)
    for rep in range(2):                                  # twice: results must not depend on scheduling
        hm.hmoe_permute(d, to_device(idx) if T else None, T, xd if T else None, xp if T else None, offs, perm, inv,
                        counts, ws, ws_bytes)
        torch.cuda.synchronize()
        ro, rp, ri = orc.permute(idx, E)
        assert np.array_equal(offs.cpu().numpy(), ro)
        assert np.array_equal(perm.cpu().numpy()[:A], rp)
        assert np.array_equal(inv.cpu().numpy()[:A], ri)
        assert np.array_equal(counts.numpy(), np.diff(ro))
        if T:
            got = xp.view(torch.int16).cpu().numpy().view(np.uint16)[:A]
            assert np.array_equal(got, orc.gather_rows(xb, rp, K))


def test_permute_workspace_too_small(hm):
    d = hm.make_desc(64, 64, 8, 2, 8, hm.HMOE_BF16)
    t = torch.zeros(64, dtype=torch.int32, device=DEV)
    with pytest.raises(hm.HmoeError) as ei:
        hm.hmoe_permute(d, t, 4, None, None, t, t, t, None, t, 8)
    assert ei.value.status == hm.HMOE_ERR_WORKSPACE


# ----------------------------------------------------------------------------------------- combine
@pytest.mark.parametrize("dtype", [wl.BF16, wl.F32])
@pytest.mark.parametrize("T,K,H,shared", [(7, 2, 256, False), (33, 6, 2048, True), (1, 8, 3584, True)])
def test_combine(hm, dtype, T, K, H, shared):
    say("combine", dtype, T, K, H, shared)
    rng = np.random.default_rng(T + K)
    A = T * K
    o = wl.store(rng.standard_normal((A, H)).astype(np.float32), dtype)
    osh = wl.store(rng.standard_normal((T, H)).astype(np.float32), dtype)
    w = rng.random((T, K)).astype(np.float32)
    inv = rng.permutation(A).astype(np.int32)
    d = hm.make_desc(H, 64, 64, K, 64, hm.HMOE_BF16 if dtype == wl.BF16 else hm.HMOE_F32)
    y = torch.empty(T, H, dtype=torch.bfloat16 if dtype == wl.BF16 else torch.float32, device=DEV)
    hm.hmoe_combine(d, to_device(o), to_device(inv), to_device(w), to_device(osh) if shared else None, T, y)
    ref = np.zeros((T, H))
    of = wl.as_f64(o)
    for t in range(T):
        for j in range(K):
            ref[t] += float(w[t, j]) * of[inv[t * K + j]]
        if shared:
            ref[t] += wl.as_f64(osh)[t]
    assert max_rel_err(to_host_f32(y), ref) < (1e-2 if dtype == wl.BF16 else 1e-6)


# ----------------------------------------------------------------------------------------- router logits
@pytest.mark.parametrize("name,T", [("toy", 16), ("dsv2lite", 50)])
def test_router_logits(hm, name, T):
    say("router_logits", name, T)
    shape = wl.SHAPES[name]
    x = wl.make_x(shape, 3, T)
    wg = wl.store(np.random.default_rng(1).standard_normal((shape.n_experts, shape.hidden)).astype(np.float32) * 0.05,
                  shape.dtype)
    d = desc_of(hm, shape)
    lg = torch.empty(T, shape.n_experts, dtype=torch.float32, device=DEV)
    hm.hmoe_router_logits(d, to_device(x), to_device(wg), T, lg)
    ref = orc.router_logits(wl.as_f64(x), wl.as_f64(wg))
    assert np.abs(lg.cpu().numpy() - ref).max() <= 1e-5 * np.abs(ref).max()


@pytest.mark.parametrize("E,H", [(8, 4096), (60, 128), (64, 2048), (100, 3584), (256, 64)])
def test_router_logits_decode_batches(hm, E, H):
    """T <= 8 takes the one-block kernel: against the oracle, and the same bits as the many-token kernel
    gives for the same rows."""
    say("router_logits small", E, H)
    rng = np.random.default_rng(E + H)
    x = wl.store(rng.standard_normal((40, H)).astype(np.float32), wl.BF16)
    wg = wl.store(rng.standard_normal((E, H)).astype(np.float32) * 0.05, wl.BF16)
    d = hm.make_desc(H, 64, E, 1, E, hm.HMOE_BF16)
    xd, wd = to_device(x), to_device(wg)
    big = torch.empty(40, E, dtype=torch.float32, device=DEV)
    hm.hmoe_router_logits(d, xd, wd, 40, big)
    ref = orc.router_logits(wl.as_f64(x), wl.as_f64(wg))
    assert np.abs(big.cpu().numpy() - ref).max() <= 1e-5 * np.abs(ref).max()
    for T in (1, 3, 8):
        small = torch.full((T, E), 99.0, dtype=torch.float32, device=DEV)
        hm.hmoe_router_logits(d, xd, wd, T, small)
        assert np.array_equal(small.cpu().numpy(), big.cpu().numpy()[:T])


# ----------------------------------------------------------------------------------------- FFN paths
def _ffn_case(hm, shape, counts, path, seed=0):
    """Grouped FFN over hand-made ragged row groups, every kernel path, against the oracle."""
    E = shape.n_experts
    lay = wl.make_layer(shape, seed, n_tokens=1)
    d = desc_of(hm, shape, n_slots=E)
    offsets = np.zeros(E + 1, np.int32)
    offsets[1:] = np.cumsum(counts)
    A = int(offsets[-1])
    rng = np.random.default_rng(seed + 5)
    xp = wl.store(rng.standard_normal((A, shape.hidden)).astype(np.float32), shape.dtype)
    layer = hm.MoELayer(d, lay.experts, (), None, max_tokens=max(1, (A + shape.top_k - 1) // shape.top_k + 1))
    o = torch.zeros(A, shape.hidden, dtype=layer.dt, device=DEV)
    ws_bytes = hm.hmoe_ffn_workspace_bytes(d, A)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=DEV)
    hm.hmoe_expert_ffn_grouped(d, layer.cache, to_device(xp), to_device(offsets), A, None, o, ws, ws_bytes, path)
    torch.cuda.synchronize()
    got = to_host_f32(o)
    ref = np.zeros((A, shape.hidden))
    for e in range(E):
        lo, hi = offsets[e], offsets[e + 1]
        if hi > lo:
            ref[lo:hi] = orc.expert_ffn(wl.as_f64(xp[lo:hi]), *(wl.as_f64(m) for m in lay.experts[e]))
    layer.close()
    return got, ref


def test_ffn_reference_fp32(hm):
    say("ffn reference fp32")
    shape = wl.small_shape(dtype=wl.F32, hidden=72, ffn=100, n_experts=5, top_k=2)
    got, ref = _ffn_case(hm, shape, [3, 0, 7, 1, 4], 1)
    assert max_rel_err(got, ref) < 1e-5


@pytest.mark.parametrize("path", [1, 2, 3])
@pytest.mark.parametrize("hidden,ffn,counts", [
    (128, 192, [3, 0, 7, 1, 40, 0, 9, 2]),
    (256, 64, [33, 1, 0, 0, 300, 5, 64, 129]),
    (64, 320, [0, 0, 0, 1, 0, 0, 0, 0]),
])
def test_ffn_bf16_paths(hm, path, hidden, ffn, counts):
    say("ffn bf16 path", path, hidden, ffn, counts)
    shape = wl.small_shape(dtype=wl.BF16, hidden=hidden, ffn=ffn, n_experts=len(counts), top_k=2)
    got, ref = _ffn_case(hm, shape, counts, path, seed=hidden + path)
    assert max_rel_err(got, ref) < TOL[wl.BF16]
    assert np.abs(ref).max() > 1e-2


@pytest.mark.parametrize("variant", range(10))
def test_ffn_every_prefill_tile_shape(hm, variant, monkeypatch):
    """The library's tuning override selects each built-in prefill kernel in turn (0-1 weight-streaming tiles of
    128x512 with 8 waves, 2-3 of 128x256 with 4 waves, both with the height fitted to the expert; 4-5 tiles of up
    to 256 rows with one 32-row weight group per wave, whose gate and up halves meet through LDS; the pairs differ
    in non-temporal vs plain weight loads).  Ragged groups spanning several m-tiles, partial n-tiles for every tile
    width, and m-tiles of every height the fitted tiles come in (1-4 fragments of 32 rows; 2, 4, 6 and 8 for the
    256-row tiles), alone and several per expert."""
    say("ffn prefill variant", variant)
    monkeypatch.setenv("HMOE_TILED_VARIANT", str(variant))
    shape = wl.small_shape(dtype=wl.BF16, hidden=256, ffn=320, n_experts=8, top_k=2)
    got, ref = _ffn_case(hm, shape, [33, 1, 0, 0, 300, 5, 64, 129], 3, seed=variant)
    assert max_rel_err(got, ref) < TOL[wl.BF16]
    shape = wl.small_shape(dtype=wl.BF16, hidden=192, ffn=320, n_experts=8, top_k=2)
    got, ref = _ffn_case(hm, shape, [257, 97, 96, 260, 1, 31, 32, 400], 3, seed=variant)
    assert max_rel_err(got, ref) < TOL[wl.BF16]
    for hidden, ffn in ((128, 384), (384, 128), (512, 512)):
        say("ffn prefill variant", variant, "hidden", hidden, "ffn", ffn)
        shape = wl.small_shape(dtype=wl.BF16, hidden=hidden, ffn=ffn, n_experts=4, top_k=2)
        got, ref = _ffn_case(hm, shape, [130, 0, 7, 128], 3, seed=variant + hidden)
        assert max_rel_err(got, ref) < TOL[wl.BF16]


def test_cache_set_layer_checks_and_changes_no_result(hm):
    """hmoe_cache_set_layer: only a one-expert cache of the layer's hidden size and dtype takes it; a dense FFN over
    such a cache then chooses its prefill kernels as the routed layer does (here: the walking blocks, which the dense
    launch alone would not take) and gives the same bits."""
    say("cache set layer")
    routed = wl.small_shape(dtype=wl.BF16, hidden=128, ffn=1024, n_experts=32, top_k=8)
    dense = wl.small_shape(dtype=wl.BF16, hidden=128, ffn=256, n_experts=1, top_k=1)
    T = 5600   # routed: 44800 rows, 1400 per expert, (200 + 32) * 8 = 1856 tiles of 224 x 256 >= 7 * 256
    lay = wl.make_layer(dense, 3, n_tokens=1)
    d = desc_of(hm, dense, n_slots=1)
    rng = np.random.default_rng(11)
    x = wl.store(rng.standard_normal((T, dense.hidden)).astype(np.float32), dense.dtype)
    layer = hm.MoELayer(d, lay.experts, (), None, max_tokens=T + 1)
    offsets = to_device(np.array([0, T], np.int32))
    ws_bytes = hm.hmoe_ffn_workspace_bytes(d, T)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=DEV)
    outs = []
    for beside in (None, desc_of(hm, routed, n_slots=32), None):
        hm.hmoe_cache_set_layer(layer.cache, beside)
        o = torch.zeros(T, dense.hidden, dtype=layer.dt, device=DEV)
        hm.hmoe_expert_ffn_grouped(d, layer.cache, to_device(x), offsets, T, None, o, ws, ws_bytes, 3)
        torch.cuda.synchronize()
        outs.append(o.view(torch.int16).cpu().numpy().copy())
    assert (outs[0] == outs[1]).all() and (outs[0] == outs[2]).all()
    ref = orc.expert_ffn(wl.as_f64(x[:256]), *(wl.as_f64(m) for m in lay.experts[0]))
    assert max_rel_err(to_host_f32(o)[:256], ref) < TOL[wl.BF16]
    other = desc_of(hm, wl.small_shape(dtype=wl.BF16, hidden=256, ffn=1024, n_experts=32, top_k=8), n_slots=32)
    assert hm._lib.hmoe_cache_set_layer(layer.cache, ctypes.byref(other)) == hm.HMOE_ERR_INVALID_ARG   # another hidden size
    layer.close()
    two = wl.small_shape(dtype=wl.BF16, hidden=128, ffn=64, n_experts=2, top_k=1)
    lay2 = wl.make_layer(two, 4, n_tokens=1)
    layer2 = hm.MoELayer(desc_of(hm, two, n_slots=2), lay2.experts, (), None, max_tokens=4)
    assert hm._lib.hmoe_cache_set_layer(layer2.cache, ctypes.byref(desc_of(hm, routed, n_slots=32))) == hm.HMOE_ERR_INVALID_ARG
    layer2.close()


@pytest.mark.parametrize("blocks", [8, 24])
def test_ffn_blocks_that_walk_through_tiles(hm, blocks, monkeypatch):
    """The 224x256 tile in blocks that take several tiles each (variants 8 and 9, the choice for large routed
    launches): few blocks, so that every block walks through tiles of every height the tile comes in (4-7 fragments,
    experts below 97 rows padded to 4) in both directions (a higher next tile has its last rows copied after the K
    loop), of several experts and n-tiles; K ranges of 6, 8 and 10 steps (one to four turns of the K loop between the
    two steps that stand before it and the two that load the next tile; every rotation of the three activation stages
    from tile to tile); and K ranges the walking blocks do not take (an odd number of steps, fewer than 6), which go
    to the 4-wave tile."""
    say("ffn walking blocks", blocks)
    monkeypatch.setenv("HMOE_WALK_BLOCKS", str(blocks))
    counts = [225, 700, 31, 450, 0, 129, 224, 1, 600, 353, 161, 97, 900, 260, 0, 512]
    for variant, hidden, ffn in ((9, 384, 640), (8, 512, 384), (9, 640, 512), (9, 320, 192)):
        monkeypatch.setenv("HMOE_TILED_VARIANT", str(variant))
        shape = wl.small_shape(dtype=wl.BF16, hidden=hidden, ffn=ffn, n_experts=len(counts), top_k=2)
        got, ref = _ffn_case(hm, shape, counts, 3, seed=blocks + hidden)
        assert max_rel_err(got, ref) < TOL[wl.BF16]
        assert np.abs(ref).max() > 1e-3


def test_ffn_walking_blocks_equal_the_fitted_tiles_bit_for_bit(hm, monkeypatch):
    """Same k order, same arithmetic: the walking blocks (weights as the first operand of the matrix instruction, the
    accumulators transposed) give the bits of the 128-row tiles."""
    say("ffn walking blocks against fitted tiles")
    counts = [500, 33, 0, 224, 97, 1000, 7, 450]
    shape = wl.small_shape(dtype=wl.BF16, hidden=512, ffn=384, n_experts=len(counts), top_k=2)
    outs = []
    for variant in (9, 3, 8, 0):
        monkeypatch.setenv("HMOE_TILED_VARIANT", str(variant))
        got, ref = _ffn_case(hm, shape, counts, 3, seed=5)
        assert max_rel_err(got, ref) < TOL[wl.BF16]
        outs.append(np.ascontiguousarray(got).view(np.uint32).copy())
    assert all((o == outs[0]).all() for o in outs[1:])


@pytest.mark.parametrize("hidden,ffn,counts", [
    (256, 512, [64]),                        # one small dense expert, few tiles: 256-row tiles for both projections
    (256, 512, [300]),                       # one large expert: 4-wave tiles, plain loads
    (256, 512, [20] * 32 + [0, 45] * 16),    # many small experts, short K: 4-wave gate/up, 256-row down
    (128, 4096, [200, 390, 1, 250]),         # large experts, long K in the down projection: 4-wave tiles for both
    (1536, 256, [100] * 60 + [0, 399, 1, 7]),  # 128x512 tiles, non-temporal loads, for both
    (1024, 128, [200] * 63 + [333]),         # large experts, short K, many tiles: 4-wave gate/up, 128x512 down, plain loads
    (2048, 128, [1200, 1400] * 17),          # seven rounds of 224x256 tiles in the down projection: walking blocks there
    (128, 1024, [1300, 1250] * 17),          # ... and in gate/up
])
def test_ffn_prefill_choice_branches(hm, hidden, ffn, counts):
    """The prefill path without a tuning override, on launches built to take each branch of the library's kernel
    choice (tile-starved or not, experts below or above 192 rows on average, short or long K range)."""
    say("ffn prefill choice", hidden, ffn, len(counts), sum(counts))
    shape = wl.small_shape(dtype=wl.BF16, hidden=hidden, ffn=ffn, n_experts=len(counts), top_k=1)
    got, ref = _ffn_case(hm, shape, counts, 3, seed=hidden + len(counts))
    assert max_rel_err(got, ref) < TOL[wl.BF16]
    assert np.abs(ref).max() > 1e-3


@pytest.mark.parametrize("shape_id", range(6))
@pytest.mark.parametrize("gpb", [1, 2, 3])
def test_ffn_every_decode_block_shape(hm, shape_id, gpb, monkeypatch):
    """Every (waves, unroll) block shape of the decode kernel and 1-3 row groups per block, on groups of
    at most 8 rows and of more than 8 rows."""
    say("ffn decode shape", shape_id, gpb)
    monkeypatch.setenv("HMOE_SKINNY", "%d,%d" % (shape_id, gpb))
    shape = wl.small_shape(dtype=wl.BF16, hidden=256, ffn=192, n_experts=6, top_k=2)
    for counts in ([2, 0, 8, 1, 0, 3], [9, 0, 32, 1, 17, 0]):
        got, ref = _ffn_case(hm, shape, counts, 2, seed=shape_id * 4 + gpb)
        assert max_rel_err(got, ref) < TOL[wl.BF16]


def test_ffn_inactive_and_non_resident_rows_untouched(hm):
    say("ffn active list")
    shape = wl.small_shape(dtype=wl.BF16, hidden=64, ffn=64, n_experts=4, top_k=2, n_slots=2)
    lay = wl.make_layer(shape, 1, 1)
    d = desc_of(hm, shape)
    layer = hm.MoELayer(d, lay.experts, (), None, max_tokens=8)
    offsets = to_device(np.array([0, 2, 4, 6, 8], np.int32))
    xp = to_device(wl.store(np.random.default_rng(0).standard_normal((8, 64)).astype(np.float32), wl.BF16))
    ws_bytes = hm.hmoe_ffn_workspace_bytes(d, 8)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=DEV)
    for path in (1, 2, 3):
        o = torch.full((8, 64), 7.0, dtype=torch.bfloat16, device=DEV)
        hm.hmoe_expert_ffn_grouped(d, layer.cache, xp, offsets, 8, np.array([1], np.int32), o, ws, ws_bytes, path)
        got = to_host_f32(o)
        assert np.all(got[0:2] == 7.0) and np.all(got[4:8] == 7.0) and not np.any(got[2:4] == 7.0)
        o.fill_(7.0)
        hm.hmoe_expert_ffn_grouped(d, layer.cache, xp, offsets, 8, None, o, ws, ws_bytes, path)   # residents: 0, 1
        got = to_host_f32(o)
        assert np.all(got[4:8] == 7.0) and not np.any(got[0:4] == 7.0)
    with pytest.raises(hm.HmoeError) as ei:
        hm.hmoe_expert_ffn_grouped(d, layer.cache, xp, offsets, 8, np.array([3], np.int32), o, ws, ws_bytes, 1)
    assert ei.value.status == hm.HMOE_ERR_NOT_RESIDENT
    with pytest.raises(hm.HmoeError) as ei:
        hm.hmoe_expert_ffn_grouped(d, layer.cache, xp, offsets, 8, None, o, ws, 16, 1)
    assert ei.value.status == hm.HMOE_ERR_WORKSPACE
    layer.close()


# ----------------------------------------------------------------------------------------- whole layer, small
def _layer_case(hm, shape, seed, T, path=0):
    lay = wl.make_layer(shape, seed, T)
    layer = build_layer(hm, lay)
    x = to_device(lay.x)
    if lay.logits is None:
        y = layer.forward(x, None, path)
        logits = layer.logits[:T].cpu().numpy()
        ref_lg = orc.router_logits(wl.as_f64(lay.x), wl.as_f64(lay.w_router))
        assert np.abs(logits - ref_lg).max() <= (1e-5 if shape.dtype == wl.F32 else 1e-5) * np.abs(ref_lg).max() + 1e-30
    else:
        logits = lay.logits
        y = layer.forward(x, to_device(logits), path)
    torch.cuda.synchronize()
    ridx, rw = orc.route(logits, shape.top_k)
    ro, rp, ri = orc.permute(ridx, shape.n_experts)
    A = T * shape.top_k
    assert np.array_equal(layer.topk_idx[:T].cpu().numpy(), ridx)
    assert np.array_equal(layer.offsets.cpu().numpy(), ro)
    assert np.array_equal(layer.perm[:A].cpu().numpy(), rp)
    assert np.array_equal(layer.inv_perm[:A].cpu().numpy(), ri)
    y_ref = oracle_layer(lay, logits)
    err = max_rel_err(to_host_f32(y), y_ref)
    layer.close()
    return err


def test_toy_workload_fp32(hm):
    """Workload 1: 16 tokens, hidden 256, 8 experts, FFN 512, top-2, fp32, seed 0, all resident."""
    say("layer toy fp32")
    err = _layer_case(hm, wl.TOY, 0, 16)
    say("  err", err)
    assert err < TOL[wl.F32]


@pytest.mark.parametrize("path", [0, 1, 2, 3])
@pytest.mark.parametrize("T", [1, 5, 40, 300])
def test_small_bf16_layer_all_paths(hm, T, path):
    say("layer small bf16", T, path)
    shape = wl.small_shape(dtype=wl.BF16, hidden=128, ffn=192, n_experts=8, top_k=2, shared_ffn=(64, 64),
                           x_mode="rmsnorm")
    err = _layer_case(hm, shape, 7 + T, T, path)
    say("  err", err)
    assert err < TOL[wl.BF16]


def test_small_layer_with_drawn_logits_and_many_experts(hm):
    say("layer small zipf 64 experts")
    shape = wl.small_shape(dtype=wl.BF16, hidden=64, ffn=128, n_experts=64, top_k=6, shared_ffn=(64,),
                           logits_mode="zipf", x_mode="rmsnorm")
    for T in (1, 700):
        err = _layer_case(hm, shape, 21, T)
        say("  T", T, "err", err)
        assert err < TOL[wl.BF16]


@pytest.mark.parametrize("top_k", [1, 3, 5, 6, 7])
def test_layer_through_walking_blocks_with_the_gather_in_gate_up(hm, top_k, monkeypatch):
    """The whole layer with both projections in walking blocks: the gather folded into gate/up finds the token of a
    sorted row as perm / top_k, which those blocks compute by multiplication with a constant made on the host --
    here for divisors that are and are not powers of two."""
    say("layer through walking blocks, top_k", top_k)
    monkeypatch.setenv("HMOE_TILED_VARIANT", "9")
    monkeypatch.setenv("HMOE_WALK_BLOCKS", "16")
    shape = wl.small_shape(dtype=wl.BF16, hidden=384, ffn=384, n_experts=8, top_k=top_k, shared_ffn=(128,),
                           x_mode="rmsnorm")
    err = _layer_case(hm, shape, 40 + top_k, 900, 3)
    say("  err", err)
    assert err < TOL[wl.BF16]


# ----------------------------------------------------------------------------------------- cache
def test_cache_slot_maps_and_outputs_follow_the_oracle_over_decode_steps(hm):
    """Partial cache (4 slots, 8 experts): over a sequence of calls the slot map must equal the
    oracle's LRU state machine after every call, and outputs must still match (staged weights are
    the right ones, waves cover every needed expert)."""
    say("cache sequence")
    shape = wl.small_shape(dtype=wl.BF16, hidden=64, ffn=64, n_experts=8, top_k=2, n_slots=4, x_mode="rmsnorm")
    steps = [1, 1, 8, 1, 3, 8, 1, 1, 2, 8]
    lay0 = wl.make_layer(shape, 2, 8)
    layer = build_layer(hm, lay0, max_tokens=8)
    model = orc.ExpertCacheModel(8, 4)
    for i, T in enumerate(steps):
        lay = wl.make_layer(shape, 100 + i, T, with_weights=False)
        lay.experts = lay0.experts
        x = to_device(lay.x)
        hm.hmoe_router_logits(layer.desc, x, layer.w_router, T, layer.logits)
        logits = layer.logits[:T].cpu().numpy()
        y = layer.forward(x, layer.logits[:T].contiguous())
        torch.cuda.synchronize()
        ridx, _ = orc.route(logits, 2)
        plan = model.serve(np.unique(ridx).tolist())
        assert layer.slot_map() == model.slot_of, (i, plan)
        assert np.array_equal(layer.slot_of.cpu().numpy(), np.array(model.slot_of, np.int32))
        wave, slot, victim, n_waves = layer.last_plan
        for (e, s, w, v) in plan:
            assert wave[e] == w and slot[e] == s and victim[e] == v
        assert n_waves == 1 + max(p[2] for p in plan)
        lay.w_router = lay0.w_router
        err = max_rel_err(to_host_f32(y), oracle_layer(lay, logits))
        say("  step", i, "T", T, "waves", n_waves, "err", err)
        assert err < TOL[wl.BF16]
    layer.close()


def test_cache_evict_follows_the_oracle(hm):
    """hmoe_cache_evict between layer calls: host mirror, device table, the plans of the following calls (a freed
    slot is taken first, lowest first) and the outputs equal the oracle's cache model after every step."""
    say("cache evictions")
    shape = wl.small_shape(dtype=wl.BF16, hidden=64, ffn=64, n_experts=8, top_k=2, n_slots=4, x_mode="rmsnorm")
    lay0 = wl.make_layer(shape, 3, 8)
    layer = build_layer(hm, lay0, max_tokens=8)
    model = orc.ExpertCacheModel(8, 4)
    script = [("serve", 1), ("evict", 0), ("evict", 6), ("serve", 8), ("evict", 3), ("evict", 2), ("evict", 2), ("serve", 2),
              ("serve", 8), ("evict", 1), ("evict", 5), ("evict", 7), ("evict", 4), ("evict", 0), ("serve", 3), ("serve", 8)]
    for i, (what, arg) in enumerate(script):
        if what == "evict":
            hm.hmoe_cache_evict(layer.cache, arg)
            model.evict(arg)
            torch.cuda.synchronize()
        else:
            T = arg
            lay = wl.make_layer(shape, 500 + i, T, with_weights=False)
            lay.experts, lay.w_router = lay0.experts, lay0.w_router
            x = to_device(lay.x)
            hm.hmoe_router_logits(layer.desc, x, layer.w_router, T, layer.logits)
            logits = layer.logits[:T].cpu().numpy()
            y = layer.forward(x, layer.logits[:T].contiguous())
            torch.cuda.synchronize()
            ridx, _ = orc.route(logits, 2)
            plan = model.serve(np.unique(ridx).tolist())
            wave, slot, victim, n_waves = layer.last_plan
            for (e, s, w, v) in plan:
                assert wave[e] == w and slot[e] == s and victim[e] == v, (i, plan)
            err = max_rel_err(to_host_f32(y), oracle_layer(lay, logits))
            say("  step", i, "T", T, "waves", n_waves, "err", err)
            assert err < TOL[wl.BF16]
        assert layer.slot_map() == model.slot_of, (i, what, arg)
        assert np.array_equal(layer.slot_of.cpu().numpy(), np.array(model.slot_of, np.int32))
        assert [hm.hmoe_cache_occupant(layer.cache, s) for s in range(4)] == model.expert_in
    layer.close()


def test_cache_stage_errors_and_pinning(hm):
    say("cache errors")
    shape = wl.small_shape(dtype=wl.BF16, hidden=64, ffn=64, n_experts=4, top_k=2, n_slots=2)
    lay = wl.make_layer(shape, 1, 1)
    layer = build_layer(hm, lay, max_tokens=4)
    assert layer.slot_map() == [0, 1, -1, -1]
    with pytest.raises(hm.HmoeError) as ei:          # no free slot
        hm.hmoe_cache_stage(layer.cache, 2, -1, layer.h_packed[2], None, layer.copy_stream)
    assert ei.value.status == hm.HMOE_ERR_SLOT_BUSY
    hm.hmoe_cache_pin_slot(layer.cache, 0, True)
    with pytest.raises(hm.HmoeError) as ei:
        hm.hmoe_cache_stage(layer.cache, 2, 0, layer.h_packed[2], None, layer.copy_stream)
    assert ei.value.status == hm.HMOE_ERR_SLOT_BUSY
    hm.hmoe_cache_pin_slot(layer.cache, 0, False)
    hm.hmoe_cache_stage(layer.cache, 2, 0, layer.h_packed[2], None, layer.copy_stream)
    hm.hmoe_cache_evict(layer.cache, 1)
    torch.cuda.synchronize()
    assert layer.slot_map() == [-1, -1, 0, -1]
    assert layer.slot_of.cpu().tolist() == [-1, -1, 0, -1]
    assert hm.hmoe_cache_occupant(layer.cache, 0) == 2 and hm.hmoe_cache_occupant(layer.cache, 1) == -1
    hm.hmoe_cache_stage(layer.cache, 3, -1, layer.h_packed[3], None, layer.copy_stream)   # lowest free = 1
    torch.cuda.synchronize()
    assert layer.slot_map() == [-1, -1, 0, 1]
    # slot contents are the packed blobs
    got = layer.slots.cpu()
    sb = layer.slot_bytes
    assert torch.equal(got[:sb], layer.h_packed[2]) and torch.equal(got[sb:2 * sb], layer.h_packed[3])
    layer.close()


# ----------------------------------------------------------------------------------------- fused entry points
@pytest.mark.parametrize("T,E,K", [(1, 8, 2), (1, 64, 6), (4, 64, 8), (32, 64, 8), (64, 16, 16), (65, 16, 8), (128, 8, 8),
                                   (300, 64, 6), (0, 8, 2), (8, 256, 8), (2, 200, 9), (32, 8, 2), (11, 60, 6)])
def test_route_permute_fused_equals_the_two_calls(hm, T, E, K):
    """hmoe_route_permute (one launch for T <= 64 and T*K <= 1024) against the oracle, bit for bit."""
    say("route_permute", T, E, K)
    rng = np.random.default_rng(T + E + K)
    lg = rng.standard_normal((max(T, 1), E)).astype(np.float32)[:T]
    lg[::2] = np.round(lg[::2] * 2) / 2
    d = hm.make_desc(64, 64, E, K, E, hm.HMOE_BF16)
    A = T * K
    idx = torch.full((max(T, 1), K), -5, dtype=torch.int32, device=DEV)
    w = torch.zeros(max(T, 1), K, dtype=torch.float32, device=DEV)
    offs = torch.full((E + 1,), -7, dtype=torch.int32, device=DEV)
    perm = torch.full((max(A, 1),), -7, dtype=torch.int32, device=DEV)
    inv = torch.full((max(A, 1),), -7, dtype=torch.int32, device=DEV)
    counts = torch.zeros(E, dtype=torch.int32, pin_memory=True)
    ws_bytes = hm.hmoe_permute_workspace_bytes(d, T)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=DEV)
    hm.hmoe_route_permute(d, to_device(lg) if T else None, T, idx, w, offs, perm, inv, counts, ws, ws_bytes)
    torch.cuda.synchronize()
    ridx, rw = orc.route(lg, K) if T else (np.zeros((0, K), np.int32), np.zeros((0, K), np.float32))
    ro, rp, ri = orc.permute(ridx, E)
    assert np.array_equal(idx.cpu().numpy()[:T], ridx)
    np.testing.assert_allclose(w.cpu().numpy()[:T], rw, rtol=2e-6, atol=1e-7)
    assert np.array_equal(offs.cpu().numpy(), ro)
    assert np.array_equal(perm.cpu().numpy()[:A], rp) and np.array_equal(inv.cpu().numpy()[:A], ri)
    assert np.array_equal(counts.numpy(), np.diff(ro))


@pytest.mark.parametrize("T,E,K,H", [(1, 8, 2, 4096), (8, 8, 2, 256), (1, 64, 6, 2048), (4, 64, 8, 3584), (7, 60, 4, 128),
                                     (8, 128, 8, 64), (2, 200, 9, 192), (8, 256, 32, 64), (9, 64, 6, 128), (40, 8, 2, 64),
                                     (0, 8, 2, 64), (40, 128, 8, 64), (100, 256, 32, 64), (300, 200, 9, 192),
                                     (1024, 64, 6, 2048), (2048, 64, 8, 3584), (2049, 64, 8, 128)])
def test_front_end_fused_equals_the_separate_calls(hm, T, E, K, H):
    """hmoe_router_route_permute (one launch for bf16, T <= 8; the separate calls otherwise) writes the same
    bits as hmoe_router_logits + hmoe_route + hmoe_permute, and the integers the oracle derives from them."""
    say("router_route_permute", T, E, K, H)
    rng = np.random.default_rng(T + E + K + H)
    x = wl.store(rng.standard_normal((max(T, 1), H)).astype(np.float32), wl.BF16)
    wg = wl.store(rng.standard_normal((E, H)).astype(np.float32) * 0.05, wl.BF16)
    d = hm.make_desc(H, 64, E, K, E, hm.HMOE_BF16)
    A = T * K
    xd, wd = to_device(x), to_device(wg)
    ws_bytes = hm.hmoe_permute_workspace_bytes(d, T)
    ws = torch.empty(max(ws_bytes, 4), dtype=torch.uint8, device=DEV)

    def buffers():
        return dict(lg=torch.full((max(T, 1), E), 3.0, dtype=torch.float32, device=DEV),
                    idx=torch.full((max(T, 1), K), -5, dtype=torch.int32, device=DEV),
                    w=torch.zeros(max(T, 1), K, dtype=torch.float32, device=DEV),
                    offs=torch.full((E + 1,), -7, dtype=torch.int32, device=DEV),
                    perm=torch.full((max(A, 1),), -7, dtype=torch.int32, device=DEV),
                    inv=torch.full((max(A, 1),), -7, dtype=torch.int32, device=DEV),
                    counts=torch.zeros(E, dtype=torch.int32, pin_memory=True))
    f, u = buffers(), buffers()
    hm.hmoe_router_route_permute(d, xd, wd, T, f["lg"], f["idx"], f["w"], f["offs"], f["perm"], f["inv"], f["counts"],
                                 ws, ws_bytes)
    torch.cuda.synchronize()
    hm.hmoe_router_logits(d, xd, wd, T, u["lg"])
    hm.hmoe_route(d, u["lg"], T, u["idx"], u["w"])
    hm.hmoe_permute(d, u["idx"], T, None, None, u["offs"], u["perm"], u["inv"], u["counts"], ws, ws_bytes)
    torch.cuda.synchronize()
    for k in f:
        assert torch.equal(f[k].cpu(), u[k].cpu()), k
    if T:
        lg = f["lg"].cpu().numpy()[:T]
        ridx, _ = orc.route(lg, K)
        ro, rp, ri = orc.permute(ridx, E)
        assert np.array_equal(f["idx"].cpu().numpy()[:T], ridx) and np.array_equal(f["offs"].cpu().numpy(), ro)
        assert np.array_equal(f["perm"].cpu().numpy()[:A], rp) and np.array_equal(f["inv"].cpu().numpy()[:A], ri)
        ref = orc.router_logits(wl.as_f64(x[:T]), wl.as_f64(wg))
        assert np.abs(lg - ref).max() <= 1e-5 * np.abs(ref).max()


@pytest.mark.parametrize("T", [3, 70])
def test_fused_and_unfused_layers_agree(hm, T):
    """The fused call sequence (route+permute in one call, gather inside the FFN, shared expert on a side
    stream) and the plain five-call sequence give the same integers and outputs."""
    say("fused vs unfused", T)
    shape = wl.small_shape(dtype=wl.BF16, hidden=128, ffn=192, n_experts=8, top_k=2, shared_ffn=(64,), x_mode="rmsnorm")
    lay = wl.make_layer(shape, 31, T)
    d = desc_of(hm, shape)
    outs = []
    for fused in (True, False):
        layer = hm.MoELayer(d, lay.experts, lay.shared, lay.w_router, max_tokens=T, fused=fused)
        y = layer.forward(to_device(lay.x))
        torch.cuda.synchronize()
        outs.append((to_host_f32(y).copy(), layer.perm[:T * 2].cpu().numpy().copy(), layer.offsets.cpu().numpy().copy()))
        layer.close()
    assert np.array_equal(outs[0][1], outs[1][1]) and np.array_equal(outs[0][2], outs[1][2])
    assert np.array_equal(outs[0][0], outs[1][0])      # same kernels on the same rows: bit-identical outputs


@pytest.mark.parametrize("fused_sum", [False, True])
@pytest.mark.parametrize("T,shared_ffn,logits_mode", [(4, (), "router"), (2, (64,), "zipf"), (70, (64,), "zipf"),
                                                      (200, (), "router")])
def test_graph_replay_equals_eager(hm, T, shared_ffn, logits_mode, fused_sum):
    """The layer captured in a HIP graph (what the benchmark times) and replayed on fresh inputs, with eager work
    and synchronisations between the replays, gives the bits of the eager calls every time, and matches the oracle.
    Covers the decode front end in one launch, the shared expert inside the routed launches (T <= 32) and on its
    side stream (T > 32), and the prefill kernels; with fused_sum also the sum of Eq. (1) inside the down projection's
    launch (decode batches), whose eager reference is the layer with the separate combine launch."""
    say("graph replay", T, shared_ffn, logits_mode, fused_sum)
    shape = wl.small_shape(dtype=wl.BF16, hidden=128, ffn=192, n_experts=8, top_k=2, shared_ffn=shared_ffn,
                           x_mode="rmsnorm", logits_mode=logits_mode)
    lays = [wl.make_layer(shape, 50, T)] + [wl.make_layer(shape, 51 + i, T, with_weights=False) for i in range(3)]
    layer = build_layer(hm, lays[0], max_tokens=T)
    x_in = torch.zeros(T, 128, dtype=torch.bfloat16, device=DEV)
    lg_in = None if logits_mode == "router" else torch.zeros(T, 8, dtype=torch.float32, device=DEV)

    def feed(lay):
        x_in.copy_(to_device(lay.x))
        if lg_in is not None:
            lg_in.copy_(to_device(lay.logits))

    feed(lays[0])
    layer.merge_combine = fused_sum
    layer.forward(x_in, lg_in)                      # warm-up outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        y_graph = layer.forward(x_in, lg_in)
    layer.merge_combine = False                     # the eager reference sums in the separate launch
    for lay in lays[1:] + lays[:1]:
        feed(lay)
        graph.replay()
        torch.cuda.synchronize()
        got = to_host_f32(y_graph).copy()
        idx_graph = layer.topk_idx[:T].cpu().numpy().copy()
        y_graph.zero_()                             # eager work between the replays
        eager = to_host_f32(layer.forward(x_in, lg_in)).copy()
        torch.cuda.synchronize()
        assert np.array_equal(got, eager) and np.array_equal(idx_graph, layer.topk_idx[:T].cpu().numpy())
        lg = lay.logits if lay.logits is not None else layer.logits[:T].cpu().numpy()
        ref = orc.moe_layer(wl.as_f64(lay.x), lg, 2, lays[0].experts, lays[0].shared, to_f64=wl.as_f64)
        assert max_rel_err(got, ref) < TOL[wl.BF16]
    layer.close()


@pytest.mark.parametrize("T,hidden,ffn,shared_ffn,dtype", [
    (1, 128, 192, (448,), "bf16"),       # 6 routed groups per expert, 14 shared groups: extra grid rows, the last one partly empty
    (4, 256, 64, (64, 64), "bf16"),      # two shared experts packed as one
    (8, 128, 320, (64,), "bf16"),        # fewer shared groups than one grid row holds
    (9, 128, 128, (192,), "bf16"),       # more than 8 rows: the 32-row form of the kernel
    (32, 64, 64, (192,), "bf16"),
    (40, 128, 128, (128,), "bf16"),      # prefill-sized: the two calls run one after the other
    (3, 64, 64, (64,), "f32"),           # fp32: likewise
])
def test_ffn_with_shared_equals_the_two_calls(hm, T, hidden, ffn, shared_ffn, dtype):
    """hmoe_expert_ffn_grouped_with_shared writes the same bits into o_perm and o_shared as the gather call for the
    routed experts followed by the plain call for the shared expert, whether or not the launches are merged; a
    layer that uses it matches the oracle."""
    say("ffn with shared", T, hidden, ffn, shared_ffn, dtype)
    shape = wl.small_shape(dtype=wl.BF16 if dtype == "bf16" else wl.F32, hidden=hidden, ffn=ffn, n_experts=8, top_k=2,
                           shared_ffn=shared_ffn)
    lay = wl.make_layer(shape, 31 + T, T)
    layer = build_layer(hm, lay, max_tokens=T)
    d, K = layer.desc, 2
    A = T * K
    x = to_device(lay.x)
    lg = lay.logits if lay.logits is not None else orc.router_logits(wl.as_f64(lay.x), wl.as_f64(lay.w_router)).astype(np.float32)
    hm.hmoe_route_permute(d, to_device(lg), T, layer.topk_idx, layer.topk_w, layer.offsets, layer.perm, layer.inv_perm, None,
                          layer.perm_ws, layer.perm_ws_bytes)
    layer.shared_offsets.copy_(torch.tensor([0, T], dtype=torch.int32))
    o_a, s_a = torch.full_like(layer.o_perm, 5.0), torch.full_like(layer.o_shared, 5.0)
    o_b, s_b = torch.full_like(layer.o_perm, 6.0), torch.full_like(layer.o_shared, 6.0)
    hm.hmoe_expert_ffn_grouped_with_shared(d, layer.cache, x, layer.perm, layer.offsets, A, None, o_a, layer.ffn_ws,
                                           layer.ffn_ws_bytes, layer.shared_desc, layer.shared_cache, layer.shared_offsets, T,
                                           s_a, layer.shared_ws, layer.shared_ws_bytes)
    torch.cuda.synchronize()
    hm.hmoe_expert_ffn_grouped_gather(d, layer.cache, x, layer.perm, layer.offsets, A, None, o_b, layer.ffn_ws,
                                      layer.ffn_ws_bytes)
    hm.hmoe_expert_ffn_grouped(layer.shared_desc, layer.shared_cache, x, layer.shared_offsets, T, None, s_b, layer.shared_ws,
                               layer.shared_ws_bytes)
    torch.cuda.synchronize()
    assert torch.equal(o_a.cpu(), o_b.cpu()) and torch.equal(s_a.cpu(), s_b.cpu())
    # an active list: only the named experts' rows are written, the shared part is unaffected
    o_c, s_c = torch.full_like(layer.o_perm, 7.0), torch.full_like(layer.o_shared, 7.0)
    hm.hmoe_expert_ffn_grouped_with_shared(d, layer.cache, x, layer.perm, layer.offsets, A, np.array([1, 5], np.int32), o_c,
                                           layer.ffn_ws, layer.ffn_ws_bytes, layer.shared_desc, layer.shared_cache,
                                           layer.shared_offsets, T, s_c, layer.shared_ws, layer.shared_ws_bytes)
    torch.cuda.synchronize()
    offs = layer.offsets.cpu().numpy()
    got, full = to_host_f32(o_c), to_host_f32(o_b)
    for e in range(8):
        rows = slice(offs[e], offs[e + 1])
        assert np.array_equal(got[rows], full[rows]) if e in (1, 5) else np.all(got[rows] == 7.0)
    assert torch.equal(s_c.cpu(), s_b.cpu())
    # the layer (which takes this call for T <= 32 in bf16) against the oracle
    y = layer.forward(x, to_device(lg))
    torch.cuda.synchronize()
    assert max_rel_err(to_host_f32(y), oracle_layer(lay, lg)) < TOL[shape.dtype]
    # argument checks
    bad = hm.make_desc(hidden, shared_ffn[0], 2, 1, 2, d.dtype)
    with pytest.raises(hm.HmoeError) as ei:
        hm.hmoe_expert_ffn_grouped_with_shared(d, layer.cache, x, layer.perm, layer.offsets, A, None, o_a, layer.ffn_ws,
                                               layer.ffn_ws_bytes, bad, layer.shared_cache, layer.shared_offsets, T, s_a,
                                               layer.shared_ws, layer.shared_ws_bytes)
    assert ei.value.status == hm.HMOE_ERR_INVALID_ARG
    with pytest.raises(hm.HmoeError) as ei:
        hm.hmoe_expert_ffn_grouped_with_shared(d, layer.cache, x, layer.perm, layer.offsets, A, None, o_a, layer.ffn_ws,
                                               layer.ffn_ws_bytes, layer.shared_desc, layer.shared_cache,
                                               layer.shared_offsets, T, s_a, layer.shared_ws, 0)
    assert ei.value.status == hm.HMOE_ERR_WORKSPACE
    layer.close()


@pytest.mark.parametrize("E,K,hidden,ffn,shared_ffn", [(8, 2, 256, 128, (64, 64)), (64, 6, 512, 192, (128,)), (8, 2, 128, 256, ()),
                                                       (16, 4, 2048, 64, (192,))])
def test_ffn_combine_equals_the_separate_calls(hm, E, K, hidden, ffn, shared_ffn):
    """hmoe_expert_ffn_combine (FFN of routed and shared experts and the sum of Eq. (1); for decode batches the sum runs
    inside the down projection's launch, done by the last block of each column block) writes the same bits into o_perm,
    o_shared and y as the separate calls, call after call through the same counters, for batches of several sizes
    (one and several row passes), and matches the oracle."""
    say("ffn_combine", E, K, hidden, ffn, shared_ffn)
    shape = wl.small_shape(dtype=wl.BF16, hidden=hidden, ffn=ffn, n_experts=E, top_k=K, shared_ffn=shared_ffn, x_mode="rmsnorm")
    base = wl.make_layer(shape, 77, 1)
    layer = build_layer(hm, base, max_tokens=40)
    d = layer.desc
    sd = layer.shared_desc
    for rep, T in enumerate([1, 8, 3, 32, 1, 9, 40]):       # 40 tokens: not a decode batch, the separate calls inside
        lay = wl.make_layer(shape, 900 + rep, T, with_weights=False)
        lay.experts, lay.shared, lay.w_router = base.experts, base.shared, base.w_router
        A = T * K
        x = to_device(lay.x)
        lg = orc.router_logits(wl.as_f64(lay.x), wl.as_f64(lay.w_router)).astype(np.float32)
        hm.hmoe_route_permute(d, to_device(lg), T, layer.topk_idx, layer.topk_w, layer.offsets, layer.perm, layer.inv_perm, None,
                              layer.perm_ws, layer.perm_ws_bytes)
        if sd is not None:
            layer.shared_offsets.copy_(torch.tensor([0, T], dtype=torch.int32))
        o_a, y_a = torch.full_like(layer.o_perm, 5.0), torch.full_like(layer.y, 5.0)
        o_b, y_b = torch.full_like(layer.o_perm, 6.0), torch.full_like(layer.y, 6.0)
        s_a = torch.full_like(layer.o_shared, 5.0) if sd is not None else None
        s_b = torch.full_like(layer.o_shared, 6.0) if sd is not None else None
        hm.hmoe_expert_ffn_combine(d, layer.cache, x, layer.perm, layer.inv_perm, layer.topk_w, layer.offsets, T, o_a, layer.ffn_ws,
                                   layer.ffn_ws_bytes, sd, None if sd is None else layer.shared_cache,
                                   None if sd is None else layer.shared_offsets, s_a, None if sd is None else layer.shared_ws,
                                   0 if sd is None else layer.shared_ws_bytes, y_a, layer.sync, layer.sync_bytes)
        torch.cuda.synchronize()
        assert int(layer.sync.max()) == 0, "the ticket counters must be left zero"
        hm.hmoe_expert_ffn_grouped_gather(d, layer.cache, x, layer.perm, layer.offsets, A, None, o_b, layer.ffn_ws,
                                          layer.ffn_ws_bytes)
        if sd is not None:
            hm.hmoe_expert_ffn_grouped(sd, layer.shared_cache, x, layer.shared_offsets, T, None, s_b, layer.shared_ws,
                                       layer.shared_ws_bytes)
        hm.hmoe_combine(d, o_b, layer.inv_perm, layer.topk_w, s_b, T, y_b)
        torch.cuda.synchronize()
        assert torch.equal(o_a[:A].cpu(), o_b[:A].cpu()), T
        assert sd is None or torch.equal(s_a[:T].cpu(), s_b[:T].cpu()), T
        assert torch.equal(y_a[:T].cpu(), y_b[:T].cpu()), T
        assert max_rel_err(to_host_f32(y_a[:T]), oracle_layer(lay, lg)) < TOL[wl.BF16]
    # argument checks: a counter buffer that is too small, a shared layer of another hidden size
    with pytest.raises(hm.HmoeError) as ei:
        hm.hmoe_expert_ffn_combine(d, layer.cache, x, layer.perm, layer.inv_perm, layer.topk_w, layer.offsets, T, o_a, layer.ffn_ws,
                                   layer.ffn_ws_bytes, None, None, None, None, None, 0, y_a, layer.sync, 4)
    assert ei.value.status == hm.HMOE_ERR_WORKSPACE
    if sd is not None:
        bad = hm.make_desc(hidden * 2, shared_ffn[0], 1, 1, 1, d.dtype)
        with pytest.raises(hm.HmoeError) as ei:
            hm.hmoe_expert_ffn_combine(d, layer.cache, x, layer.perm, layer.inv_perm, layer.topk_w, layer.offsets, T, o_a,
                                       layer.ffn_ws, layer.ffn_ws_bytes, bad, layer.shared_cache, layer.shared_offsets, s_a,
                                       layer.shared_ws, layer.shared_ws_bytes, y_a, layer.sync, layer.sync_bytes)
        assert ei.value.status == hm.HMOE_ERR_INVALID_ARG
    layer.close()


def test_stage_after_captured_ffn_calls(hm):
    """An FFN call over a partial cache captured in a HIP graph, replayed, then an expert staged into a slot the graph
    reads, and the graph replayed again on the new slot contents: every result is the one of the weights that were in
    the slot when the call ran (the copy is ordered after the replays enqueued before it)."""
    say("stage after graph capture")
    shape = wl.small_shape(dtype=wl.BF16, hidden=128, ffn=192, n_experts=4, top_k=1, n_slots=2, x_mode="rmsnorm")
    lay = wl.make_layer(shape, 9, 1)
    layer = build_layer(hm, lay, max_tokens=64)
    d = layer.desc
    T = 48
    rng = np.random.default_rng(3)
    xb = wl.store(rng.standard_normal((T, 128)).astype(np.float32), wl.BF16)
    x = to_device(xb)
    offs = to_device(np.array([0, 20, 48, 48, 48], np.int32))      # rows 0..19 -> expert 0, rows 20..47 -> expert 1

    def ref(e, rows):
        wg, wu, wd = lay.experts[e]
        return orc.expert_ffn(wl.as_f64(xb[rows]), wl.as_f64(wg), wl.as_f64(wu), wl.as_f64(wd))

    o = torch.zeros(T, 128, dtype=torch.bfloat16, device=DEV)
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        hm.hmoe_expert_ffn_grouped(d, layer.cache, x, offs, T, None, o, layer.ffn_ws, layer.ffn_ws_bytes)   # warm-up
        side.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            hm.hmoe_expert_ffn_grouped(d, layer.cache, x, offs, T, None, o, layer.ffn_ws, layer.ffn_ws_bytes)
        for _ in range(3):
            graph.replay()
        # expert 2 into slot 0 (evicts expert 0): the copy must wait for the replays above
        hm.hmoe_cache_stage(layer.cache, 2, 0, layer.h_packed[2], side, layer.copy_stream)
        side.synchronize()
        got = to_host_f32(o).copy()
        assert max_rel_err(got[:20], ref(0, slice(0, 20))) < TOL[wl.BF16] and max_rel_err(got[20:], ref(1, slice(20, 48))) < TOL[wl.BF16]
        assert layer.slot_map() == [-1, 1, 0, -1]
        # the same graph now finds expert 0 gone (its rows stay untouched) and expert 1 still there
        o.fill_(7.0)
        graph.replay()
        offs2 = to_device(np.array([0, 0, 20, 48, 48], np.int32))  # eager: rows 0..19 -> expert 1, rows 20..47 -> expert 2
        o2 = torch.zeros(T, 128, dtype=torch.bfloat16, device=DEV)
        hm.hmoe_expert_ffn_grouped(d, layer.cache, x, offs2, T, None, o2, layer.ffn_ws, layer.ffn_ws_bytes)
        side.synchronize()
    got = to_host_f32(o)
    assert np.all(got[:20] == 7.0) and max_rel_err(got[20:], ref(1, slice(20, 48))) < TOL[wl.BF16]
    got2 = to_host_f32(o2)
    assert max_rel_err(got2[:20], ref(1, slice(0, 20))) < TOL[wl.BF16] and max_rel_err(got2[20:], ref(2, slice(20, 48))) < TOL[wl.BF16]
    layer.close()


@pytest.mark.parametrize("shape_id,gpb", [(0, 1), (1, 3), (2, 2), (3, 1), (4, 3), (5, 2)])
def test_ffn_combine_every_decode_block_shape(hm, shape_id, gpb, monkeypatch):
    """The sum inside the down projection's launch with every block shape of the decode kernel and 1-3 column groups per
    block (one ticket counter per column block, whatever its width): same bits as the separate calls."""
    say("ffn_combine decode shape", shape_id, gpb)
    monkeypatch.setenv("HMOE_SKINNY", "%d,%d" % (shape_id, gpb))
    shape = wl.small_shape(dtype=wl.BF16, hidden=320, ffn=192, n_experts=6, top_k=3, shared_ffn=(128,), x_mode="rmsnorm")
    base = wl.make_layer(shape, 5, 1)
    layer = build_layer(hm, base, max_tokens=16)
    d, sd, K = layer.desc, layer.shared_desc, 3
    for rep, T in enumerate([2, 16, 5]):
        lay = wl.make_layer(shape, 40 + rep, T, with_weights=False)
        x = to_device(lay.x)
        lg = orc.router_logits(wl.as_f64(lay.x), wl.as_f64(base.w_router)).astype(np.float32)
        hm.hmoe_route_permute(d, to_device(lg), T, layer.topk_idx, layer.topk_w, layer.offsets, layer.perm, layer.inv_perm, None,
                              layer.perm_ws, layer.perm_ws_bytes)
        layer.shared_offsets.copy_(torch.tensor([0, T], dtype=torch.int32))
        o_a, y_a, s_a = torch.full_like(layer.o_perm, 5.0), torch.full_like(layer.y, 5.0), torch.full_like(layer.o_shared, 5.0)
        o_b, y_b, s_b = torch.full_like(layer.o_perm, 6.0), torch.full_like(layer.y, 6.0), torch.full_like(layer.o_shared, 6.0)
        hm.hmoe_expert_ffn_combine(d, layer.cache, x, layer.perm, layer.inv_perm, layer.topk_w, layer.offsets, T, o_a, layer.ffn_ws,
                                   layer.ffn_ws_bytes, sd, layer.shared_cache, layer.shared_offsets, s_a, layer.shared_ws,
                                   layer.shared_ws_bytes, y_a, layer.sync, layer.sync_bytes)
        hm.hmoe_expert_ffn_grouped_with_shared(d, layer.cache, x, layer.perm, layer.offsets, T * K, None, o_b, layer.ffn_ws,
                                               layer.ffn_ws_bytes, sd, layer.shared_cache, layer.shared_offsets, T, s_b,
                                               layer.shared_ws, layer.shared_ws_bytes)
        hm.hmoe_combine(d, o_b, layer.inv_perm, layer.topk_w, s_b, T, y_b)
        torch.cuda.synchronize()
        assert int(layer.sync.max()) == 0
        assert torch.equal(o_a[:T * K].cpu(), o_b[:T * K].cpu()) and torch.equal(s_a[:T].cpu(), s_b[:T].cpu())
        assert torch.equal(y_a[:T].cpu(), y_b[:T].cpu()), (shape_id, gpb, T)
    layer.close()
