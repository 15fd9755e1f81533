"""Host-side checks of libhmoe that need no GPU: the library loads, exports every symbol the
header declares, rejects bad arguments before touching the device, and packs weights into the
documented slot layout."""
import ctypes
import os
import re

import numpy as np
import pytest

import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def hm():
    import paper_2504_05897_amd as hm
    return hm


def test_library_exports_every_declared_symbol(hm):
    header = open(os.path.join(ROOT, "include", "hmoe.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(hmoe_[a-z_]+)\s*\(", header))
    assert declared == set(hm.EXPORTS)
    lib = ctypes.CDLL(os.path.join(ROOT, "paper_2504_05897_amd", "libhmoe.so"))
    for name in declared:
        assert hasattr(lib, name), name


def test_status_strings(hm):
    assert hm._lib.hmoe_status_string(0) == b"ok"
    for code in range(-6, 0):
        assert hm._lib.hmoe_status_string(code) not in (b"ok", b"unknown status")


def test_bad_descriptors_are_rejected_on_the_host(hm):
    bad = [hm.make_desc(0, 64, 8, 2, 8, 1), hm.make_desc(64, 64, 8, 9, 8, 1), hm.make_desc(64, 64, 8, 2, 9, 1),
           hm.make_desc(64, 64, 8, 2, 8, 7), hm.make_desc(64, -1, 8, 2, 8, 0)]
    for d in bad:
        assert hm._lib.hmoe_route(ctypes.byref(d), None, 4, None, None, None) == hm.HMOE_ERR_INVALID_ARG
        assert hm.hmoe_slot_bytes(d) == 0
    too_many = hm.make_desc(64, 64, 300, 2, 8, 1)
    assert hm._lib.hmoe_route(ctypes.byref(too_many), None, 4, None, None, None) == hm.HMOE_ERR_UNSUPPORTED
    ok = hm.make_desc(64, 64, 8, 2, 8, 1)
    assert hm._lib.hmoe_route(ctypes.byref(ok), None, -1, None, None, None) == hm.HMOE_ERR_INVALID_ARG
    assert hm._lib.hmoe_route(ctypes.byref(ok), None, 4, None, None, None) == hm.HMOE_ERR_INVALID_ARG
    assert hm._lib.hmoe_route(ctypes.byref(ok), None, 0, None, None, None) == hm.HMOE_OK      # T = 0: no-op
    odd = hm.make_desc(72, 64, 8, 2, 8, 1)                                                    # bf16 needs H % 64 == 0
    buf = np.zeros(16, np.uint8)
    assert hm._lib.hmoe_pack_expert(ctypes.byref(odd), buf.ctypes.data, buf.ctypes.data, buf.ctypes.data,
                                    buf.ctypes.data) == hm.HMOE_ERR_UNSUPPORTED


def test_slot_bytes(hm):
    assert hm.hmoe_slot_bytes(hm.make_desc(4096, 14336, 8, 2, 4, 1)) == 3 * 4096 * 14336 * 2
    assert hm.hmoe_slot_bytes(hm.make_desc(256, 512, 8, 2, 8, 0)) == 3 * 256 * 512 * 4
    assert hm.hmoe_slot_bytes(hm.make_desc(8, 3, 2, 1, 2, 0)) % 256 == 0


def test_pack_fp32_is_plain_concatenation(hm):
    rng = np.random.default_rng(0)
    d = hm.make_desc(24, 40, 4, 2, 4, 0)
    wg, wu, wd = (rng.standard_normal(s).astype(np.float32) for s in ((40, 24), (40, 24), (24, 40)))
    out = np.zeros(hm.hmoe_slot_bytes(d) // 4, np.float32)
    hm.hmoe_pack_expert(d, wg, wu, wd, out)
    n = 24 * 40
    assert np.array_equal(out[:n], wg.ravel()) and np.array_equal(out[n:2 * n], wu.ravel())
    assert np.array_equal(out[2 * n:3 * n], wd.ravel())


def test_pack_bf16_tile_layout(hm):
    """32-row x 16-k tiles, 1 KiB each, lane l of a tile holds row l%32, k 8*(l/32)..+8; gate and up
    interleaved in 32-row groups; tiles ordered [row group][k tile]."""
    hid, ffn = 128, 192
    d = hm.make_desc(hid, ffn, 4, 2, 4, 1)
    # distinct bit patterns so that every element is identifiable
    wg = (np.arange(ffn * hid, dtype=np.uint32) % 60000).astype(np.uint16).reshape(ffn, hid)
    wu = ((np.arange(ffn * hid, dtype=np.uint32) * 7 + 1) % 60000).astype(np.uint16).reshape(ffn, hid)
    wd = ((np.arange(ffn * hid, dtype=np.uint32) * 13 + 5) % 60000).astype(np.uint16).reshape(hid, ffn)
    out = np.zeros(hm.hmoe_slot_bytes(d) // 2, np.uint16)
    hm.hmoe_pack_expert(d, wg, wu, wd, out)

    def expect(mat, n_rows, k_len, row_map):
        res = np.zeros(n_rows * k_len, np.uint16)
        kt = k_len // 16
        for nb in range(n_rows // 32):
            for kb in range(kt):
                for lane in range(64):
                    src_row = row_map(nb, lane % 32)
                    k0 = kb * 16 + 8 * (lane // 32)
                    base = ((nb * kt + kb) * 64 + lane) * 8
                    res[base:base + 8] = mat(src_row)[k0:k0 + 8]
        return res

    gu = expect(lambda rg: (wu if rg[0] else wg)[rg[1]], 2 * ffn, hid,
                lambda nb, r: (nb % 2, 32 * (nb // 2) + r))
    dn = expect(lambda row: wd[row], hid, ffn, lambda nb, r: 32 * nb + r)
    assert np.array_equal(out[:2 * ffn * hid], gu)
    assert np.array_equal(out[2 * ffn * hid:3 * ffn * hid], dn)


def test_workload_shapes_fit_the_kernels(hm):
    for s in wl.SHAPES.values():
        if s.dtype == wl.BF16:
            assert s.hidden % 64 == 0 and s.ffn % 64 == 0
            for f in s.shared_ffn:
                assert f % 64 == 0


def test_traffic_table_names_kernels_that_exist():
    """profiles/traffic.json (HBM bytes per launch from the counter runs, copied by bench.py into roofline.traffic)
    must name kernels that the sources still define."""
    import json
    import re
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    with open(os.path.join(root, "profiles", "traffic.json")) as fh:
        table = json.load(fh)
    csrc = os.path.join(root, "paper_2504_05897_amd", "csrc")
    text = "".join(open(os.path.join(csrc, f)).read() for f in os.listdir(csrc))
    assert table
    for key, entry in table.items():
        assert entry["bytes"] > 0 and re.fullmatch(r"\w+/\w+(\+w4)?", key), key
        base = entry["kernel"].split("<")[0]
        assert re.search(r"\b%s\b" % re.escape(base), text), "%s: kernel %s is gone; profile again" % (key, base)


def test_new_entry_points_reject_bad_arguments_on_the_host(hm):
    """hmoe_permute_static, hmoe_expert_ffn_combine and hmoe_expert_ffn_staged check what the host can check before
    they touch the device."""
    ok = hm.make_desc(64, 64, 8, 2, 8, 1)
    big = hm.make_desc(64, 64, 256, 32, 256, 1)
    lib = hm._lib
    assert lib.hmoe_permute_static(ctypes.byref(ok), None, -1, None, None, None, None, None, None, None) == hm.HMOE_ERR_INVALID_ARG
    assert lib.hmoe_permute_static(ctypes.byref(big), None, 40000, None, None, None, None, None, None, None) == hm.HMOE_ERR_WORKSPACE
    assert b"HMOE_PERMUTE_STATIC_BYTES" in lib.hmoe_last_error()
    assert hm.hmoe_permute_workspace_bytes(big, 40000) > hm.HMOE_PERMUTE_STATIC_BYTES
    assert hm.hmoe_ffn_combine_sync_bytes(ok) >= (64 // 32) * 4 and hm.hmoe_ffn_combine_sync_bytes(ok) % 256 == 0
    args = [None] * 22
    args[0] = ctypes.byref(ok)
    args[7], args[10], args[16], args[19], args[20] = 4, 0, 0, 0, 0
    assert lib.hmoe_expert_ffn_combine(*args) == hm.HMOE_ERR_INVALID_ARG          # no perm / inv_perm / weights / y
    args[7] = 0
    assert lib.hmoe_expert_ffn_combine(*args) == hm.HMOE_OK                       # T = 0: no-op
    sargs = [None] * 19
    sargs[0] = ctypes.byref(ok)
    sargs[5], sargs[10], sargs[11] = 0, 0, 0
    assert lib.hmoe_expert_ffn_staged(*sargs) == hm.HMOE_ERR_INVALID_ARG          # no cache, no counts, no plan arrays
    assert lib.hmoe_cache_set_layer(None, ctypes.byref(ok)) == hm.HMOE_ERR_INVALID_ARG      # no cache
