"""4-bit expert weights (HMOE_BF16_W4): the library's host-side quantiser and slot layout against the
oracle's quantiser, code for code and scale for scale.  No GPU."""
import numpy as np
import pytest

import workloads as wl
from oracle import w4_oracle as w4


@pytest.fixture(scope="module")
def hm():
    import paper_2504_05897_amd as hm
    return hm


def unpack_matrix(units_u32, scales_u16, n_rows, k_len, packed_row):
    """Reads codes [n_rows, k_len] and scales [n_rows, k_len/128] back out of the slot layout: 1 KiB units of
    16 rows x 128 k ordered [row group][unit]; lane l = 16 (k block of 8 within a k-step of 32) + row; dword t = k-step
    t of the unit; code j at bit 16 (j & 1) + 4 (j >> 1).  packed_row(n) = row index inside the packed matrix."""
    codes = np.zeros((n_rows, k_len), np.uint8)
    scales = np.zeros((n_rows, k_len // 128), np.uint16)
    for n in range(n_rows):
        pn = packed_row(n)
        for k in range(k_len):
            lane = ((k % 32) // 8) * 16 + pn % 16
            dword = (((pn // 16) * (k_len // 128) + k // 128) * 64 + lane) * 4 + (k % 128) // 32
            shift = 16 * (k & 1) + 4 * ((k % 8) >> 1)
            codes[n, k] = (int(units_u32[dword]) >> shift) & 15
        for g in range(k_len // 128):
            scales[n, g] = scales_u16[((pn // 16) * (k_len // 128) + g) * 16 + pn % 16]
    return codes, scales


def test_pack_w4_equals_the_oracle_quantiser(hm):
    hid, ffn = 256, 128
    d = hm.make_desc(hid, ffn, 4, 2, 4, hm.HMOE_BF16_W4)
    hf = hid * ffn
    assert hm.hmoe_slot_bytes(d) == hf + hf // 32 + hf // 2 + hf // 64
    rng = np.random.default_rng(3)
    mats = [wl.f32_to_bf16_bits((rng.standard_normal(s) * 0.02).astype(np.float32)) for s in ((ffn, hid), (ffn, hid), (hid, ffn))]
    mats[0][5, :128] = 0                      # a group of zeros
    mats[2][7, 3] = wl.f32_to_bf16_bits(np.array([0.5], np.float32))[0]   # one outlier in a group
    out = np.zeros(hm.hmoe_slot_bytes(d), np.uint8)
    hm.hmoe_pack_expert(d, *mats, out)
    gu_units = out[:hf].view(np.uint32)
    gu_scales = out[hf:hf + hf // 32].view(np.uint16)
    dn_units = out[hf + hf // 32:hf + hf // 32 + hf // 2].view(np.uint32)
    dn_scales = out[hf + hf // 32 + hf // 2:].view(np.uint16)
    for which, (mat, units, scales, n_rows, k_len, prow) in enumerate([
            (mats[0], gu_units, gu_scales, ffn, hid, lambda n: 32 * (n // 16) + n % 16),          # gate: even 16-row groups
            (mats[1], gu_units, gu_scales, ffn, hid, lambda n: 32 * (n // 16) + 16 + n % 16),     # up: odd groups
            (mats[2], dn_units, dn_scales, hid, ffn, lambda n: n)]):
        codes, sc = unpack_matrix(units, scales, n_rows, k_len, prow)
        ref_codes, ref_scales = w4.quantize_w4(wl.as_f32(mat))
        assert np.array_equal(codes, ref_codes), which
        assert np.array_equal(sc, wl.f32_to_bf16_bits(ref_scales)), which
        assert np.array_equal(wl.as_f32(sc), ref_scales)            # the oracle's scales are bfloat16 values


def test_w4_shape_requirements(hm):
    for hid, ffn in [(192, 128), (128, 192), (64, 64)]:
        d = hm.make_desc(hid, ffn, 4, 2, 4, hm.HMOE_BF16_W4)
        assert hm.hmoe_slot_bytes(d) == 0
        with pytest.raises(hm.HmoeError) as ei:
            hm.hmoe_pack_expert(d, np.zeros((ffn, hid), np.uint16), np.zeros((ffn, hid), np.uint16),
                                np.zeros((hid, ffn), np.uint16), np.zeros(16, np.uint8))
        assert ei.value.status == hm.HMOE_ERR_UNSUPPORTED
