"""Pins for the oracle of the 4-bit weight format: hand-computed codes and scales, the error bound the
rounding rule implies, idempotence, and the bf16 rounding of the scale."""
import numpy as np

from oracle import w4_oracle as w4


def test_hand_case():
    row = np.zeros(256, np.float32)
    row[:6] = [0.7, -0.35, 0.1, -0.7, 0.05, 0.049]
    row[128:131] = [3.0, -1.0, 1.5]
    codes, scales = w4.quantize_w4(row[None])
    # group 0: 0.7 / 7 = 0.1 -> nearest bfloat16 is 0.10009765625 (0x3DCD)
    assert scales[0, 0] == np.float32(0.10009765625)
    # 0.7/s = 6.993 -> 7; -0.35/s = -3.4966 -> -3; 0.1/s = 0.999 -> 1; -0.7 -> -7; 0.05/s = 0.4995 -> 0; 0.049 -> 0
    assert codes[0, :6].tolist() == [15, 5, 9, 1, 8, 8] and np.all(codes[0, 6:128] == 8)
    # group 1: 3/7 = 0.428571 -> bfloat16 0.427734375 (0x3EDB); 3/s = 7.0137 -> 7; -1/s = -2.338 -> -2; 1.5/s = 3.507 -> 4
    assert scales[0, 1] == np.float32(0.427734375)
    assert codes[0, 128:131].tolist() == [15, 6, 12]
    deq = w4.dequantize_w4(codes, scales)
    assert deq[0, 0] == 7 * 0.10009765625 and deq[0, 1] == -3 * 0.10009765625 and deq[0, 130] == 4 * 0.427734375


def test_zero_group_and_ranges():
    w = np.zeros((3, 128), np.float32)
    w[1, 5] = -2.0
    codes, scales = w4.quantize_w4(w)
    assert scales[0, 0] == 0 and np.all(codes[0] == 8) and np.all(w4.dequantize_w4(codes, scales)[0] == 0)
    assert codes[1, 5] == 1 and codes.min() >= 0 and codes.max() <= 15        # -7 -> code 1; code 0 (-8) is never needed


def test_error_bound_and_idempotence():
    rng = np.random.default_rng(0)
    w = (rng.standard_normal((40, 512)) * 0.02).astype(np.float32)
    w = w.view(np.uint32) >> 16 << 16                                          # make the values bfloat16-representable
    w = w.astype(np.uint32).view(np.float32)
    codes, scales = w4.quantize_w4(w)
    deq = w4.dequantize_w4(codes, scales)
    s = np.repeat(scales.astype(np.float64), 128, axis=1)
    # nearest code: at most half a step away (the largest element of a group may sit a hair beyond +-7 steps
    # because the scale itself was rounded to bfloat16: 2^-9 relative, i.e. < 0.03 of a step)
    assert np.all(np.abs(deq - w) <= 0.5 * s + 0.03 * s + 1e-12)
    # every group uses the full range on one side
    m = np.abs(codes.astype(np.int32) - 8).reshape(40, 4, 128).max(axis=2)
    assert np.all(m == 7)
    # quantising the dequantised values again changes nothing
    codes2, scales2 = w4.quantize_w4(deq.astype(np.float32))
    assert np.array_equal(codes, codes2) and np.array_equal(scales, scales2)


def test_scale_rounding_is_nearest_even_bfloat16():
    v = np.array([1.0, 1.00390625, 1.01171875, 1.0 + 2 ** -9, 1.0 + 3 * 2 ** -9], np.float32)
    # 1 + 2^-8 is halfway between 1 and 1 + 2^-7: ties to even (1.0); 1 + 3*2^-8 ties to 1 + 2^-6
    assert w4._bf16_round(v).tolist() == [1.0, 1.0, 1.015625, 1.0, 1.0078125]
