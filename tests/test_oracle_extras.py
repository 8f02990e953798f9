"""Pins for the oracle's helpers around the step (CPU only): per-tensor sums of squares and the
value of 16-bit gradient patterns."""
import math

import numpy as np
import pytest
import torch


def test_tensor_sumsq_hand_case(oracle):
    """Small integers, sums written out by hand."""
    g = np.array([[1, 2, 3, 4, 5], [0, -1, 0, 2, 0]], dtype=np.float32)
    m = np.array([[1, 1, 1, 1, 1], [2, 0, 0, 0, -2]], dtype=np.float32)
    x = np.array([[0, 0, 3, 0, 4], [1, 2, 2, 0, 0]], dtype=np.float32)
    out = oracle.tensor_sumsq(g, m, x, [0, 2, 2, 5])            # tensors: columns 0-1, none, 2-4
    want = np.array([[[5, 2, 0], [1, 4, 5]],
                     [[0, 0, 0], [0, 0, 0]],
                     [[50, 3, 25], [4, 4, 4]]], dtype=np.float64)
    np.testing.assert_array_equal(out, want)


def test_tensor_sumsq_against_exact_summation(oracle):
    r = np.random.default_rng(5)
    n, d = 3, 200
    arrs = [r.standard_normal((n, d)).astype(np.float32) for _ in range(3)]
    offsets = [0, 1, 64, 64, 130, 200]
    out = oracle.tensor_sumsq(*arrs, offsets)
    for t in range(5):
        for i in range(n):
            for q in range(3):
                exact = math.fsum(float(v) * float(v) for v in arrs[q][i, offsets[t]:offsets[t + 1]])
                assert abs(out[t, i, q] - exact) <= 1e-13 * max(exact, 1.0)
    # the tensors partition the columns: per-node totals are the whole-row sums
    total = out.sum(axis=0)
    for q in range(3):
        np.testing.assert_allclose(total[:, q], (arrs[q].astype(np.float64) ** 2).sum(axis=1), rtol=1e-13)


@pytest.mark.parametrize("fmt,dtype", [("bf16", torch.bfloat16), ("f16", torch.float16)])
def test_widen16_against_a_library_conversion_on_every_pattern(oracle, fmt, dtype):
    """All 65536 patterns: the field-by-field value equals what the tensor library's own
    conversion to float32 gives (NaNs compared as NaNs)."""
    bits = np.arange(65536, dtype=np.int64).astype(np.uint16)
    mine = oracle.widen16(bits, fmt)
    lib = torch.from_numpy(bits.view(np.int16)).view(dtype).to(torch.float32).numpy().astype(np.float64)
    nan = np.isnan(lib)
    np.testing.assert_array_equal(np.isnan(mine), nan)
    np.testing.assert_array_equal(mine[~nan], lib[~nan])


def test_widen16_known_values(oracle):
    # 1.0, -2.0, smallest normal, largest finite, a subnormal, in both formats
    assert oracle.widen16([0x3F80, 0xC000, 0x0080, 0x7F7F, 0x0001], "bf16").tolist() == [
        1.0, -2.0, 2.0 ** -126, (2 - 2.0 ** -7) * 2.0 ** 127, 2.0 ** -133]
    assert oracle.widen16([0x3C00, 0xC000, 0x0400, 0x7BFF, 0x0001], "f16").tolist() == [
        1.0, -2.0, 2.0 ** -14, 65504.0, 2.0 ** -24]
