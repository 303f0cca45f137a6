"""Pins for the oracle's integer inner product (Section 4): a hand-worked
example, the identity with the inner product of the dequantized values, and
the reduction to the uniform-quantization formula when the tail is empty."""
import os

import numpy as np
import pytest

from oracle import pwlq_ref as R

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _example():
    d = {}
    with open(os.path.join(GOLD, "linear_worked_example.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            k, *v = line.split()
            d[k] = [float(x) for x in v]
    return d


def test_worked_example():
    d = _example()
    bits = int(d["bits"][0])
    w = np.array([d["w"]], np.float32)
    p = np.array(d["p"], np.float32)
    m = np.array(d["m"], np.float32)
    codes, flags, _ = R.quantize(w, bits, p, m)
    xq = np.array([d["x_q"]], np.int8)
    y, acc = R.linear(xq, d["s_x"][0], d["z_x"][0], codes, flags, bits, p, m, want_acc=True)
    assert acc[:, 0, 0].tolist() == [int(v) for v in d["acc"]]
    assert y[0, 0] == d["y"][0]


def _case(rng, M, K, N, bits, dist="laplace"):
    w = (rng.laplace(0, 0.05, (N, K)) if dist == "laplace" else rng.standard_normal((N, K)))
    w = w.astype(np.float32)
    s = R.search(w, bits, 50)
    codes, flags, w_hat = R.quantize(w, bits, s["p_star"], s["m"])
    xq = rng.integers(-128, 128, (M, K)).astype(np.int8)
    return w, s, codes, flags, w_hat, xq


@pytest.mark.parametrize("bits", [2, 3, 4, 6, 8])
def test_equals_inner_product_of_dequantized_values(bits):
    # <X_hat, W_hat> with X_hat = s_x X_q + z_x and W_hat from the quantizer; the
    # integer path uses step*code where the quantizer snaps the top code to the
    # end point, so the two agree to binary32 rounding of the steps
    rng = np.random.default_rng(bits)
    w, s, codes, flags, w_hat, xq = _case(rng, 5, 96, 7, bits)
    s_x, z_x = 0.0173, -1.234
    y = R.linear(xq, s_x, z_x, codes, flags, bits, s["p_star"], s["m"])
    x_hat = np.float64(np.float32(s_x)) * xq.astype(np.float64) + np.float64(np.float32(z_x))
    direct = x_hat @ w_hat.astype(np.float64).T
    scale = np.abs(x_hat) @ np.abs(w_hat.astype(np.float64)).T
    assert np.max(np.abs(y - direct) / scale) < 3e-7


def test_integer_sums_by_masked_matmul():
    rng = np.random.default_rng(10)
    bits = 4
    w, s, codes, flags, _, xq = _case(rng, 9, 128, 11, bits, "normal")
    _, acc = R.linear(xq, 1.0, 0.0, codes, flags, bits, s["p_star"], s["m"], want_acc=True)
    mag = (codes & 7).astype(np.int64)
    sg = np.where(codes & 8, -1, 1).astype(np.int64)
    wq = mag * sg
    x = xq.astype(np.int64)
    np.testing.assert_array_equal(acc[0], x @ (wq * (flags == 0)).T)
    np.testing.assert_array_equal(acc[1], x @ (wq * (flags == 1)).T)
    np.testing.assert_array_equal(acc[2], x @ (sg * (flags == 1)).T)


def test_empty_tail_is_the_uniform_formula():
    # p = m: every weight is a centre weight and Section 4's Eq. for uniform
    # quantization remains: <X_hat, W_hat> = C0 <X_q, W_q> + C1 with C0 = s_x s_w,
    # C1 = z_x s_w <W_q, 1>
    rng = np.random.default_rng(12)
    bits, K, N, M = 5, 64, 4, 3
    w = rng.standard_normal((N, K)).astype(np.float32)
    m = np.abs(w).max(axis=1)
    codes, flags, _ = R.quantize(w, bits, m, m)
    assert not flags.any()
    xq = rng.integers(-128, 128, (M, K)).astype(np.int8)
    s_x, z_x = 0.031, 0.77
    y, acc = R.linear(xq, s_x, z_x, codes, flags, bits, m, m, want_acc=True)
    assert not acc[1].any() and not acc[2].any()
    L = 2 ** (bits - 1) - 1
    s_w = (m / np.float32(L)).astype(np.float32).astype(np.float64)
    wq = (codes & (2 ** (bits - 1) - 1)).astype(np.int64) * np.where(codes & 2 ** (bits - 1), -1, 1)
    C0 = np.float64(np.float32(s_x)) * s_w
    C1 = np.float64(np.float32(z_x)) * s_w * wq.sum(axis=1)
    np.testing.assert_allclose(y, (xq.astype(np.int64) @ wq.T) * C0 + C1, rtol=1e-14, atol=1e-14)


def test_linear_argument_checks():
    x = np.zeros((2, 8), np.int8)
    c = np.zeros((3, 8), np.uint8)
    p = np.ones(3, np.float32)
    with pytest.raises(ValueError):
        R.linear(x, 1.0, 0.0, c, c, 9, p, p)
    with pytest.raises(ValueError):
        R.linear(x, 1.0, 0.0, c, c[:2], 4, p, p)
