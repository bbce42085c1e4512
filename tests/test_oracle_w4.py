"""Pins of the oracle's 4-bit-weight linear layer (the draft model's weights: abstract and Section 4) against
things other than itself: a hand-derived group, grids on which the quantizer is lossless (the layer is then a
plain matrix product), unit vectors, the error bound of round-to-nearest, brute force in exact rational
arithmetic on tiny sizes."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import quantspec_oracle as O


def test_hand_derived_row():
    """One row, one group of 16: weights 0.5 k - 2 for k = 0..15 -> min -2, max 5.5, S = 7.5 / 15 = 0.5, Z = -2,
    codes 0..15, decode exact; y for x = (1, ..., 1) is sum_k (0.5 k - 2) = 60 - 32 = 28."""
    w = (0.5 * np.arange(16) - 2.0).astype(np.float16).reshape(1, 16)
    c, s, z = O.quantize_w(w, 16)
    assert float(s[0, 0]) == 0.5 and float(z[0, 0]) == -2.0
    assert c[0].tolist() == list(range(16))
    assert np.array_equal(O.decode_w(c, s, z, 16), w.astype(np.float64))
    x = np.ones((1, 16), np.float16)
    assert O.linear_w4(x, c, s, z, 16)[0, 0] == 28.0
    x = np.arange(16, dtype=np.float16).reshape(1, 16)          # sum_k k (0.5 k - 2) = 0.5 * 1240 - 2 * 120
    assert O.linear_w4(x, c, s, z, 16)[0, 0] == 0.5 * 1240 - 240


@pytest.mark.parametrize("n,k,g", [(5, 256, 128), (16, 64, 32), (3, 384, 64)])
def test_lossless_grid_is_a_plain_matrix_product(n, k, g):
    """Weights Z + c 2^e with c in 0..15 and both ends present in every group: the codes are c, the decoded weights
    are the weights, and the layer equals numpy's float64 matrix product of the unquantized operands."""
    rng = np.random.default_rng(n * k + g)
    c0 = rng.integers(0, 16, (n, k))
    c0 = c0.reshape(n, k // g, g)
    c0[:, :, 0], c0[:, :, 1] = 0, 15
    c0 = c0.reshape(n, k)
    e = rng.integers(-6, 3, (n, k // g))
    zz = rng.integers(-8, 8, (n, k // g)) * 0.25
    w = (np.repeat(zz, g, axis=1) + c0 * np.repeat(2.0 ** e, g, axis=1)).astype(np.float16)
    c, s, z = O.quantize_w(w, g)
    assert np.array_equal(c, c0)
    assert np.array_equal(s.astype(np.float64), 2.0 ** e) and np.array_equal(z.astype(np.float64), zz)
    x = rng.standard_normal((4, k)).astype(np.float16)
    ref = x.astype(np.float64) @ w.astype(np.float64).T
    assert np.abs(O.linear_w4(x, c, s, z, g) - ref).max() <= 1e-12 * np.abs(ref).max()


def test_unit_vectors_read_out_the_decoded_weights_and_the_rounding_bound_holds():
    rng = np.random.default_rng(3)
    n, k, g = 7, 256, 128
    w = (rng.standard_normal((n, k)) * rng.choice([0.02, 1.0, 30.0], (n, 1))).astype(np.float16)
    c, s, z = O.quantize_w(w, g)
    assert c.min() >= 0 and c.max() <= 15
    x = np.eye(k, dtype=np.float16)
    y = O.linear_w4(x, c, s, z, g)                      # y[k, n] = w_hat[n, k]
    w_hat = y.T
    for row in range(n):                                # written out element by element, not through decode_w
        for col in range(k):
            grp = col // g
            assert w_hat[row, col] == float(c[row, col]) * float(s[row, grp]) + float(z[row, grp])
    # round to nearest: |w - w_hat| <= S / 2 (a little more where the stored fp16 S falls short of the range)
    bound = np.repeat(s.astype(np.float64), g, axis=1) * (0.5 + 2.0 ** -9)
    assert (np.abs(w.astype(np.float64) - w_hat) <= bound).all()
    # and the layer's error follows: |y - x W^T| <= sum_k |x_k| S / 2
    xr = rng.standard_normal((3, k)).astype(np.float16)
    err = np.abs(O.linear_w4(xr, c, s, z, g) - xr.astype(np.float64) @ w.astype(np.float64).T)
    assert (err <= np.abs(xr.astype(np.float64)) @ bound.T + 1e-12).all()


def test_brute_force_in_rational_arithmetic():
    """Tiny sizes, every step in exact fractions: nearest of the 16 levels Z + c S (ties cannot occur for these
    inputs: checked), then the dot products."""
    rng = np.random.default_rng(11)
    n, k, g = 3, 8, 4
    w = rng.integers(-40, 40, (n, k)).astype(np.float16) / np.float16(8)
    x = rng.integers(-9, 9, (2, k)).astype(np.float16) / np.float16(4)
    c, s, z = O.quantize_w(w, g)
    for row in range(n):
        for grp in range(k // g):
            S, Z = Fraction(float(s[row, grp])), Fraction(float(z[row, grp]))
            for col in range(grp * g, (grp + 1) * g):
                t = (Fraction(float(w[row, col])) - Z) / S
                dist = sorted((abs(t - lvl), lvl) for lvl in range(16))
                assert dist[0][0] != dist[1][0], "tie: pick other inputs"
                assert int(c[row, col]) == dist[0][1]
    y = O.linear_w4(x, c, s, z, g)
    for m in range(2):
        for row in range(n):
            acc = Fraction(0)
            for col in range(k):
                grp = col // g
                acc += Fraction(float(x[m, col])) * (int(c[row, col]) * Fraction(float(s[row, grp])) + Fraction(float(z[row, grp])))
            assert Fraction(float(y[m, row])) == acc        # small dyadic numbers: float64 holds them exactly


def test_constant_group_and_zero_input():
    w = np.full((2, 128), 0.75, np.float16)
    c, s, z = O.quantize_w(w, 128)
    assert not c.any() and (s == np.float16(1.0)).all() and (z == np.float16(0.75)).all()
    x = np.ones((1, 128), np.float16)
    assert np.array_equal(O.linear_w4(x, c, s, z, 128), np.full((1, 2), 96.0))
    assert not O.linear_w4(np.zeros((1, 128), np.float16), c, s, z, 128).any()
