"""Pins of the oracle's quantizer (Section 4.2, Section 4.3.1) against things other than itself:
hand-derived fixtures, exhaustive identities, brute-force nearest-level search in exact rational
arithmetic, error bounds, and the statistical claims the paper makes about the lower plane."""
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import quantspec_oracle as O
from paper_2502_10424_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "worked_groups.txt")


def _load_golden():
    groups = []
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        name, s, z, items = [p.strip() for p in line.split("|")]
        rows = [tuple(float(v) for v in it.split(":")) for it in items.split()]
        groups.append((name, float(s), float(z), np.array(rows)))
    return groups


@pytest.mark.parametrize("name,s,z,rows", _load_golden(), ids=lambda v: v if isinstance(v, str) else None)
def test_hand_derived_groups(name, s, z, rows):
    x = rows[:, 0].astype(np.float16)
    assert np.array_equal(x.astype(np.float64), rows[:, 0]), "fixture must be fp16-exact"
    # statistics / scale / zero from the group itself
    sg, zg = O.scale_zero(x.min(), x.max())
    assert float(sg) == s and float(zg) == z
    u, l = O.encode(x, sg, zg)
    assert u.tolist() == rows[:, 1].astype(int).tolist()
    assert l.tolist() == rows[:, 2].astype(int).tolist()
    # decode through both the key path (group along tokens) and the value path (group along channels)
    g = len(x)
    ku, kl, ks, kz = O.quantize_k(x.reshape(g, 1), g)
    vu, vl, vs, vz = O.quantize_v(x.reshape(1, g), g)
    assert ku.ravel().tolist() == u.tolist() and vu.ravel().tolist() == u.tolist()
    assert kl.ravel().tolist() == l.tolist() and vl.ravel().tolist() == l.tolist()
    for lower, col in ((False, 3), (True, 4)):
        assert np.array_equal(O.decode_k(ku, kl, ks, kz, g, lower).ravel(), rows[:, col])
        assert np.array_equal(O.decode_v(vu, vl, vs, vz, g, lower).ravel(), rows[:, col])


def test_grouping_axes_hand_example():
    """Keys: statistics per channel over the G tokens; values: per token over the G channels
    (Section 4.3.1, Appendix D).  On [[0,30],[15,45]] the two axes give different metadata."""
    m = np.array([[0, 30], [15, 45]], np.float16)
    ku, kl, ks, kz = O.quantize_k(m, 2)
    assert ks.tolist() == [[1.0, 1.0]] and kz.tolist() == [[0.0, 30.0]]
    assert ku.tolist() == [[0, 0], [15, 15]]
    vu, vl, vs, vz = O.quantize_v(m, 2)
    assert vs.tolist() == [[2.0], [2.0]] and vz.tolist() == [[0.0], [15.0]]
    assert vu.tolist() == [[0, 15], [0, 15]]


def test_k_groups_are_independent_blocks_of_g_tokens():
    rng = np.random.default_rng(1)
    k = rng.standard_normal((12, 3)).astype(np.float16)
    u, l, s, z = O.quantize_k(k, 4)
    assert s.shape == (3, 3)
    for g in range(3):
        ug, lg, sg, zg = O.quantize_k(k[4 * g:4 * g + 4], 4)
        assert np.array_equal(u[4 * g:4 * g + 4], ug) and np.array_equal(l[4 * g:4 * g + 4], lg)
        assert np.array_equal(s[g], sg[0]) and np.array_equal(z[g], zg[0])
        assert np.array_equal(zg[0], k[4 * g:4 * g + 4].min(axis=0))


def test_int8_split_exhaustive():
    """C_INT8 = 16 C_U + C_L is a bijection between [0,15] x [-8,7] and 256 consecutive integers."""
    us, ls = np.meshgrid(np.arange(16), np.arange(-8, 8), indexing="ij")
    c8 = O.int8_code(us.astype(np.uint8), ls.astype(np.int8))
    assert sorted(c8.ravel().tolist()) == list(range(-8, 248))
    u2, l2 = O.split_int8(c8)
    assert np.array_equal(u2, us) and np.array_equal(l2, ls)


def test_decode_identity_exact():
    """C_U S + C_L S/16 + Z == (16 C_U + C_L)(S/16) + Z exactly in float64 (x16 is a power of two)."""
    rng = np.random.default_rng(2)
    s = np.abs(rng.standard_normal((5, 7))).astype(np.float16) + np.float16(0.01)
    z = rng.standard_normal((5, 7)).astype(np.float16)
    u = rng.integers(0, 16, (5 * 4, 7)).astype(np.uint8)
    l = rng.integers(-8, 8, (5 * 4, 7)).astype(np.int8)
    a = O.decode_k(u, l, s, z, 4, True)
    se = np.repeat(s.astype(np.float64), 4, axis=0)
    ze = np.repeat(z.astype(np.float64), 4, axis=0)
    b = O.int8_code(u, l).astype(np.float64) * (se / 16.0) + ze
    assert np.array_equal(a, b)


def _nearest_level_exact(x, s, z, lo, hi, step_div):
    """Brute force: the code c in [lo,hi] whose level z + c*s/step_div is nearest to x, in exact
    rational arithmetic.  Returns (best code, True if the two best are within a relative 1e-6
    of a step, i.e. x sits on a rounding boundary up to binary32 rounding noise)."""
    fx, fs, fz = Fraction(float(x)), Fraction(float(s)) / step_div, Fraction(float(z))
    d = sorted((abs(fx - (fz + c * fs)), c) for c in range(lo, hi + 1))
    near_tie = (d[1][0] - d[0][0]) < fs * Fraction(1, 10**5)
    return d[0][1], near_tie


def test_codes_equal_bruteforce_nearest_level():
    """U is the nearest of the 16 levels Z + k S; given U, L is the nearest of the 16 levels
    U S + Z + l S/16 (the paper's two-stage order).  Exact rational search, no rint, no division."""
    rng = np.random.default_rng(3)
    n_checked = 0
    for trial in range(40):
        x = (rng.standard_normal(16) * rng.choice([0.01, 1.0, 30.0])
             + rng.choice([0.0, 5.0, -100.0])).astype(np.float16)
        s, z = O.scale_zero(x.min(), x.max())
        u, l = O.encode(x, s, z)
        for i in range(16):
            ub, tie_u = _nearest_level_exact(x[i], s, z, 0, 15, 1)
            if tie_u:
                continue
            assert ub == u[i]
            base = Fraction(float(z)) + int(u[i]) * Fraction(float(s))
            fs = Fraction(float(s)) / 16
            d = sorted((abs(Fraction(float(x[i])) - (base + c * fs)), c) for c in range(-8, 8))
            if (d[1][0] - d[0][0]) < fs * Fraction(1, 10**3):
                continue
            assert d[0][1] == l[i]
            n_checked += 1
    assert n_checked > 500


def test_binary32_codes_match_ideal_float64_quantizer_except_near_ties():
    rng = np.random.default_rng(4)
    x = (rng.standard_normal((64, 128)) * 3).astype(np.float16)
    u, l, s, z = O.quantize_v(x, 128)
    se, ze = s.astype(np.float64), z.astype(np.float64)
    t = (x.astype(np.float64) - ze) / se
    u64 = np.clip(np.rint(t), 0, 15)
    e64 = x.astype(np.float64) - (u64 * se + ze)
    l64 = np.clip(np.rint(e64 / (se / 16)), -8, 7)
    frac_u = np.abs(np.abs(t - np.floor(t)) - 0.5)
    t16 = e64 / (se / 16)
    frac_l = np.abs(np.abs(t16 - np.floor(t16)) - 0.5)
    du = u.astype(np.int64) != u64.astype(np.int64)
    dl = (l.astype(np.int64) != l64.astype(np.int64)) & ~du
    assert np.all(frac_u[du] < 1e-3) and np.all(frac_l[dl] < 1e-2)
    assert du.mean() < 1e-3 and dl.mean() < 1e-2
    assert np.abs(u.astype(np.int64) - u64).max() <= 1


def test_error_bounds_and_clamp_rate():
    """|x - xhat4| <= S/2 ; |x - xhat8| <= S/32 unless the lower code was clamped at +7 (then <= S/16).
    Clamping happens only where E_U/(S/16) rounds to +8."""
    w = synth.WORKLOADS["tiny"]
    k, v = synth.gen_unit_kv(w.config_id, 0, 0, 0, 1024)
    for (u, l, s, z), x, dec in ((O.quantize_k(k, 128), k, O.decode_k), (O.quantize_v(v, 128), v, O.decode_v)):
        x64 = x.astype(np.float64)
        x4, x8 = dec(u, l, s, z, 128, False), dec(u, l, s, z, 128, True)
        if dec is O.decode_k:
            se = np.repeat(s.astype(np.float64), 128, axis=0)
        else:
            se = np.repeat(s.astype(np.float64), 128, axis=1)
        slack = 1e-6 * se
        assert np.all(np.abs(x64 - x4) <= se / 2 + slack)
        e8 = np.abs(x64 - x8)
        assert np.all(e8 <= se / 16 + slack)
        over = e8 > se / 32 + slack
        assert np.all(l[over] == 7), "only +7-clamped lower codes may exceed half a lower step"
        assert 0.0 < over.mean() < 1 / 16
        assert u.min() == 0 and u.max() == 15 and l.min() == -8 and l.max() == 7
        # every group has both end codes (min -> 0, max -> 15)
        if dec is O.decode_v:
            assert np.all(u.min(axis=1) == 0) and np.all(u.max(axis=1) == 15)
        else:
            ug = u.reshape(-1, 128, 128)
            assert np.all(ug.min(axis=1) == 0) and np.all(ug.max(axis=1) == 15)
        # the error left by C_U is symmetric around zero with a mean near zero (Section 4.2)
        assert abs(l.astype(np.float64).mean()) < 0.1
        assert abs((x64 - x4).mean()) < 0.01 * se.mean()


def test_degenerate_groups():
    x = np.full((4, 4), 2.5, np.float16)
    u, l, s, z = O.quantize_v(x, 4)
    assert np.all(u == 0) and np.all(l == 0) and np.all(s == 1.0) and np.all(z == 2.5)
    assert np.array_equal(O.decode_v(u, l, s, z, 4, True), x.astype(np.float64))
    # range below fp16 resolution of the scale: (max - min)/15 rounds to 0 -> S := 1, codes 0
    tiny = np.array([[0.0, 6e-8, 0.0, 0.0]], np.float16)
    u, l, s, z = O.quantize_v(tiny, 4)
    assert s[0, 0] == 1.0 and np.all(u == 0) and np.all(l == 0)


def test_on_grid_data_is_lossless():
    """Data on the 4-bit grid decodes exactly from the upper plane alone; data on the 8-bit grid
    decodes exactly from both planes."""
    rng = np.random.default_rng(5)
    kk = rng.integers(0, 16, (8, 16))
    kk[0, :], kk[1, :] = 0, 15
    x4 = (-2.0 + 0.25 * kk).astype(np.float16)
    u, l, s, z = O.quantize_k(x4, 8)
    assert np.array_equal(u, kk) and np.all(l == 0)
    assert np.array_equal(O.decode_k(u, l, s, z, 8, False), x4.astype(np.float64))
    c = rng.integers(0, 241, (8, 16))
    c[0, :], c[1, :] = 0, 240
    x8 = (1.0 + c / 64.0).astype(np.float16)          # S = 0.25, S/16 = 1/64; all fp16-exact
    assert np.array_equal(x8.astype(np.float64), 1.0 + c / 64.0)
    u, l, s, z = O.quantize_k(x8, 8)
    assert np.all(s == 0.25) and np.all(z == 1.0)
    # c = 16k + 8 is the tie of the upper code: for odd k it rounds up (U = k+1, L = -8, exact);
    # for even k it rounds down and E_U = +8 steps does not fit [-8, 7] (the clamp case, off by S/16).
    clamp_case = ((c % 16) == 8) & ((c // 16) % 2 == 0)
    dec = O.decode_k(u, l, s, z, 8, True)
    assert np.array_equal(dec[~clamp_case], x8.astype(np.float64)[~clamp_case])
    assert np.array_equal(O.int8_code(u, l)[~clamp_case], c[~clamp_case])
    assert np.array_equal(O.int8_code(u, l)[clamp_case], c[clamp_case] - 1)
    assert clamp_case.any() and (((c % 16) == 8) & ~clamp_case).any()


def test_axis_choice_direction_on_outlier_keys():
    """Per-channel grouping of keys beats per-token grouping when a few channels are outliers
    (direction of Table 5); the synthetic key recipe is built to show exactly that."""
    w = synth.WORKLOADS["tiny"]
    k, _ = synth.gen_unit_kv(w.config_id, 0, 0, 1, 1024)
    ch = synth.outlier_channels(w.config_id, 0, 0, 1)
    k64 = k.astype(np.float64)
    u, l, s, z = O.quantize_k(k, 128)
    e_chan = O.decode_k(u, l, s, z, 128, False) - k64
    u, l, s, z = O.quantize_v(k, 128)                   # token-wise grouping applied to keys
    e_tok = O.decode_v(u, l, s, z, 128, False) - k64
    normal = np.setdiff1d(np.arange(128), ch)
    rms = lambda e: np.sqrt((e ** 2).mean())
    assert rms(e_tok[:, normal]) > 3.0 * rms(e_chan[:, normal])
    assert rms(e_tok) > 1.5 * rms(e_chan)


def test_planted_mistakes_are_caught():
    """The pins above must fail for plausible mistakes: truncation instead of RTN, error computed
    against the wrong sign, grouping along the wrong axis."""
    x = np.array([7.25, 0.0, 15.0, 3.96875, 8.5, 11.3125, 2.5, 7.5], np.float16)
    s, z = O.scale_zero(x.min(), x.max())
    u, l = O.encode(x, s, z)
    t = (x.astype(np.float32) - z.astype(np.float32)) / s.astype(np.float32)
    assert not np.array_equal(np.floor(t).astype(np.uint8), u)          # truncation differs
    wrong_l = np.clip(np.rint((u * s.astype(np.float32) + z - x.astype(np.float32)) * 16), -8, 7)
    assert not np.array_equal(wrong_l.astype(np.int8), l)                # flipped sign differs
    m = np.array([[0, 30], [15, 45]], np.float16)
    assert not np.array_equal(O.quantize_k(m, 2)[0], O.quantize_v(m, 2)[0])
