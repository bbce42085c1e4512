"""GPU parity of the draft model's 4-bit-weight linear layer (abstract; Section 4) against the oracle: codes,
scales and zeros bit for bit, outputs within 2e-3 of the largest output of a row (fp16 outputs, binary32 sums)."""
import sys

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

TOL = 2e-3


def _say(msg):
    print(f"[case] {msg}", flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def env():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from oracle import quantspec_oracle as O
    from paper_2502_10424_amd import binding as B
    B.lib()
    return dict(torch=torch, O=O, B=B)


def _weights(rng, n, k):
    """Rows of different magnitude, a few outlier input channels, a per-row offset."""
    w = rng.standard_normal((n, k)) * rng.choice([0.01, 0.05, 1.0], (n, 1)) + 0.02 * rng.standard_normal((n, 1))
    w[:, rng.integers(0, k, 6)] *= 8.0
    return w.astype(np.float16)


def _check_layer(env, w, xs, tag):
    torch, O, B = env["torch"], env["O"], env["B"]
    n, k = w.shape
    layer = B.W4Linear(n, k)
    B.qs_w4_quantize(layer, torch.from_numpy(w).cuda())
    codes, scale, zero = [t.cpu().numpy() for t in B.qs_w4_export(layer)]
    c, s, z = O.quantize_w(w, 128)
    assert np.array_equal(codes, c), tag
    assert np.array_equal(scale.view(np.uint16), s.view(np.uint16)) and np.array_equal(zero.view(np.uint16), z.view(np.uint16)), tag
    for x in xs:
        y = B.qs_w4_linear(layer, torch.from_numpy(x).cuda()).cpu().numpy().astype(np.float64)
        torch.cuda.synchronize()
        ref = O.linear_w4(x, c, s, z, 128)
        assert np.isfinite(y).all(), tag
        err = float((np.abs(y - ref).max(axis=1) / np.abs(ref).max(axis=1)).max())
        _say(f"{tag} m={x.shape[0]}: max rel err {err:.2e}")
        assert err <= TOL, tag


@pytest.mark.parametrize("n,k", [(16, 128), (48, 384), (256, 1024), (4096, 4096), (1024, 11008), (160, 32768)])
def test_linear_parity(env, n, k):
    """From one block to the sizes of a 7B model's projections (4096 x 4096, 11008 inputs) and the longest row the
    kernel takes; 1, 3 and 16 rows of x; block counts that do not divide by the eight waves or by the look-ahead."""
    rng = np.random.default_rng(n + k)
    w = _weights(rng, n, k)
    xs = [rng.standard_normal((m, k)).astype(np.float16) for m in (1, 3, 16)]
    _check_layer(env, w, xs, f"W4 {n}x{k}")


def test_linear_edge_values(env):
    """Constant rows (S = 1), rows of zeros, weights and inputs of large and tiny magnitude (outputs inside fp16),
    a unit-vector input."""
    rng = np.random.default_rng(5)
    n, k = 32, 512
    w = _weights(rng, n, k)
    w[0] = 0.75
    w[1] = 0.0
    w[2] = (rng.standard_normal(k) * 100).astype(np.float16)
    w[3] = (rng.standard_normal(k) * 1e-4).astype(np.float16)
    x_unit = np.zeros((1, k), np.float16)
    x_unit[0, 130] = 1.0
    xs = [x_unit, (rng.standard_normal((2, k)) * 10).astype(np.float16), (rng.standard_normal((2, k)) * 1e-3).astype(np.float16)]
    _check_layer(env, w, xs, "W4 edge values")


def test_linear_is_deterministic_and_rejects_bad_arguments(env):
    torch, B = env["torch"], env["B"]
    rng = np.random.default_rng(9)
    n, k = 512, 2048
    layer = B.W4Linear(n, k)
    B.qs_w4_quantize(layer, torch.from_numpy(_weights(rng, n, k)).cuda())
    x = torch.from_numpy(rng.standard_normal((4, k)).astype(np.float16)).cuda()
    y0 = B.qs_w4_linear(layer, x).clone()
    for _ in range(3):
        assert torch.equal(B.qs_w4_linear(layer, x), y0)
    assert B.qs_w4_bytes(n, k) == (n // 16) * (k // 128) * 1088
    assert B.qs_w4_bytes(n + 8, k) == 0 and B.qs_w4_bytes(n, k + 64) == 0 and B.qs_w4_bytes(n, 65536) == 0
    with pytest.raises(B.QsError):
        B.qs_w4_linear(layer, torch.zeros((17, k), dtype=torch.float16, device="cuda"))
