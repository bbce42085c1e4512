"""qs_attn_static - the attention calls with the split-K partials in the library's built-in scratch array -
against qs_attn_draft / qs_attn_verify with a caller workspace: same kernels, same plan, so the outputs
must agree bit for bit (fixed ranges) on two calls in a row, the second on a smaller input."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2502_10424_amd import binding as B
    from tests import gpu_util as U
    B.lib()
    return dict(torch=torch, B=B, U=U)


def _case(env, seed, bsz, hkv, rep, n_groups, nb):
    rng = np.random.default_rng(seed)
    t = 128 * n_groups + nb
    k = (rng.standard_normal((bsz, hkv, t, 128)) * 1.5).astype(np.float16)
    v = rng.standard_normal((bsz, hkv, t, 128)).astype(np.float16)
    cache = env["U"].make_device_cache(k, v, hkv * rep, nb)
    cache.flags = env["B"].QS_FLAG_FIXED_RANGES       # bit-reproducible: the comparison below is exact
    return cache, rng


def test_static_scratch_matches_caller_workspace(env):
    torch, B = env["torch"], env["B"]
    print("[case] qs_attn_static: 3 x 2 kv-heads x 4, 24 groups + 200 buffered; then 1 x 2 x 1, 3 groups + 17", flush=True)
    for seed, (bsz, hkv, rep, n_groups, nb, nq) in enumerate([(3, 2, 4, 24, 200, 5), (1, 2, 1, 3, 17, 3)]):
        cache, rng = _case(env, 40 + seed, bsz, hkv, rep, n_groups, nb)
        assert B.qs_workspace_bytes(cache, nq) <= B.QS_STATIC_WS_BYTES
        for verify, n in ((False, 1), (True, nq)):
            q = torch.from_numpy(rng.standard_normal((bsz, n, hkv * rep, 128)).astype(np.float16)).cuda()
            lse_a = torch.empty((bsz, n, hkv * rep), dtype=torch.float32, device="cuda")
            lse_b = torch.empty_like(lse_a)
            ref = (B.qs_attn_verify if verify else B.qs_attn_draft)(cache, q, 0.1, lse=lse_a)
            out = torch.full_like(q, float("nan"))
            B.qs_attn_static(cache, q, 0.1, verify, out=out, lse=lse_b)
            torch.cuda.synchronize()
            assert torch.equal(out.view(torch.int16), ref.view(torch.int16)), (seed, verify)
            assert torch.equal(lse_a, lse_b)


def test_static_scratch_rejects_what_does_not_fit(env):
    torch, B = env["torch"], env["B"]
    cache = B.KVCache(256, 64, 8, 512, 264)
    cache.n_quant[:] = 512
    cache.n_buf[:] = 256
    q = torch.zeros((256, 16, 64, 128), dtype=torch.float16, device="cuda")
    assert B.qs_workspace_bytes(cache, 16) > B.QS_STATIC_WS_BYTES
    with pytest.raises(B.QsError) as e:
        B.qs_attn_static(cache, q, 0.1, True)
    assert e.value.code == B.QS_ERR_WORKSPACE
