"""GPU parity at the full sizes of the baseline workloads, in the launch configuration bench.py times.

Every (sequence, kv-head) unit named by a test is checked whole: the oracle recomputes the unit from the
seeds in a worker process (tests/oracle_pool.py), all its query rows - draft and verify - are compared
element by element, and the unit's planes and metadata are compared bit for bit over their full length
(by digest; a mismatch is then located array by array).  The GPU side runs under the default planner
setting and under QS_FLAG_FIXED_RANGES."""
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
    from paper_2502_10424_amd import binding as B, synth
    from tests import gpu_util as U, oracle_pool as P
    B.lib()
    return dict(torch=torch, B=B, synth=synth, U=U, P=P)


def _device_cache(env, w, layer):
    """Cache of one layer exactly as bench.py builds it: host K/V from the seeded generator, prefill
    quantization on the device, the last n_buf tokens in the fp16 buffer."""
    torch, B, synth = env["torch"], env["B"], env["synth"]
    cache = B.KVCache(w.batch, w.n_q_heads, w.n_kv_heads, w.n_quant + 128, w.n_buf + 8)
    # generate, upload and quantize one sequence at a time to bound the fp16 staging memory
    one = synth.Workload(w.name, w.config_id, 1, w.n_q_heads, w.n_kv_heads, w.ctx, w.n_buf)
    for b in range(w.batch):
        k = np.empty((1, w.n_kv_heads, w.ctx, w.head_dim), np.float16)
        v = np.empty_like(k)
        for h in range(w.n_kv_heads):
            k[0, h], v[0, h] = synth.gen_unit_kv(w.config_id, layer, b, h, w.ctx, w.head_dim)
        kd, vd = torch.from_numpy(k).cuda(), torch.from_numpy(v).cuda()
        B.qs_quantize_prefill(env["U"]._seq_view(cache, b), kd, vd, w.n_quant)
        cache.k_buf[b, :, :w.n_buf] = kd[0, :, w.n_quant:]
        cache.v_buf[b, :, :w.n_buf] = vd[0, :, w.n_quant:]
        del kd, vd, k, v
    del one
    cache.n_quant[:] = w.n_quant
    cache.n_buf[:] = w.n_buf
    torch.cuda.synchronize()
    return cache


def _check_units(env, w, units, layer=0):
    """units: (sequence, kv-head) pairs to check whole."""
    torch, B, U, P, synth = env["torch"], env["B"], env["U"], env["P"], env["synth"]
    sm = 1.0 / float(np.sqrt(w.head_dim))
    rep = w.n_q_heads // w.n_kv_heads
    _say(f"{w.name} layer {layer}: device cache")
    cache = _device_cache(env, w, layer)
    qd = torch.from_numpy(synth.gen_layer_q(w, 1, layer=layer)).cuda()
    qv = torch.from_numpy(synth.gen_layer_q(w, w.nq_verify, layer=layer)).cuda()
    outs = {}
    for tag, flags in (("queue", 0), ("fixed", B.QS_FLAG_FIXED_RANGES)):
        cache.flags = flags
        outs[tag] = (B.qs_attn_draft(cache, qd, sm).cpu().numpy(), B.qs_attn_verify(cache, qv, sm).cpu().numpy())
        assert np.isfinite(outs[tag][0]).all() and np.isfinite(outs[tag][1]).all()
    _say(f"{w.name} layer {layer}: oracle for {len(units)} units x {rep} q-heads x (1 + {w.nq_verify}) rows")
    worst = {"draft": 0.0, "verify": 0.0}
    jobs = [(w.name, layer, b, h, sm) for b, h in units]
    for ref in P.map_units(jobs):
        _, _, b, kvh, _ = ref["job"]
        e = U.export_unit(cache, b, kvh, w.n_quant)
        for name in P.PLANE_NAMES:
            assert P.digest(e[name]) == ref["digests"][name], f"{w.name}: {name} differs for unit ({b},{kvh})"
        heads = slice(kvh * rep, (kvh + 1) * rep)
        for tag, (out_d, out_v) in outs.items():
            for what, out, r in (("draft", out_d, ref["draft"]), ("verify", out_v, ref["verify"])):
                err = U.rel_err(out[b, :, heads], r)
                worst[what] = max(worst[what], err)
                assert err <= TOL, f"{w.name} {what} ({tag}) unit ({b},{kvh}): {err}"
    _say(f"{w.name} layer {layer}: worst rel err draft {worst['draft']:.2e}, verify {worst['verify']:.2e}")
    del cache
    torch.cuda.empty_cache()


def test_tiny_full(env):
    w = env["synth"].WORKLOADS["tiny"]
    _check_units(env, w, [(0, h) for h in range(w.n_kv_heads)])


def test_mha32k_full(env):
    w = env["synth"].WORKLOADS["mha32k"]
    _check_units(env, w, [(0, h) for h in range(w.n_kv_heads)])


def test_mha128k_full(env):
    """The workload bench.py's headline figures are quoted on: all 32 units, all rows."""
    w = env["synth"].WORKLOADS["mha128k"]
    _check_units(env, w, [(0, h) for h in range(w.n_kv_heads)])


def test_gqa128k_batch4_full(env):
    """All 32 units, all 20 rows (4 q-heads x 5 queries) of each."""
    w = env["synth"].WORKLOADS["gqa128k_b4"]
    _check_units(env, w, [(b, h) for b in range(w.batch) for h in range(w.n_kv_heads)])


@pytest.mark.parametrize("layer", [0, 31])
def test_stack64k_batch8_layer(env, layer):
    """First and last layer of the 32-layer stack workload (every layer has the same shape; layers differ
    by seed): sequences 0 and 7, all kv-heads, all rows."""
    w = env["synth"].WORKLOADS["stack64k_b8"]
    _check_units(env, w, [(b, h) for b in (0, 7) for h in range(w.n_kv_heads)], layer=layer)
