"""GPU parity over a whole speculative-decoding loop (Algorithm 1) with the buffer policy of Section 4.3.2:
gamma draft steps (append one token, draft attention), one target step (gamma + 1 queries over the same
tokens), simulated acceptance with rollback of rejected tokens, and a flush of G tokens whenever the
verified buffer holds 2G or more.  Every attention output is compared with the oracle, and at the end the
planes must equal the oracle's bit for bit (append-only: no group is ever re-quantized).
Also: the same calls captured in a HIP graph and replayed must reproduce the eager results."""
import sys

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

TOL = 2e-3
G = 128


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
    from tests import gpu_util as U
    B.lib()
    return dict(torch=torch, O=O, B=B, U=U)


@pytest.mark.parametrize("gamma,hq,hkv,lockstep", [(4, 4, 2, False), (1, 2, 2, False), (6, 8, 2, False), (3, 4, 1, True)])
def test_speculation_loop_with_rollback(env, gamma, hq, hkv, lockstep):
    torch, O, B, U = env["torch"], env["O"], env["B"], env["U"]
    rng = np.random.default_rng(1000 + gamma)
    bsz = 2
    # prompt lengths differ per sequence (each flushes alone) unless lockstep (both flush in one call)
    prefill = [3 * G + 40, 3 * G + 40] if lockstep else [3 * G + 40, 2 * G + 7]
    nq = gamma + 1
    buf_cap = 2 * G + nq                                 # a cycle starts with n_buf < 2G and adds at most gamma + 1
    sm = 0.1
    n_cycles = 400 // nq + 20                            # enough tokens for at least one flush per sequence
    cache = B.KVCache(bsz, hq, hkv, 16 * G, buf_cap)
    oc = O.CacheOracle(bsz, hq, hkv, 128, G)
    draw = lambda *shape: (rng.standard_normal(shape) * 1.3).astype(np.float16)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    names = ("ku", "kl", "ks", "kz", "vu", "vl", "vs", "vz", "kbuf", "vbuf")

    def oracle_flush_one(b):
        single = O.CacheOracle(1, hq, hkv, 128, G)
        for name in names:
            getattr(single, name)[0] = getattr(oc, name)[b]
        single.flush(G)
        for name in names:
            getattr(oc, name)[b] = getattr(single, name)[0]

    def oracle_append(tok_k, tok_v):                     # tok_*: [bsz, n_new, hkv, 128]
        for b in range(bsz):
            for h in range(hkv):
                oc.append(b, h, tok_k[b, :, h], tok_v[b, :, h])

    # ---- prefill: quantize in batches of G so that G <= n_buf < 2G stay in full precision ----
    for b in range(bsz):
        k, v = draw(1, hkv, prefill[b], 128), draw(1, hkv, prefill[b], 128)
        nb = prefill[b] - ((prefill[b] - G) // G) * G
        tq = prefill[b] - nb
        assert G <= nb < 2 * G and tq % G == 0
        ob = O.build_cache(k, v, hq, G, nb)
        for name in names:
            getattr(oc, name)[b] = getattr(ob, name)[0]
        kd, vd = dev(k), dev(v)
        B.qs_quantize_prefill(U._seq_view(cache, b), kd, vd, tq)
        cache.n_quant[b] = tq
        cache.k_buf[b, :, :nb] = kd[0, :, tq:]
        cache.v_buf[b, :, :nb] = vd[0, :, tq:]
        cache.n_buf[b] = nb

    worst, n_flush_all, n_flush_one = 0.0, 0, 0
    for cycle in range(n_cycles):
        # ---- gamma draft passes: each appends its input token's K/V, then attends with the upper plane ----
        kd_, vd_ = draw(bsz, gamma, hkv, 128), draw(bsz, gamma, hkv, 128)
        for i in range(gamma):
            B.qs_append(cache, dev(kd_[:, i:i + 1]), dev(vd_[:, i:i + 1]))
            cache.n_buf += 1
            oracle_append(kd_[:, i:i + 1], vd_[:, i:i + 1])
            q = draw(bsz, 1, hq, 128)
            out = B.qs_attn_draft(cache, dev(q), sm).cpu().numpy()
            ref, _ = oc.attn_draft(q, sm)
            worst = max(worst, U.rel_err(out, ref))
        # ---- target pass: its own K/V for the same gamma positions plus one more replace the draft's ----
        cache.n_buf -= gamma
        for b in range(bsz):
            oc.reject(b, gamma)
        kt, vt = draw(bsz, nq, hkv, 128), draw(bsz, nq, hkv, 128)
        B.qs_append(cache, dev(kt), dev(vt))
        cache.n_buf += nq
        oracle_append(kt, vt)
        q = draw(bsz, nq, hq, 128)
        out = B.qs_attn_verify(cache, dev(q), sm).cpu().numpy()
        ref, _ = oc.attn_verify(q, sm)
        worst = max(worst, U.rel_err(out, ref))
        # ---- simulated acceptance: v of the gamma drafts survive; the rest leave the buffer ----
        drops = [gamma - int(rng.binomial(gamma, 0.8)) for _ in range(bsz)]
        for b in range(bsz):
            drop = drops[0] if lockstep else drops[b]
            cache.n_buf[b] -= drop
            oc.reject(b, drop)
        # ---- flush the older half of every buffer that holds 2G verified tokens ----
        full = [b for b in range(bsz) if cache.n_buf[b] >= 2 * G]
        if len(full) == bsz:
            B.qs_quantize_flush(cache, G)
            oc.flush(G)
            n_flush_all += 1
        else:
            for b in full:                               # one sequence alone, through a view of its storage
                sub = U._seq_view(cache, b)
                sub.n_quant[0], sub.n_buf[0] = cache.n_quant[b], cache.n_buf[b]
                B.qs_quantize_flush(sub, G)
                oracle_flush_one(b)
                n_flush_one += 1
        for b in full:
            cache.n_quant[b] += G
            cache.n_buf[b] -= G
        for b in range(bsz):
            assert cache.n_buf[b] == oc.n_buf(b) and G <= cache.n_buf[b] < 2 * G
            assert cache.n_quant[b] == oc.n_quant(b)
    _say(f"gamma {gamma}: {n_cycles} cycles, worst rel err {worst:.2e}, flushes {n_flush_all} joint + {n_flush_one} single")
    assert worst <= TOL
    assert n_flush_all + n_flush_one >= 2 and (n_flush_all > 0) == lockstep
    torch.cuda.synchronize()
    for b in range(bsz):
        for h in range(hkv):
            U.assert_unit_equals_oracle(cache, oc, b, h)


def test_hip_graph_replay_matches_eager(env):
    """Draft, verify and flush captured in one HIP graph; replayed three times with eager work and
    synchronizations in between; every replay must reproduce the eager results exactly."""
    torch, B, U = env["torch"], env["B"], env["U"]
    B.KVCache.default_flags = B.QS_FLAG_FIXED_RANGES   # exact comparison below: fixed ranges whatever the planner would pick
    try:
        _graph_replay_case(torch, B, U)
    finally:
        B.KVCache.default_flags = 0


def _graph_replay_case(torch, B, U):
    rng = np.random.default_rng(77)
    t, nb = 6 * G, 2 * G
    k = rng.standard_normal((2, 2, t + nb, 128)).astype(np.float16)
    v = rng.standard_normal((2, 2, t + nb, 128)).astype(np.float16)
    qd = torch.from_numpy(rng.standard_normal((2, 1, 4, 128)).astype(np.float16)).cuda()
    qv = torch.from_numpy(rng.standard_normal((2, 5, 4, 128)).astype(np.float16)).cuda()

    def fresh():
        return U.make_device_cache(k, v, 4, nb, q_cap=t + G, buf_cap=nb + 8)

    # eager reference
    c = fresh()
    ws = torch.zeros(B.qs_workspace_bytes(c, 5), dtype=torch.uint8, device="cuda")
    e_d = B.qs_attn_draft(c, qd, 0.1, workspace=ws).clone()
    e_v = B.qs_attn_verify(c, qv, 0.1, workspace=ws).clone()
    B.qs_quantize_flush(c, G)
    torch.cuda.synchronize()
    checked = B.PLANES + ("k_buf",)
    e_planes = [getattr(c, n).clone() for n in checked]

    c2 = fresh()
    o_d, o_v = torch.empty_like(qd), torch.empty_like(qv)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):          # warm-up on a non-default stream, as capture uses one
        B.qs_attn_draft(c2, qd, 0.1, out=o_d, workspace=ws, stream=side)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        cs = torch.cuda.current_stream()   # the capturing stream: the library launches on the stream it is given
        B.qs_attn_draft(c2, qd, 0.1, out=o_d, workspace=ws, stream=cs)
        B.qs_attn_verify(c2, qv, 0.1, out=o_v, workspace=ws, stream=cs)
        B.qs_quantize_flush(c2, G, stream=cs)
    for rep in range(3):
        # restore the state the graph starts from (the flush inside it moves the buffer)
        c3 = fresh()
        for n in B.PLANES + ("k_buf", "v_buf"):
            getattr(c2, n).copy_(getattr(c3, n))
        o_d.zero_(); o_v.zero_()
        (torch.ones(1000, device="cuda") * rep).sum().item()      # unrelated eager work + a synchronization
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(o_d, e_d) and torch.equal(o_v, e_v), f"replay {rep}"
        for n, ref in zip(checked, e_planes):
            assert torch.equal(getattr(c2, n), ref), f"replay {rep}: {n}"
