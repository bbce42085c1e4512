"""GPU parity: the HIP library against the CPU oracle on the same seeded inputs.

Bar: codes, scales and zeros bit-exact; attention outputs within a maximum relative error of 2e-3
per output vector (max_d |gpu - ref| / max_d |ref|; fp16 output, fp32 accumulation)."""
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
    from paper_2502_10424_amd import binding as B, synth
    from tests import gpu_util as U
    B.lib()
    return dict(torch=torch, O=O, B=B, synth=synth, U=U)


def _workload_tensors(synth, w, ctx=None):
    k, v = synth.gen_layer_kv(w, n_tokens=ctx)
    return k, v


def _run_attn(env, cache, q, sm_scale, verify):
    torch, B = env["torch"], env["B"]
    qd = torch.from_numpy(q).cuda()
    lse = torch.empty(q.shape[:3], dtype=torch.float32, device="cuda")
    fn = B.qs_attn_verify if verify else B.qs_attn_draft
    out = fn(cache, qd, sm_scale, lse=lse)
    torch.cuda.synchronize()
    return out.cpu().numpy(), lse.cpu().numpy()


def _check_attn(env, cache, oc, q, sm_scale, verify, rows=None, tag="", ref_sm=None):
    """ref_sm: softmax scale the oracle uses, if not sm_scale (a caller that rescaled its keys)."""
    U = env["U"]
    out, lse = _run_attn(env, cache, q, sm_scale, verify)
    ref, ref_lse = (oc.attn_verify if verify else oc.attn_draft)(q, sm_scale if ref_sm is None else ref_sm, rows=rows)
    if rows is not None:
        sel = np.zeros(ref.shape[:1] + ref.shape[2:3], bool)
        for b, h in rows:
            sel[b, h] = True
        out, ref = out.transpose(0, 2, 1, 3)[sel], ref.transpose(0, 2, 1, 3)[sel]
        lse, ref_lse = lse.transpose(0, 2, 1)[sel], ref_lse.transpose(0, 2, 1)[sel]
    assert np.isfinite(out).all(), tag
    err = U.rel_err(out, ref)
    lerr = float(np.abs(lse - ref_lse).max())
    _say(f"{tag}: max rel err {err:.2e}, max |lse diff| {lerr:.2e}")
    assert err <= TOL, f"{tag}: {err}"
    assert lerr <= 2e-3, f"{tag}: lse {lerr}"
    return err


# ------------------------------------------------------------------------------------------------
def test_quantize_codes_bit_exact_tiny(env):
    """Workload 'tiny': prefill-quantize 1792 tokens of 8 kv-heads, then flush the 256 buffered tokens."""
    synth, O, U, B = env["synth"], env["O"], env["U"], env["B"]
    w = synth.WORKLOADS["tiny"]
    k, v = _workload_tensors(synth, w)
    _say("tiny prefill quantize")
    cache = U.make_device_cache(k, v, w.n_q_heads, w.n_buf, q_cap=w.ctx, buf_cap=264)
    oc = O.build_cache(k, v, w.n_q_heads, w.group, w.n_buf)
    for h in range(w.n_kv_heads):
        U.assert_unit_equals_oracle(cache, oc, 0, h)
    _say("tiny flush 256")
    B.qs_quantize_flush(cache, 256)
    cache.n_quant += 256
    cache.n_buf -= 256
    oc.flush(256)
    for h in range(w.n_kv_heads):
        U.assert_unit_equals_oracle(cache, oc, 0, h)


@pytest.mark.parametrize("n_flush,n_buf,buf_cap", [(128, 428, 440), (128, 129, 264), (128, 128, 264), (256, 326, 400), (384, 517, 520)])
def test_flush_moves_long_buffers(env, n_flush, n_buf, buf_cap):
    """The rows left in the buffer after a flush move to its start: one flushed group (the flush
    kernel moves them itself, here up to three rounds of 128 rows) and several groups (separate
    kernel), with sources and destinations overlapping."""
    torch, O, U, B = env["torch"], env["O"], env["U"], env["B"]
    rng = np.random.default_rng(n_flush + n_buf)
    bsz, hkv, hq = 2, 3, 6
    t = 256 + n_buf
    k = rng.standard_normal((bsz, hkv, t, 128)).astype(np.float16)
    v = (rng.standard_normal((bsz, hkv, t, 128)) * 2 - 1).astype(np.float16)
    _say(f"flush {n_flush} of {n_buf} buffered tokens, capacity {buf_cap}")
    cache = U.make_device_cache(k, v, hq, n_buf, q_cap=256 + 512, buf_cap=buf_cap)
    oc = O.build_cache(k, v, hq, 128, n_buf)
    B.qs_quantize_flush(cache, n_flush)
    cache.n_quant += n_flush
    cache.n_buf -= n_flush
    oc.flush(n_flush)
    torch.cuda.synchronize()
    for b in range(bsz):
        for h in range(hkv):
            U.assert_unit_equals_oracle(cache, oc, b, h)


def test_flush_with_overlapping_buffer_move(env):
    """Paper cadence: G tokens are flushed while more than G stay behind (source and destination of
    the move overlap), on ragged batch lengths; repeated until the planes hold three more groups."""
    torch, synth, O, U, B = env["torch"], env["synth"], env["O"], env["U"], env["B"]
    rng = np.random.default_rng(5)
    bsz, hkv, hq = 3, 2, 4
    t = 128 * 4 + 261
    k = (rng.standard_normal((bsz, hkv, t, 128)) * rng.choice([0.05, 1, 20], (bsz, hkv, 1, 128))).astype(np.float16)
    v = (rng.standard_normal((bsz, hkv, t, 128)) + 3).astype(np.float16)
    nb = [261, 133, 261 - 128]
    # same total tokens per sequence is not required: cut each sequence to its own length
    tq = [128, 256, 384]
    ks = np.zeros_like(k); vs = np.zeros_like(v)
    for b in range(bsz):
        ks[b, :, :tq[b] + nb[b]] = k[b, :, :tq[b] + nb[b]]
        vs[b, :, :tq[b] + nb[b]] = v[b, :, :tq[b] + nb[b]]
    cache = B.KVCache(bsz, hq, hkv, 1024, 264)
    oc = O.CacheOracle(bsz, hq, hkv, 128, 128)
    kd, vd = torch.from_numpy(ks).cuda(), torch.from_numpy(vs).cuda()
    for b in range(bsz):
        sub = U._seq_view(cache, b)
        B.qs_quantize_prefill(sub, kd[b:b + 1].contiguous(), vd[b:b + 1].contiguous(), tq[b])
        cache.n_quant[b] = tq[b]
        cache.k_buf[b, :, :nb[b]] = kd[b, :, tq[b]:tq[b] + nb[b]]
        cache.v_buf[b, :, :nb[b]] = vd[b, :, tq[b]:tq[b] + nb[b]]
        cache.n_buf[b] = nb[b]
        for h in range(hkv):
            oc.append(b, h, ks[b, h, :tq[b] + nb[b]], vs[b, h, :tq[b] + nb[b]])
    # oracle: quantize each prefix in one go
    for b in range(bsz):
        for h in range(hkv):
            ku, kl, ks_, kz = O.quantize_k(oc.kbuf[b][h][:tq[b]], 128)
            vu, vl, vs_, vz = O.quantize_v(oc.vbuf[b][h][:tq[b]], 128)
            oc.ku[b][h], oc.kl[b][h], oc.ks[b][h], oc.kz[b][h] = ku, kl, ks_, kz
            oc.vu[b][h], oc.vl[b][h], oc.vs[b][h], oc.vz[b][h] = vu, vl, vs_, vz
            oc.kbuf[b][h] = oc.kbuf[b][h][tq[b]:].copy(); oc.vbuf[b][h] = oc.vbuf[b][h][tq[b]:].copy()
    _say("ragged flush 128 with overlap")
    B.qs_quantize_flush(cache, 128)
    cache.n_quant += 128; cache.n_buf -= 128
    oc.flush(128)
    torch.cuda.synchronize()
    for b in range(bsz):
        for h in range(hkv):
            U.assert_unit_equals_oracle(cache, oc, b, h)
    # attention over the ragged state, draft and verify
    q = rng.standard_normal((bsz, 5, hq, 128)).astype(np.float16)
    _check_attn(env, cache, oc, q, 0.09, True, tag="ragged verify after flush")
    _check_attn(env, cache, oc, q[:, :1].copy(), 0.09, False, tag="ragged draft after flush")


def test_quantizer_edge_values(env):
    """Constant groups, sub-resolution ranges, huge ranges, ties: still bit-exact."""
    torch, O, U, B = env["torch"], env["O"], env["U"], env["B"]
    rng = np.random.default_rng(6)
    k = rng.standard_normal((1, 2, 256, 128)).astype(np.float16)
    v = rng.standard_normal((1, 2, 256, 128)).astype(np.float16)
    k[0, 0, :128, 3] = 1.5                      # constant channel -> S := 1, codes 0
    k[0, 0, :128, 4] = 0.0; k[0, 0, 5, 4] = 6e-8   # range below the resolution of the fp16 scale
    k[0, 0, :128, 5] = np.linspace(-60000, 60000, 128).astype(np.float16)   # near the fp16 limits
    k[0, 1, :128, 7] = (np.arange(128) % 31) * 0.5                          # exact ties at .5 steps
    v[0, 0, 9, :] = -2.25
    v[0, 0, 10, :] = (np.arange(128) % 16).astype(np.float16)              # on the 4-bit grid
    v[0, 1, 11, :] = (np.arange(128) % 31) * 0.5
    v[0, 1, 12, :] = 0; v[0, 1, 12, 100] = 65504
    _say("edge-value quantize")
    cache = U.make_device_cache(k, v, 2, 0, q_cap=256, buf_cap=8)
    oc = O.build_cache(k, v, 2, 128, 0)
    for h in range(2):
        U.assert_unit_equals_oracle(cache, oc, 0, h)


def test_bulk_quantize_bit_exact(env):
    """Enough (group, unit) pairs for the prefill quantization to take its bulk kernel: 8 units x 64
    groups.  Units differ in what they stress: plain normal data, coarse grids full of exact rounding
    ties, ranges so small that the fp16 scale is subnormal, outlier channels and constant stretches."""
    torch, O, U, B = env["torch"], env["O"], env["U"], env["B"]
    rng = np.random.default_rng(61)
    t = 64 * 128
    k = (rng.standard_normal((2, 4, t, 128)) * 1.3).astype(np.float16)
    v = (rng.standard_normal((2, 4, t, 128)) * 1.3).astype(np.float16)
    k[0, 1] = (rng.integers(-40, 41, (t, 128)) * 0.125).astype(np.float16)          # ties at every step
    v[0, 1] = (rng.integers(-40, 41, (t, 128)) * 0.0625).astype(np.float16)
    k[0, 2] = (rng.integers(0, 40, (t, 128)) * 2.0 ** -24).astype(np.float16)       # subnormal scales
    v[0, 2] = (rng.integers(0, 25, (t, 128)) * 2.0 ** -24).astype(np.float16)
    k[0, 3, :, ::17] *= 30                                                           # outlier channels
    v[0, 3, ::5] = 0.75                                                              # constant tokens
    k[1, 0, 128:384, 5] = -3.0                                                       # constant channel groups
    k[1, 1] = np.clip(rng.standard_normal((t, 128)) * 20000, -65504, 65504).astype(np.float16)
    v[1, 1] = np.clip(rng.standard_normal((t, 128)) * 20000, -65504, 65504).astype(np.float16)
    _say("bulk quantize, 8 units x 64 groups")
    cache = U.make_device_cache(k, v, 4, 0, q_cap=t, buf_cap=8)
    oc = O.build_cache(k, v, 4, 128, 0)
    for b in range(2):
        for h in range(4):
            U.assert_unit_equals_oracle(cache, oc, b, h)


@pytest.mark.parametrize("verify", [False, True], ids=["draft", "verify"])
def test_attention_tiny_workload(env, verify):
    """Workload 'tiny' (GQA 32/8, ctx 2048 = 1792 quantized + 256 buffered): 1 draft query, 5 verify queries."""
    synth, O, U = env["synth"], env["O"], env["U"]
    w = synth.WORKLOADS["tiny"]
    k, v = _workload_tensors(synth, w)
    cache = U.make_device_cache(k, v, w.n_q_heads, w.n_buf, buf_cap=264)
    oc = O.build_cache(k, v, w.n_q_heads, w.group, w.n_buf)
    nq = w.nq_verify if verify else 1
    q = synth.gen_layer_q(w, nq)
    _check_attn(env, cache, oc, q, 1.0 / np.sqrt(128), verify, tag=f"tiny {'verify' if verify else 'draft'}")


@pytest.mark.parametrize("hq,hkv,nq", [(2, 2, 1), (4, 1, 2), (8, 2, 3), (16, 2, 5), (8, 1, 8), (16, 2, 7), (3, 3, 4), (2, 2, 12), (8, 2, 16)])
def test_attention_row_shapes(env, hq, hkv, nq):
    """1..64 query rows per kv-head (one to several 8-row MFMA tiles and row batches), ragged lengths,
    buffer lengths that end inside a 16-token tile."""
    O, U = env["O"], env["U"]
    rng = np.random.default_rng(100 + hq * 10 + nq)
    bsz = 2
    nb = [nq + 3, 77]
    tq = [384, 128]
    t = max(a + b for a, b in zip(tq, nb))
    k = np.zeros((bsz, hkv, t, 128), np.float16); v = np.zeros_like(k)
    cache_k, cache_v = [], []
    for b in range(bsz):
        n = tq[b] + nb[b]
        k[b, :, :n] = (rng.standard_normal((hkv, n, 128)) * 1.5).astype(np.float16)
        v[b, :, :n] = rng.standard_normal((hkv, n, 128)).astype(np.float16)
    # build per sequence (different totals): device side through ragged helper, oracle side directly
    torch, B = env["torch"], env["B"]
    cache = B.KVCache(bsz, hq, hkv, 512, 80)
    oc = O.CacheOracle(bsz, hq, hkv, 128, 128)
    kd, vd = torch.from_numpy(k).cuda(), torch.from_numpy(v).cuda()
    for b in range(bsz):
        sub = U._seq_view(cache, b)
        B.qs_quantize_prefill(sub, kd[b:b + 1].contiguous(), vd[b:b + 1].contiguous(), tq[b])
        cache.n_quant[b] = tq[b]; cache.n_buf[b] = nb[b]
        cache.k_buf[b, :, :nb[b]] = kd[b, :, tq[b]:tq[b] + nb[b]]
        cache.v_buf[b, :, :nb[b]] = vd[b, :, tq[b]:tq[b] + nb[b]]
        ob = O.build_cache(k[b:b + 1, :, :tq[b] + nb[b]], v[b:b + 1, :, :tq[b] + nb[b]], hq, 128, nb[b])
        for name in ("ku", "kl", "ks", "kz", "vu", "vl", "vs", "vz", "kbuf", "vbuf"):
            getattr(oc, name)[b] = getattr(ob, name)[0]
    q = rng.standard_normal((bsz, nq, hq, 128)).astype(np.float16)
    _check_attn(env, cache, oc, q, 0.11, True, tag=f"verify hq{hq} hkv{hkv} nq{nq}")
    if nq == 1:
        _check_attn(env, cache, oc, q, 0.11, False, tag=f"draft hq{hq} hkv{hkv}")


@pytest.mark.parametrize("hq,hkv,nq,tq", [(4, 4, 1, 0), (8, 2, 5, 0), (16, 2, 7, 0), (4, 2, 3, 1024)])
def test_attention_long_fp16_buffer(env, hq, hkv, nq, tq):
    """Buffers far longer than a decode-time one: every chunk of the buffer walks many 32-token blocks.
    With tq == 0 the cache has no quantized region at all (q_cap 0, no planes): plain fp16 attention,
    the baseline the quantized paths are compared with.  Lengths are ragged and differ per sequence."""
    torch, O, U, B = env["torch"], env["O"], env["U"], env["B"]
    rng = np.random.default_rng(300 + hq + nq)
    bsz = 2
    nb = [5003, 2311]
    cache = B.KVCache(bsz, hq, hkv, tq, 5120)
    if tq == 0:
        for name in B.PLANES:
            assert getattr(cache, name).numel() == 0
    oc = O.CacheOracle(bsz, hq, hkv, 128, 128)
    for b in range(bsz):
        n = tq + nb[b]
        k = (rng.standard_normal((1, hkv, n, 128)) * 1.5).astype(np.float16)
        v = rng.standard_normal((1, hkv, n, 128)).astype(np.float16)
        kd, vd = torch.from_numpy(k).cuda(), torch.from_numpy(v).cuda()
        if tq:
            B.qs_quantize_prefill(U._seq_view(cache, b), kd, vd, tq)
        cache.n_quant[b], cache.n_buf[b] = tq, nb[b]
        cache.k_buf[b, :, :nb[b]] = kd[0, :, tq:]
        cache.v_buf[b, :, :nb[b]] = vd[0, :, tq:]
        ob = O.build_cache(k, v, hq, 128, nb[b])
        for name in ("ku", "kl", "ks", "kz", "vu", "vl", "vs", "vz", "kbuf", "vbuf"):
            getattr(oc, name)[b] = getattr(ob, name)[0]
    q = rng.standard_normal((bsz, nq, hq, 128)).astype(np.float16)
    _check_attn(env, cache, oc, q, 0.1, True, tag=f"long buffer verify hq{hq} hkv{hkv} nq{nq} tq{tq}")
    if nq == 1:
        _check_attn(env, cache, oc, q, 0.1, False, tag=f"long buffer draft hq{hq} hkv{hkv} tq{tq}")


def _random_case(env, rng, bsz, hkv, rep, nq, max_groups, max_buf):
    """One seeded random cache (ragged quantized and buffer lengths per sequence) on both sides."""
    torch, O, U, B = env["torch"], env["O"], env["U"], env["B"]
    hq = hkv * rep
    tq = [128 * int(rng.integers(0, max_groups + 1)) for _ in range(bsz)]
    nb = [int(rng.integers(nq, max_buf + 1)) for _ in range(bsz)]
    cache = B.KVCache(bsz, hq, hkv, max(max(tq), 128), max(nb) + 3)
    oc = O.CacheOracle(bsz, hq, hkv, 128, 128)
    scale = float(rng.choice([0.05, 1.0, 30.0]))
    for b in range(bsz):
        n = tq[b] + nb[b]
        k = (rng.standard_normal((1, hkv, n, 128)) * scale).astype(np.float16)
        v = (rng.standard_normal((1, hkv, n, 128)) * scale + rng.uniform(-2, 2)).astype(np.float16)
        kd, vd = torch.from_numpy(k).cuda(), torch.from_numpy(v).cuda()
        if tq[b]:
            B.qs_quantize_prefill(U._seq_view(cache, b), kd, vd, tq[b])
        cache.n_quant[b], cache.n_buf[b] = tq[b], nb[b]
        cache.k_buf[b, :, :nb[b]] = kd[0, :, tq[b]:]
        cache.v_buf[b, :, :nb[b]] = vd[0, :, tq[b]:]
        ob = O.build_cache(k, v, hq, 128, nb[b])
        for name in ("ku", "kl", "ks", "kz", "vu", "vl", "vs", "vz", "kbuf", "vbuf"):
            getattr(oc, name)[b] = getattr(ob, name)[0]
    q = (rng.standard_normal((bsz, nq, hq, 128)) / scale).astype(np.float16)
    return cache, oc, q, f"B{bsz} Hkv{hkv} rep{rep} nq{nq} tq{tq} nb{nb} scale{scale}"


def test_attention_random_shapes(env):
    """Seeded sweep over batch, head counts, GQA ratios, query counts, ragged lengths and magnitudes:
    every kernel instantiation and planner branch (few / many units, chunk counts 1..many) is hit."""
    rng = np.random.default_rng(4242)
    for case in range(24):
        bsz = int(rng.integers(1, 4))
        hkv = int(rng.choice([1, 2, 3, 8]))
        rep = int(rng.choice([1, 2, 4, 8]))
        nq = int(rng.integers(1, 9))
        cache, oc, q, tag = _random_case(env, rng, bsz, hkv, rep, nq, max_groups=6, max_buf=140)
        _check_attn(env, cache, oc, q, 0.09, True, tag=f"random {case} verify {tag}")
        if nq == 1 or case % 3 == 0:
            _check_attn(env, cache, oc, q[:, -1:], 0.09, False, tag=f"random {case} draft {tag}")


def test_attention_maximum_batch(env):
    """256 sequences (the most the by-value length arrays hold), different lengths each: 512 units."""
    B = env["B"]
    rng = np.random.default_rng(64)
    cache, oc, q, tag = _random_case(env, rng, B.QS_MAX_BATCH, 2, 2, 2, max_groups=2, max_buf=40)
    _check_attn(env, cache, oc, q, 0.09, True, tag=f"batch {B.QS_MAX_BATCH} verify {tag[:40]}")
    _check_attn(env, cache, oc, q[:, -1:], 0.09, False, tag=f"batch {B.QS_MAX_BATCH} draft {tag[:40]}")


@pytest.mark.parametrize("hq,hkv,nq", [(4, 2, 1), (8, 2, 5), (16, 2, 5)])
def test_paged_cache_matches_oracle(env, hq, hkv, nq):
    """Group-table mode: the 128-token groups of every unit live at shuffled places of a shared pool.
    Prefill, a flush (which appends through the table) and both attention passes must give exactly
    what the oracle gives; the oracle knows nothing about placement."""
    torch, O, U, B = env["torch"], env["O"], env["U"], env["B"]
    rng = np.random.default_rng(900 + hq + nq)
    bsz, tq, nb, q_cap = 3, 5 * 128, 128 + nq + 9, 8 * 128
    n_logical = bsz * hkv * (q_cap // 128)
    pool = n_logical + 7
    cache = B.KVCache(bsz, hq, hkv, q_cap, nb + 8, pool_groups=pool)
    table = rng.permutation(pool)[:n_logical].astype(np.int32).reshape(bsz, hkv, q_cap // 128)
    cache.group_table.copy_(torch.from_numpy(table))
    cache.upper.fill_(0xA5)                  # whatever sits in unused pool places must not matter
    cache.lower.fill_(0x5A)
    k = (rng.standard_normal((bsz, hkv, tq + nb, 128)) * 1.5).astype(np.float16)
    v = rng.standard_normal((bsz, hkv, tq + nb, 128)).astype(np.float16)
    kd, vd = torch.from_numpy(k).cuda(), torch.from_numpy(v).cuda()
    B.qs_quantize_prefill(cache, kd, vd, tq)
    cache.n_quant[:] = tq
    cache.k_buf[:, :, :nb] = kd[:, :, tq:]
    cache.v_buf[:, :, :nb] = vd[:, :, tq:]
    cache.n_buf[:] = nb
    oc = O.build_cache(k, v, hq, 128, nb)
    q = rng.standard_normal((bsz, nq, hq, 128)).astype(np.float16)
    _check_attn(env, cache, oc, q, 0.1, True, tag=f"paged verify hq{hq} hkv{hkv} nq{nq}")
    _check_attn(env, cache, oc, q[:, -1:], 0.1, False, tag=f"paged draft hq{hq} hkv{hkv}")
    B.qs_quantize_flush(cache, 128)          # group 5 of every unit goes to its table entry
    cache.n_quant += 128
    cache.n_buf -= 128
    oc.flush(128)
    for b in range(bsz):
        for h in range(hkv):
            U.assert_unit_equals_oracle(cache, oc, b, h)
    _check_attn(env, cache, oc, q, 0.1, True, tag=f"paged verify after flush hq{hq} hkv{hkv} nq{nq}")
    # pool places no table entry points at are untouched
    used = np.zeros(pool, bool)
    used[table.reshape(-1)] = True
    up = cache.upper.view(pool, -1).cpu().numpy()
    assert (up[~used] == 0xA5).all()


def test_attention_degenerate_cases(env):
    """Buffer only (no quantized tokens); buffer holding exactly the nq query tokens; peaked softmax."""
    O, U = env["O"], env["U"]
    rng = np.random.default_rng(7)
    k = rng.standard_normal((1, 2, 200, 128)).astype(np.float16)
    v = rng.standard_normal((1, 2, 200, 128)).astype(np.float16)
    q = rng.standard_normal((1, 4, 4, 128)).astype(np.float16)
    cache = U.make_device_cache(k, v, 4, 200, q_cap=128, buf_cap=256)
    oc = O.build_cache(k, v, 4, 128, 200)
    _check_attn(env, cache, oc, q, 0.1, True, tag="buffer only verify")
    _check_attn(env, cache, oc, q[:, :1].copy(), 0.1, False, tag="buffer only draft")
    k2 = rng.standard_normal((1, 2, 256 + 4, 128)).astype(np.float16)
    v2 = rng.standard_normal((1, 2, 256 + 4, 128)).astype(np.float16)
    cache = U.make_device_cache(k2, v2, 4, 4, buf_cap=8)
    oc = O.build_cache(k2, v2, 4, 128, 4)
    _check_attn(env, cache, oc, q, 0.1, True, tag="buffer == nq tokens")
    # one key dominates: scores up to ~ +40 above the rest
    k3 = k2.copy(); k3[0, :, 100, :] = (q[0, 0, 0] * 2).astype(np.float16)
    cache = U.make_device_cache(k3, v2, 4, 4, buf_cap=8)
    oc = O.build_cache(k3, v2, 4, 128, 4)
    _check_attn(env, cache, oc, q, 0.15, True, tag="peaked softmax")


def test_attention_large_and_small_magnitudes(env):
    """Queries and keys far from unit scale: q * S would overflow fp16 without the per-row power-of-two
    prescale of the queries (|q| ~ 3000, key scales ~ 40), and tiny queries must not lose precision."""
    O, U = env["O"], env["U"]
    rng = np.random.default_rng(21)
    t, nb = 384, 19
    for qmag, kmag in ((3000.0, 100.0), (1e-3, 0.05), (20000.0, 1.0)):
        k = (rng.standard_normal((1, 2, t + nb, 128)) * kmag).astype(np.float16)
        v = (rng.standard_normal((1, 2, t + nb, 128)) * 7).astype(np.float16)
        q = np.clip(rng.standard_normal((1, 3, 4, 128)) * qmag, -60000, 60000).astype(np.float16)
        q[0, 1, 2] = 0                                  # an all-zero query row: uniform attention
        cache = U.make_device_cache(k, v, 4, nb, buf_cap=32)
        oc = O.build_cache(k, v, 4, 128, nb)
        sm = 2.0 / (qmag * kmag * np.sqrt(128))
        _check_attn(env, cache, oc, q, sm, True, tag=f"verify |q|~{qmag:g} |k|~{kmag:g}")
        _check_attn(env, cache, oc, q[:, :1].copy(), sm, False, tag=f"draft |q|~{qmag:g} |k|~{kmag:g}")


@pytest.mark.parametrize("vmag", [1e-3, 1e-2, 0.1, 100.0, 3000.0])
def test_attention_value_magnitudes(env, vmag):
    """Values six orders of magnitude apart, flat and peaked softmax.  p * S_V travels as fp16; the
    reference exponent of the online softmax follows the largest value scale, so small value ranges
    keep their bits.  (Below about 1e-3 the fp16 *output* itself runs into subnormals.)"""
    O, U = env["O"], env["U"]
    rng = np.random.default_rng(int(vmag * 1000) + 3)
    t, nb = 1024, 19
    for qmag in (0.3, 4.0):
        k = rng.standard_normal((1, 2, t + nb, 128)).astype(np.float16)
        v = (rng.standard_normal((1, 2, t + nb, 128)) * vmag).astype(np.float16)
        q = (rng.standard_normal((1, 3, 4, 128)) * qmag).astype(np.float16)
        cache = U.make_device_cache(k, v, 4, nb, buf_cap=32)
        oc = O.build_cache(k, v, 4, 128, nb)
        _check_attn(env, cache, oc, q, 0.088, True, tag=f"verify |v|~{vmag:g} |q|~{qmag:g}")
        _check_attn(env, cache, oc, q[:, :1].copy(), 0.088, False, tag=f"draft |v|~{vmag:g} |q|~{qmag:g}")


@pytest.mark.parametrize("kmag", [1e-4, 1e-3, 1e-2, 0.1, 100.0, 3000.0])
def test_attention_key_magnitudes(env, kmag):
    """Keys seven orders of magnitude apart with a softmax scale that keeps the scores at O(1), flat and
    peaked.  q * S_K travels as two fp16 numbers, q normalised to at most 1 per row and the scales of a
    group of keys lifted by a power of two taken from the largest of them, so neither large nor tiny
    key spreads cost accuracy (1e-4: the scales themselves are fp16 subnormals)."""
    O, U = env["O"], env["U"]
    rng = np.random.default_rng(int(kmag * 10) + 11)
    t, nb = 1024, 19
    for peak in (0.5, 3.0):
        k = (rng.standard_normal((1, 2, t + nb, 128)) * kmag).astype(np.float16)
        v = rng.standard_normal((1, 2, t + nb, 128)).astype(np.float16)
        q = rng.standard_normal((1, 3, 4, 128)).astype(np.float16)
        sm = peak / (kmag * np.sqrt(128))
        cache = U.make_device_cache(k, v, 4, nb, buf_cap=32)
        oc = O.build_cache(k, v, 4, 128, nb)
        _check_attn(env, cache, oc, q, sm, True, tag=f"verify |k|~{kmag:g} peak {peak}")
        _check_attn(env, cache, oc, q[:, :1].copy(), sm, False, tag=f"draft |k|~{kmag:g} peak {peak}")


@pytest.mark.parametrize("kmag", [1e-2, 1e-3])
def test_attention_tiny_keys_through_the_documented_rescaling(env, kmag):
    """Scaling fp16 keys by a power of two scales S and Z by the same and leaves the codes alone, so a cache
    that holds the lifted keys, called with sm_scale divided by the lift, answers the unscaled problem, which
    is what the oracle computes here.  (What a caller with tiny keys had to do before the kernel lifted the
    key scales itself; kept as a property of the quantizer and the attention calls.)"""
    O, U = env["O"], env["U"]
    rng = np.random.default_rng(int(1e4 * kmag) + 3)
    t, nb = 1024, 19
    lift = 2.0 ** np.ceil(np.log2(1.0 / kmag))
    for peak in (0.5, 3.0):
        k = (rng.standard_normal((1, 2, t + nb, 128)) * kmag).astype(np.float16)
        v = rng.standard_normal((1, 2, t + nb, 128)).astype(np.float16)
        q = rng.standard_normal((1, 3, 4, 128)).astype(np.float16)
        sm = peak / (kmag * np.sqrt(128))
        k_lifted = (k.astype(np.float32) * np.float32(lift)).astype(np.float16)
        assert np.array_equal(k_lifted.astype(np.float32), k.astype(np.float32) * np.float32(lift))   # exact
        cache = U.make_device_cache(k_lifted, v, 4, nb, buf_cap=32)
        oc = O.build_cache(k, v, 4, 128, nb)                   # the problem as posed
        _check_attn(env, cache, oc, q, sm / lift, True, ref_sm=sm, tag=f"verify |k|~{kmag:g} x {lift:g}, peak {peak}")
        _check_attn(env, cache, oc, q[:, :1].copy(), sm / lift, False, ref_sm=sm, tag=f"draft |k|~{kmag:g} x {lift:g}, peak {peak}")


def test_attention_value_scale_jumps(env):
    """Value scales that change by many orders of magnitude inside one chunk: near-zero values at the
    start (an attention-sink-like prefix), a stretch 2000 times larger than the rest, constant rows.
    The reference exponent has to rise in mid-stream and rescale what was accumulated before."""
    O, U = env["O"], env["U"]
    rng = np.random.default_rng(77)
    t, nb = 2048, 21
    k = rng.standard_normal((2, 1, t + nb, 128)).astype(np.float16)
    v = (rng.standard_normal((2, 1, t + nb, 128)) * 0.5).astype(np.float16)
    v[:, :, :70] *= np.float16(1e-4)            # tiny scales first
    v[:, :, 700:900] *= np.float16(2000.0)      # then a jump of seven orders of magnitude
    v[0, :, 1000:1010] = 0.25                   # constant rows: S := 1
    v[1, :, 1500:] *= np.float16(1e-3)          # and small again (the exponent stays up)
    q = (rng.standard_normal((2, 4, 2, 128)) * 1.5).astype(np.float16)
    cache = U.make_device_cache(k, v, 2, nb, buf_cap=32)
    oc = O.build_cache(k, v, 2, 128, nb)
    _check_attn(env, cache, oc, q, 0.088, True, tag="verify, value scale jumps")
    _check_attn(env, cache, oc, q[:, :1].copy(), 0.088, False, tag="draft, value scale jumps")


def test_attention_lossless_grid_matches_unquantized(env):
    """Property that holds without the oracle's quantizer: 4-bit-grid data through the draft pass equals
    plain fp64 attention over the original tensors."""
    torch, U = env["torch"], env["U"]
    rng = np.random.default_rng(8)
    t, nb = 512, 40
    kk = rng.integers(0, 16, (1, 2, t + nb, 128)); kk[:, :, 0::128] = 0; kk[:, :, 1::128] = 15
    vv = rng.integers(0, 16, (1, 2, t + nb, 128)); vv[..., 0] = 0; vv[..., 1] = 15
    k = (-1.0 + kk * 0.125).astype(np.float16)
    v = (0.5 + vv * 0.25).astype(np.float16)
    q = rng.standard_normal((1, 1, 4, 128)).astype(np.float16)
    cache = U.make_device_cache(k, v, 4, nb, buf_cap=64)
    out, _ = _run_attn(env, cache, q, 0.08, False)
    kt = torch.tensor(k.astype(np.float64)).repeat_interleave(2, dim=1)
    vt = torch.tensor(v.astype(np.float64)).repeat_interleave(2, dim=1)
    qt = torch.tensor(q.astype(np.float64)).permute(0, 2, 1, 3)
    ref = torch.nn.functional.scaled_dot_product_attention(qt, kt, vt, scale=0.08).permute(0, 2, 1, 3).numpy()
    assert U.rel_err(out, ref) <= TOL


def test_split_count_invariance(env):
    """The result must not depend on how the quantized region is cut into chunks: the same cache with
    different batch sizes (hence different chunk counts per unit) gives the same outputs per sequence."""
    synth, U, B, torch = env["synth"], env["U"], env["B"], env["torch"]
    rng = np.random.default_rng(9)
    k1 = (rng.standard_normal((1, 1, 128 * 40 + 64, 128))).astype(np.float16)
    v1 = rng.standard_normal(k1.shape).astype(np.float16)
    q1 = rng.standard_normal((1, 3, 2, 128)).astype(np.float16)
    reps = 64   # 64 units -> far fewer chunks per unit than a single unit gets
    cache1 = U.make_device_cache(k1, v1, 2, 64)
    cacheN = U.make_device_cache(np.repeat(k1, reps, 0), np.repeat(v1, reps, 0), 2, 64)
    o1, _ = _run_attn(env, cache1, q1, 0.09, True)
    oN, _ = _run_attn(env, cacheN, np.repeat(q1, reps, 0), 0.09, True)
    # identical sequences agree to rounding only: which wave takes which group is decided at run time
    assert U.rel_err(oN, np.repeat(oN[:1], reps, 0).astype(np.float64)) <= 2e-3   # a step or two of the fp16 output
    assert U.rel_err(oN[:1], o1.astype(np.float64)) <= 1e-3
