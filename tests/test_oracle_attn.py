"""Pins of the oracle's attention and cache state machine (Appendix A, Algorithm 1, Section 4.3.2)
against a library routine (float64 torch SDPA with an explicit mask), pure-Python brute force,
closed forms and invariants."""
import math

import numpy as np
import torch

from oracle import quantspec_oracle as O


def _sdpa(q, keys, vals, n_vis, sm_scale, rep):
    """Library reference: q [nq,Hq,D]; keys/vals [Hkv,T,D] float64; n_vis[i] visible tokens of query i."""
    nq, hq, d = q.shape
    t = keys.shape[1]
    qt = torch.tensor(q.astype(np.float64)).permute(1, 0, 2)[None]              # [1,Hq,nq,D]
    kt = torch.tensor(keys).repeat_interleave(rep, dim=0)[None]                 # [1,Hq,T,D]
    vt = torch.tensor(vals).repeat_interleave(rep, dim=0)[None]
    mask = torch.arange(t)[None, :] < torch.tensor(n_vis)[:, None]              # [nq,T]
    o = torch.nn.functional.scaled_dot_product_attention(qt, kt, vt, attn_mask=mask[None, None], scale=sm_scale)
    return o[0].permute(1, 0, 2).numpy()                                        # [nq,Hq,D]


def _rand_cache(rng, batch, hq, hkv, d, g, tq, nb, scale=1.0):
    k = (rng.standard_normal((batch, hkv, tq + nb, d)) * scale).astype(np.float16)
    v = rng.standard_normal((batch, hkv, tq + nb, d)).astype(np.float16)
    return k, v, O.build_cache(k, v, hq, g, nb)


def test_buffer_only_matches_library_attention_mha_and_gqa():
    rng = np.random.default_rng(10)
    for hq, hkv in ((4, 4), (8, 2)):
        k, v, c = _rand_cache(rng, 2, hq, hkv, 16, 16, 0, 37)
        nq = 5
        q = rng.standard_normal((2, nq, hq, 16)).astype(np.float16)
        for fn in (c.attn_draft, c.attn_verify):
            out, _ = fn(q, 0.25)
            for b in range(2):
                ref = _sdpa(q[b], k[b].astype(np.float64), v[b].astype(np.float64),
                            [37 - nq + i + 1 for i in range(nq)], 0.25, hq // hkv)
                assert np.allclose(out[b], ref, rtol=1e-12, atol=1e-13)


def test_lossless_grid_cache_matches_unquantized_library_attention():
    """4-bit-grid data: the draft pass equals attention over the original tensors;
    8-bit-grid data (no +8 residual): the verify pass does."""
    rng = np.random.default_rng(11)
    g = d = 16
    tq, nb, hq, hkv = 48, 9, 4, 2
    kk = rng.integers(0, 16, (1, hkv, tq + nb, d)); kk[:, :, 0::g, :] = 0; kk[:, :, 1::g, :] = 15
    vv = rng.integers(0, 16, (1, hkv, tq + nb, d)); vv[..., 0] = 0; vv[..., 1] = 15
    k4 = (-1.0 + kk * 0.125).astype(np.float16)
    v4 = (0.5 + vv * 0.25).astype(np.float16)
    c = O.build_cache(k4, v4, hq, g, nb)
    q = rng.standard_normal((1, 3, hq, d)).astype(np.float16)
    vis = [tq + nb - 3 + i + 1 for i in range(3)]
    ref = _sdpa(q[0], k4[0].astype(np.float64), v4[0].astype(np.float64), vis, 0.3, 2)
    assert np.allclose(c.attn_draft(q, 0.3)[0][0], ref, rtol=1e-12, atol=1e-13)
    assert np.allclose(c.attn_verify(q, 0.3)[0][0], ref, rtol=1e-12, atol=1e-13)
    c8k = rng.integers(0, 15, (1, hkv, tq + nb, d)) * 16 + rng.integers(-7, 8, (1, hkv, tq + nb, d))
    c8k = np.clip(c8k, 0, 240); c8k[:, :, 0::g, :] = 0; c8k[:, :, 1::g, :] = 240
    c8v = np.clip(rng.integers(0, 15, c8k.shape) * 16 + rng.integers(-7, 8, c8k.shape), 0, 240)
    c8v[..., 0] = 0; c8v[..., 1] = 240
    k8 = (2.0 + c8k / 128.0).astype(np.float16)
    v8 = (-1.0 + c8v / 64.0).astype(np.float16)
    assert np.array_equal(k8.astype(np.float64), 2.0 + c8k / 128.0)
    c = O.build_cache(k8, v8, hq, g, nb)
    ref = _sdpa(q[0], k8[0].astype(np.float64), v8[0].astype(np.float64), vis, 0.3, 2)
    assert np.allclose(c.attn_verify(q, 0.3)[0][0], ref, rtol=1e-12, atol=1e-13)
    assert not np.allclose(c.attn_draft(q, 0.3)[0][0], ref, rtol=1e-6, atol=1e-6)   # 4 bits do lose here


def test_matches_library_attention_on_decoded_cache():
    rng = np.random.default_rng(12)
    g = d = 32
    tq, nb, hq, hkv, nq = 96, 40, 6, 2, 4
    k, v, c = _rand_cache(rng, 1, hq, hkv, d, g, tq, nb, scale=2.0)
    q = rng.standard_normal((1, nq, hq, d)).astype(np.float16)
    vis = [tq + nb - nq + i + 1 for i in range(nq)]
    for lower, fn in ((False, c.attn_draft), (True, c.attn_verify)):
        keys = np.stack([np.concatenate([c.decoded(0, h, lower)[0], c.kbuf[0][h].astype(np.float64)]) for h in range(hkv)])
        vals = np.stack([np.concatenate([c.decoded(0, h, lower)[1], c.vbuf[0][h].astype(np.float64)]) for h in range(hkv)])
        ref = _sdpa(q[0], keys, vals, vis, 0.2, hq // hkv)
        assert np.allclose(fn(q, 0.2)[0][0], ref, rtol=1e-12, atol=1e-13)
    # the buffer part of keys is the original fp16 data, untouched
    assert np.array_equal(c.kbuf[0][1], k[0, 1, tq:])


def test_bruteforce_python_loops_tiny():
    """G = D = 4, integers small enough to follow by hand; every step redone with Python floats."""
    k = np.array([[[[0, 4, 8, 1], [15, 4, 0, 2], [3, 9, 2, 3], [7, 19, 4, 16],      # group 0 (quantized)
                    [1, 1, 1, 1], [2, 0, 1, 3]]]], np.float16)                       # buffer (2 tokens)
    v = np.array([[[[0, 15, 5, 10], [30, 0, 10, 20], [1, 2, 3, 16], [4, 4, 4, 34],
                    [1, 0, 0, 0], [0, 1, 0, 0]]]], np.float16)
    c = O.build_cache(k, v, 1, 4, 2)
    q = np.array([[[[1, 0, -1, 0.5]], [[0.5, 0.5, 0, 0]]]], np.float16)              # nq = 2
    sm = 0.5
    for lower, fn in ((False, c.attn_draft), (True, c.attn_verify)):
        out, lse = fn(q, sm)
        # decode by hand
        keys, vals = [], []
        for t in range(4):
            krow, vrow = [], []
            vmin, vmax = min(map(float, v[0, 0, t])), max(map(float, v[0, 0, t]))
            sv = float(np.float16((vmax - vmin) / 15)) or 1.0
            for ch in range(4):
                col = [float(k[0, 0, tt, ch]) for tt in range(4)]
                sk = float(np.float16((max(col) - min(col)) / 15)) or 1.0
                for (x, s, z, dst) in ((float(k[0, 0, t, ch]), sk, min(col), krow), (float(v[0, 0, t, ch]), sv, vmin, vrow)):
                    u = min(15, max(0, round((x - z) / s)))       # Python round = ties to even
                    e = x - (u * s + z)
                    l = min(7, max(-8, round(e / (s / 16))))
                    dst.append(u * s + z + (l * s / 16 if lower else 0.0))
            keys.append(krow); vals.append(vrow)
        for t in (4, 5):
            keys.append([float(a) for a in k[0, 0, t]]); vals.append([float(a) for a in v[0, 0, t]])
        for i in range(2):
            nvis = 4 + 2 - 2 + i + 1
            s = [sm * sum(float(q[0, i, 0, dd]) * keys[t][dd] for dd in range(4)) for t in range(nvis)]
            m = max(s)
            w = [math.exp(a - m) for a in s]
            den = sum(w)
            o = [sum(w[t] * vals[t][dd] for t in range(nvis)) / den for dd in range(4)]
            assert np.allclose(out[0, i, 0], o, rtol=1e-12, atol=1e-12)
            assert abs(lse[0, i, 0] - (m + math.log(den))) < 1e-12


def test_softmax_properties():
    rng = np.random.default_rng(13)
    g = d = 16
    tq, nb = 64, 20
    k, v, c = _rand_cache(rng, 1, 2, 2, d, g, tq, nb)
    q = rng.standard_normal((1, 1, 2, d)).astype(np.float16)
    # weights sum to one: recompute scores independently, use the oracle's log-normaliser
    out, lse = c.attn_draft(q, 0.25)
    for h in range(2):
        kd, vd = c.decoded(0, h, False)
        keys = np.concatenate([kd, c.kbuf[0][h].astype(np.float64)])
        s = 0.25 * keys @ q[0, 0, h].astype(np.float64)
        assert abs(np.exp(s - lse[0, 0, h]).sum() - 1.0) < 1e-12
    # q = 0 -> uniform weights -> mean of the decoded values over the visible tokens
    out0, lse0 = c.attn_verify(np.zeros_like(q), 0.25)
    for h in range(2):
        vd = np.concatenate([c.decoded(0, h, True)[1], c.vbuf[0][h].astype(np.float64)])
        assert np.allclose(out0[0, 0, h], vd.mean(axis=0), rtol=1e-12)
        assert abs(lse0[0, 0, h] - math.log(tq + nb)) < 1e-12
    # constant value rows -> the output is that row whatever the keys are
    # (the row sits on the 4-bit grid, so quantized and buffered tokens carry the same row)
    row = (-1.0 + 0.25 * np.arange(d)).astype(np.float16)
    vconst = np.broadcast_to(row, v.shape).copy()
    cc = O.build_cache(k, vconst, 2, g, nb)
    outc, _ = cc.attn_draft(q, 0.25)
    assert np.allclose(outc[0, 0], row.astype(np.float64)[None].repeat(2, 0), rtol=1e-12, atol=1e-12)
    # one dominant key: output ~ its decoded value row
    kbig = k.copy()
    kbig[0, :, 7, :] = 0
    qd = np.zeros_like(q); qd[..., 3] = 8.0
    kbig[0, :, :, 3] = 0; kbig[0, :, 7, 3] = 60.0
    cb = O.build_cache(kbig, v, 2, g, nb)
    outb, _ = cb.attn_verify(qd, 1.0)
    assert np.allclose(outb[0, 0, 1], cb.decoded(0, 1, True)[1][7], atol=1e-9)


def test_verify_equals_independent_single_query_calls():
    """Causal mask among the gamma+1 target tokens: query i sees buffer tokens [0, nb-nq+i]."""
    rng = np.random.default_rng(14)
    g = d = 16
    tq, nb, nq = 32, 23, 5
    k, v, c = _rand_cache(rng, 1, 4, 2, d, g, tq, nb)
    q = rng.standard_normal((1, nq, 4, d)).astype(np.float16)
    out, lse = c.attn_verify(q, 0.3)
    for i in range(nq):
        keep = tq + nb - nq + i + 1
        ci = O.build_cache(k[:, :, :keep], v[:, :, :keep], 4, g, keep - tq)
        oi, li = ci.attn_verify(q[:, i:i + 1], 0.3)
        assert np.allclose(out[:, i], oi[:, 0], rtol=1e-12, atol=1e-14)
        assert np.allclose(lse[:, i], li[:, 0], rtol=1e-12)
    # the last query sees everything; the first one does not see the last nq-1 tokens
    vv = v.copy(); vv[:, :, -1] += 1
    c2 = O.build_cache(k, vv, 4, g, nb)
    out2, _ = c2.attn_verify(q, 0.3)
    assert np.array_equal(out2[:, :nq - 1], out[:, :nq - 1]) and not np.allclose(out2[:, nq - 1], out[:, nq - 1])


def test_gqa_equals_mha_with_duplicated_kv_heads():
    rng = np.random.default_rng(15)
    g = d = 16
    k, v, c = _rand_cache(rng, 2, 8, 2, d, g, 32, 17)
    q = rng.standard_normal((2, 3, 8, d)).astype(np.float16)
    cm = O.build_cache(np.repeat(k, 4, axis=1), np.repeat(v, 4, axis=1), 8, g, 17)
    for a, b in ((c.attn_draft, cm.attn_draft), (c.attn_verify, cm.attn_verify)):
        assert np.array_equal(a(q, 0.25)[0], b(q, 0.25)[0])


def test_rows_subset_matches_full():
    rng = np.random.default_rng(16)
    k, v, c = _rand_cache(rng, 2, 4, 2, 16, 16, 32, 17)
    q = rng.standard_normal((2, 2, 4, 16)).astype(np.float16)
    full, _ = c.attn_verify(q, 0.25)
    part, _ = c.attn_verify(q, 0.25, rows=[(1, 2)])
    assert np.array_equal(part[1, :, 2], full[1, :, 2]) and np.isnan(part[0]).all()


def test_flush_is_append_only_and_equals_from_scratch():
    """Decode loop of Algorithm 1 with the buffer policy of Section 4.3.2: after any number of
    appends/flushes the cache equals a from-scratch quantization of the same history, groups that
    were quantized once are never touched again, and G <= n_buf <= 2G holds between steps."""
    rng = np.random.default_rng(17)
    g = d = 8
    hq = hkv = 2
    total = 9 * g + 3
    k = rng.standard_normal((1, hkv, total, d)).astype(np.float16)
    v = rng.standard_normal((1, hkv, total, d)).astype(np.float16)
    start = 2 * g + 5                                   # prefill: quantize all but the last G..2G tokens
    c = O.build_cache(k[:, :, :start], v[:, :, :start], hq, g, start - g)
    assert c.n_quant(0) == g and g <= c.n_buf(0) <= 2 * g
    snap = None
    for t in range(start, total):
        for h in range(hkv):
            c.append(0, h, k[0, h, t], v[0, h, t])
        if c.n_buf(0) == 2 * g:
            snap = [a[0][0].copy() for a in (c.ku, c.kl, c.ks, c.kz, c.vu, c.vl, c.vs, c.vz)]
            c.flush(g)
            for old, new in zip(snap, (c.ku, c.kl, c.ks, c.kz, c.vu, c.vl, c.vs, c.vz)):
                assert np.array_equal(new[0][0][:old.shape[0]], old)
        assert g <= c.n_buf(0) <= 2 * g
    ref = O.build_cache(k, v, hq, g, c.n_buf(0))
    assert c.n_quant(0) == ref.n_quant(0)
    for a, b in ((c.ku, ref.ku), (c.kl, ref.kl), (c.ks, ref.ks), (c.kz, ref.kz),
                 (c.vu, ref.vu), (c.vl, ref.vl), (c.vs, ref.vs), (c.vz, ref.vz), (c.kbuf, ref.kbuf), (c.vbuf, ref.vbuf)):
        for h in range(hkv):
            assert np.array_equal(a[0][h], b[0][h])
    q = rng.standard_normal((1, 2, hq, d)).astype(np.float16)
    assert np.array_equal(c.attn_verify(q, 0.4)[0], ref.attn_verify(q, 0.4)[0])
    # rejected draft tokens only shorten the buffer
    nb = c.n_buf(0)
    c.reject(0, 2)
    assert c.n_buf(0) == nb - 2 and c.n_quant(0) == ref.n_quant(0)


def test_split_merge_identity():
    """Flash-Decoding compatibility (Appendix E): chunk partials (m, l, o) merged with the
    log-sum-exp rule equal the one-pass result; the buffer is just one more chunk."""
    rng = np.random.default_rng(18)
    k, v, c = _rand_cache(rng, 1, 1, 1, 16, 16, 64, 20)
    q = rng.standard_normal((1, 1, 1, 16)).astype(np.float16)
    out, lse = c.attn_draft(q, 0.25)
    kd, vd = c.decoded(0, 0, False)
    chunks = [(kd[:16], vd[:16]), (kd[16:64], vd[16:64]), (c.kbuf[0][0].astype(np.float64), c.vbuf[0][0].astype(np.float64))]
    parts = [O.attend(q[0, :, 0], kk, vv, [kk.shape[0]], 0.25) for kk, vv in chunks]
    lses = np.array([p[1][0] for p in parts])
    w = np.exp(lses - lses.max()); w /= w.sum()
    merged = sum(wi * p[0][0] for wi, p in zip(w, parts))
    assert np.allclose(merged, out[0, 0, 0], rtol=1e-12, atol=1e-14)
    assert abs(lses.max() + math.log(np.exp(lses - lses.max()).sum()) - lse[0, 0, 0]) < 1e-12


def test_planted_attention_mistakes_are_caught():
    """A transposed operand, a dropped softmax scale, or an off-by-one causal mask must not survive
    the library comparison above: show that each changes the library result measurably."""
    rng = np.random.default_rng(19)
    k, v, c = _rand_cache(rng, 1, 2, 2, 16, 16, 16, 9)
    q = rng.standard_normal((1, 3, 2, 16)).astype(np.float16)
    out, _ = c.attn_verify(q, 0.25)
    keys = np.stack([np.concatenate([c.decoded(0, h, True)[0], c.kbuf[0][h].astype(np.float64)]) for h in range(2)])
    vals = np.stack([np.concatenate([c.decoded(0, h, True)[1], c.vbuf[0][h].astype(np.float64)]) for h in range(2)])
    good = [16 + 9 - 3 + i + 1 for i in range(3)]
    assert np.allclose(_sdpa(q[0], keys, vals, good, 0.25, 1), out[0], rtol=1e-12, atol=1e-13)
    assert not np.allclose(_sdpa(q[0], keys, vals, [n - 1 for n in good], 0.25, 1), out[0], rtol=1e-6)
    assert not np.allclose(_sdpa(q[0], keys, vals, good, 1.0, 1), out[0], rtol=1e-6)
    assert not np.allclose(_sdpa(q[0], keys[::-1].copy(), vals, good, 0.25, 1), out[0], rtol=1e-6)
