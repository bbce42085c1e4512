"""CPU oracle for QuantSpec's hierarchical 4-bit KV cache and its decode attention.

THIS IS TEST INFRASTRUCTURE, NOT A PRODUCT PATH.  It is a plain, slow,
float64 numpy implementation of what the HIP library computes, written from the
paper alone.  It shares no code with the HIP path and must never be imported by
it; only the tests, the smoke check and the benchmark's CPU-baseline leg may
call it.

What it follows
---------------
* Section 4.2 (the hierarchical cache): an asymmetric round-to-nearest 4-bit
  code C_U in [0, 15] is computed first, then the quantization error E_U of that
  code is quantized with symmetric round-to-nearest into C_L in [-8, 7]; the
  lower plane has no metadata of its own, its scale is S_INT4 / 2^4, and
  C_INT8 = 2^4 C_U + C_L,  x_hat = C_U S + C_L S / 2^4 + Z.
* Section 4.3.1 and Appendix D (Table 5): keys are grouped per channel over G
  consecutive tokens, values per token over the G = head_dim channels.
* Section 4.3.2: a full-precision buffer holds the most recent tokens; every G
  tokens its oldest G tokens are quantized, appended to the planes, and the rest
  moves to the front.
* Appendix A: decode attention is plain multi-head attention of the query over
  the concatenated cache (here: decoded quantized tokens, then buffer tokens).
* Algorithm 1: the draft pass reads C_U and the buffer; the target pass reads
  C_U, C_L and the buffer, for gamma + 1 query tokens at once.
* Abstract and Section 4 (first paragraph): the draft model's weights are INT4.  quantize_w /
  linear_w4 at the end of this file: the same quantizer, one (S, Z) per output row and G input
  channels, and the layer y = x W_hat^T in float64 (pins: tests/test_oracle_w4.py).

Readings where the paper is silent (each is also listed in the design notes):
* scale/zero: Z = min, S = (max - min) / 15, stored as fp16; S == 0 -> S := 1.
* the code decisions are taken in IEEE binary32 with the *stored* fp16 S and Z,
  one operation at a time (no fused multiply-add), ties to even.  Decode and
  attention are float64.
* E_U / (S/16) can reach +8, which [-8, 7] cannot hold: it is clamped to 7.
* verify query i (0-based, nq queries) sees every quantized token and buffer
  tokens [0, n_buf - nq + i]: the caller has written the nq speculated tokens as
  the last nq buffer tokens.  A draft query is the nq = 1 case over C_U only.
* grouped-query attention: q-head h reads kv-head h // (Hq // Hkv).

Parity pins: see tests/test_oracle_*.py.  End-to-end numeric values are
*parity unpinned against the paper* (it prints no worked example of this path);
every function below is pinned by hand-derived fixtures, brute force, closed
forms, invariants and library routines instead.
"""
from __future__ import annotations

import numpy as np

F16, F32, F64 = np.float16, np.float32, np.float64


# --------------------------------------------------------------------------
# Section 4.2: group statistics, scale / zero, the two code planes
# --------------------------------------------------------------------------
def scale_zero(mn: np.ndarray, mx: np.ndarray):
    """Asymmetric 4-bit scale and zero-point of a group from its min and max (fp16 in, fp16 out).

    Section 4.2 writes dequantization as C * S + Z with C_U in [0, 15]; the
    range [min, max] is therefore mapped onto the 15 steps between code 0 and 15.
    """
    mn = np.asarray(mn, F16)
    mx = np.asarray(mx, F16)
    s = ((mx.astype(F32) - mn.astype(F32)) / F32(15.0)).astype(F16)   # binary32 ops, RNE to fp16
    s = np.where(s == F16(0), F16(1.0), s).astype(F16)
    return s, mn.copy()


def encode(x: np.ndarray, s: np.ndarray, z: np.ndarray):
    """Upper and lower 4-bit codes of fp16 values x for (broadcastable) fp16 scale s and zero z.

    Section 4.2, in its order: C_U first (asymmetric RTN into [0, 15]); then the
    error E_U = x - (C_U S + Z) of that code; then C_L = RTN(E_U / (S / 2^4)) into
    [-8, 7].  All in binary32, one rounding per operation, ties to even.
    """
    x = np.asarray(x, F16).astype(F32)
    s = np.asarray(s, F16).astype(F32)
    z = np.asarray(z, F16).astype(F32)
    t = (x - z) / s
    u = np.clip(np.rint(t), F32(0), F32(15))
    deq_u = u * s + z                     # separate multiply and add (numpy never fuses)
    e_u = x - deq_u
    s_l = s / F32(16.0)
    l = np.clip(np.rint(e_u / s_l), F32(-8), F32(7))
    return u.astype(np.uint8), l.astype(np.int8)


def quantize_k(k: np.ndarray, group: int):
    """Keys [T, D] fp16 -> (U uint8 [T, D], L int8 [T, D], S fp16 [T/G, D], Z fp16 [T/G, D]).

    Per-channel grouping (Section 4.3.1): one (S, Z) per channel per G consecutive tokens.
    """
    k = np.asarray(k, F16)
    t, d = k.shape
    assert t % group == 0
    kg = k.reshape(t // group, group, d)
    s, z = scale_zero(kg.min(axis=1), kg.max(axis=1))           # [T/G, D]
    u, l = encode(kg, s[:, None, :], z[:, None, :])
    return u.reshape(t, d), l.reshape(t, d), s, z


def quantize_v(v: np.ndarray, group: int):
    """Values [T, D] fp16 -> (U [T, D], L [T, D], S fp16 [T, D/G], Z fp16 [T, D/G]).

    Per-token grouping (Section 4.3.1): one (S, Z) per token per G consecutive
    channels; with G = head_dim that is one pair per token.
    """
    v = np.asarray(v, F16)
    t, d = v.shape
    assert d % group == 0
    vg = v.reshape(t, d // group, group)
    s, z = scale_zero(vg.min(axis=2), vg.max(axis=2))           # [T, D/G]
    u, l = encode(vg, s[:, :, None], z[:, :, None])
    return u.reshape(t, d), l.reshape(t, d), s, z


def int8_code(u: np.ndarray, l: np.ndarray) -> np.ndarray:
    """C_INT8 = 2^4 C_U + C_L (Section 4.2); with C_L in [-8, 7] it spans [-8, 247]."""
    return 16 * u.astype(np.int32) + l.astype(np.int32)


def split_int8(c8: np.ndarray):
    """Inverse of int8_code: the unique (C_U, C_L) with C_U in [0,15], C_L in [-8,7]."""
    c8 = np.asarray(c8, np.int32)
    u = (c8 + 8) >> 4
    return u.astype(np.uint8), (c8 - 16 * u).astype(np.int8)


def _expand_k_meta(m: np.ndarray, group: int) -> np.ndarray:
    return np.repeat(m.astype(F64), group, axis=0)              # [T/G, D] -> [T, D]


def _expand_v_meta(m: np.ndarray, group: int) -> np.ndarray:
    return np.repeat(m.astype(F64), group, axis=1)              # [T, D/G] -> [T, D]


def decode_k(u, l, s, z, group: int, use_lower: bool) -> np.ndarray:
    """x_hat = C_U S + [C_L S / 2^4] + Z for keys, float64 (Section 4.2)."""
    se, ze = _expand_k_meta(s, group), _expand_k_meta(z, group)
    x = u.astype(F64) * se + ze
    if use_lower:
        x = x + l.astype(F64) * (se / 16.0)
    return x


def decode_v(u, l, s, z, group: int, use_lower: bool) -> np.ndarray:
    """x_hat = C_U S + [C_L S / 2^4] + Z for values, float64 (Section 4.2)."""
    se, ze = _expand_v_meta(s, group), _expand_v_meta(z, group)
    x = u.astype(F64) * se + ze
    if use_lower:
        x = x + l.astype(F64) * (se / 16.0)
    return x


# --------------------------------------------------------------------------
# Appendix A: attention of one kv-head's queries over quantized ++ buffer tokens
# --------------------------------------------------------------------------
def attend(q: np.ndarray, keys: np.ndarray, values: np.ndarray, n_visible, sm_scale: float):
    """Plain softmax attention, float64, one pass, no splitting.

    q [R, D]; keys, values [T, D]; n_visible[r] = number of leading tokens row r may see.
    Returns (out [R, D], lse [R]) with lse the natural-log normaliser.
    """
    q = np.asarray(q).astype(F64)
    keys = np.asarray(keys).astype(F64)
    values = np.asarray(values).astype(F64)
    out = np.empty((q.shape[0], values.shape[1]), F64)
    lse = np.empty(q.shape[0], F64)
    for r in range(q.shape[0]):
        n = int(n_visible[r])
        s = (keys[:n] @ q[r]) * sm_scale
        m = s.max()
        p = np.exp(s - m)
        den = p.sum()
        out[r] = (p / den) @ values[:n]
        lse[r] = m + np.log(den)
    return out, lse


class CacheOracle:
    """Hierarchical cache of one layer: planes + metadata + fp16 buffer, per (sequence, kv-head).

    Codes are kept unpacked (one uint8 / int8 per element).  Lengths may differ per sequence.
    """

    def __init__(self, batch: int, n_q_heads: int, n_kv_heads: int, head_dim: int, group: int):
        assert n_q_heads % n_kv_heads == 0
        self.batch, self.hq, self.hkv, self.d, self.g = batch, n_q_heads, n_kv_heads, head_dim, group
        e = lambda dt, *shape: np.empty(shape, dt)
        mk = lambda f: [[f() for _ in range(n_kv_heads)] for _ in range(batch)]
        self.ku = mk(lambda: e(np.uint8, 0, head_dim))
        self.kl = mk(lambda: e(np.int8, 0, head_dim))
        self.ks = mk(lambda: e(F16, 0, head_dim))
        self.kz = mk(lambda: e(F16, 0, head_dim))
        self.vu = mk(lambda: e(np.uint8, 0, head_dim))
        self.vl = mk(lambda: e(np.int8, 0, head_dim))
        self.vs = mk(lambda: e(F16, 0, head_dim // group))
        self.vz = mk(lambda: e(F16, 0, head_dim // group))
        self.kbuf = mk(lambda: e(F16, 0, head_dim))
        self.vbuf = mk(lambda: e(F16, 0, head_dim))

    # -- Section 4.3.2 / Algorithm 1: buffer handling ---------------------------------
    def append(self, b: int, h: int, k_new: np.ndarray, v_new: np.ndarray):
        """New tokens' K/V go to the end of the full-precision buffer (Appendix A concat)."""
        self.kbuf[b][h] = np.concatenate([self.kbuf[b][h], np.asarray(k_new, F16).reshape(-1, self.d)])
        self.vbuf[b][h] = np.concatenate([self.vbuf[b][h], np.asarray(v_new, F16).reshape(-1, self.d)])

    def reject(self, b: int, n_drop: int):
        """Drop the last n_drop buffer tokens of sequence b (rejected draft tokens)."""
        if n_drop:
            for h in range(self.hkv):
                self.kbuf[b][h] = self.kbuf[b][h][:-n_drop]
                self.vbuf[b][h] = self.vbuf[b][h][:-n_drop]

    def n_buf(self, b: int) -> int:
        return self.kbuf[b][0].shape[0]

    def n_quant(self, b: int) -> int:
        return self.ku[b][0].shape[0]

    def flush(self, n_tokens: int):
        """Quantize the oldest n_tokens buffer tokens of every unit, append them to the planes,
        and make the remaining buffer tokens the front of the buffer."""
        assert n_tokens % self.g == 0
        for b in range(self.batch):
            for h in range(self.hkv):
                assert self.kbuf[b][h].shape[0] >= n_tokens
                ku, kl, ks, kz = quantize_k(self.kbuf[b][h][:n_tokens], self.g)
                vu, vl, vs, vz = quantize_v(self.vbuf[b][h][:n_tokens], self.g)
                cat = np.concatenate
                self.ku[b][h] = cat([self.ku[b][h], ku]); self.kl[b][h] = cat([self.kl[b][h], kl])
                self.ks[b][h] = cat([self.ks[b][h], ks]); self.kz[b][h] = cat([self.kz[b][h], kz])
                self.vu[b][h] = cat([self.vu[b][h], vu]); self.vl[b][h] = cat([self.vl[b][h], vl])
                self.vs[b][h] = cat([self.vs[b][h], vs]); self.vz[b][h] = cat([self.vz[b][h], vz])
                self.kbuf[b][h] = self.kbuf[b][h][n_tokens:].copy()
                self.vbuf[b][h] = self.vbuf[b][h][n_tokens:].copy()

    # -- Algorithm 1: DRAFT (upper plane) and TARGET (both planes) attention ----------------
    def decoded(self, b: int, h: int, use_lower: bool):
        k = decode_k(self.ku[b][h], self.kl[b][h], self.ks[b][h], self.kz[b][h], self.g, use_lower)
        v = decode_v(self.vu[b][h], self.vl[b][h], self.vs[b][h], self.vz[b][h], self.g, use_lower)
        return k, v

    def attention(self, q: np.ndarray, sm_scale: float, use_lower: bool, rows=None):
        """q fp16 [batch, nq, Hq, D] -> (out float64 [batch, nq, Hq, D], lse float64 [batch, nq, Hq]).

        rows: optional iterable of (b, q-head) pairs to compute (others are left NaN); used to
        sample outputs of workloads too large to evaluate whole.
        """
        q = np.asarray(q)
        bsz, nq, hq, d = q.shape
        assert (bsz, hq, d) == (self.batch, self.hq, self.d)
        rep = self.hq // self.hkv
        out = np.full((bsz, nq, hq, d), np.nan, F64)
        lse = np.full((bsz, nq, hq), np.nan, F64)
        want = None if rows is None else set(rows)
        for b in range(bsz):
            for kvh in range(self.hkv):
                heads = [h for h in range(kvh * rep, (kvh + 1) * rep) if want is None or (b, h) in want]
                if not heads:
                    continue
                kq, vq = self.decoded(b, kvh, use_lower)
                keys = np.concatenate([kq, self.kbuf[b][kvh].astype(F64)])
                vals = np.concatenate([vq, self.vbuf[b][kvh].astype(F64)])
                tq, nb = kq.shape[0], self.kbuf[b][kvh].shape[0]
                assert nb >= nq
                vis = [tq + nb - nq + i + 1 for i in range(nq)]
                for h in heads:
                    o, l = attend(q[b, :, h, :], keys, vals, vis, sm_scale)
                    out[b, :, h, :] = o
                    lse[b, :, h] = l
        return out, lse

    def attn_draft(self, q, sm_scale, rows=None):
        """DRAFT of Algorithm 1: upper 4-bit plane + buffer."""
        return self.attention(q, sm_scale, use_lower=False, rows=rows)

    def attn_verify(self, q, sm_scale, rows=None):
        """TARGET of Algorithm 1: upper and lower planes (INT8) + buffer, nq = gamma + 1 causal queries."""
        return self.attention(q, sm_scale, use_lower=True, rows=rows)


def build_cache(k: np.ndarray, v: np.ndarray, n_q_heads: int, group: int, n_buf) -> CacheOracle:
    """Prefill of Algorithm 1: from fp16 K, V [batch, Hkv, T, D] quantize all but the last
    n_buf[b] tokens (in batches of G) and keep those in the buffer.  n_buf: int or per-sequence list."""
    bsz, hkv, t, d = k.shape
    nb = [n_buf] * bsz if np.isscalar(n_buf) else list(n_buf)
    c = CacheOracle(bsz, n_q_heads, hkv, d, group)
    for b in range(bsz):
        assert (t - nb[b]) % group == 0
        for h in range(hkv):
            c.append(b, h, k[b, h], v[b, h])
    # flush sequence by sequence (lengths may differ)
    for b in range(bsz):
        tq = t - nb[b]
        for h in range(hkv):
            if tq:
                ku, kl, ks, kz = quantize_k(c.kbuf[b][h][:tq], group)
                vu, vl, vs, vz = quantize_v(c.vbuf[b][h][:tq], group)
                c.ku[b][h], c.kl[b][h], c.ks[b][h], c.kz[b][h] = ku, kl, ks, kz
                c.vu[b][h], c.vl[b][h], c.vs[b][h], c.vz[b][h] = vu, vl, vs, vz
                c.kbuf[b][h] = c.kbuf[b][h][tq:].copy()
                c.vbuf[b][h] = c.vbuf[b][h][tq:].copy()
    return c


# --------------------------------------------------------------------------
# The draft model's linear layers: 4-bit weights (abstract; Section 4, first paragraph; Section 5.3's ablation)
# --------------------------------------------------------------------------
# The paper quantizes the draft's weights into INT4 and names no quantizer for them (it cites weight-only
# methods in its related work).  Reading: the quantizer of Section 4.2 itself, upper plane only - asymmetric
# round-to-nearest, C in [0, 15], w_hat = C S + Z - with one (S, Z) per output row and per G consecutive
# input channels (the group size of Section 5.1, 128), S and Z stored in fp16.  That is what quantize_v
# computes for a [rows, channels] matrix, so the pinned functions above serve here unchanged.
def quantize_w(w: np.ndarray, group: int):
    """Weights [N, K] fp16 (y = x W^T) -> (C uint8 [N, K], S fp16 [N, K/G], Z fp16 [N, K/G])."""
    c, _, s, z = quantize_v(w, group)
    return c, s, z


def decode_w(c: np.ndarray, s: np.ndarray, z: np.ndarray, group: int) -> np.ndarray:
    """w_hat = C S + Z in float64, [N, K]."""
    se = np.repeat(np.asarray(s, F16).astype(F64), group, axis=1)
    ze = np.repeat(np.asarray(z, F16).astype(F64), group, axis=1)
    return c.astype(F64) * se + ze


def linear_w4(x: np.ndarray, c: np.ndarray, s: np.ndarray, z: np.ndarray, group: int) -> np.ndarray:
    """y[m, n] = sum_k x[m, k] w_hat[n, k] in float64; x fp16 [M, K]."""
    return np.asarray(x, F16).astype(F64) @ decode_w(c, s, z, group).T
