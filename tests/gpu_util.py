"""Helpers shared by the GPU parity tests: move seeded host tensors into a device cache through the
library's own entry points, and pull results back for comparison with the oracle."""
import numpy as np
import torch

from oracle import quantspec_oracle as O
from paper_2502_10424_amd import binding as B


def make_device_cache(k, v, n_q_heads, n_buf, q_cap=None, buf_cap=None, group=128, pool_groups=None):
    """k, v: host fp16 [B, Hkv, T, D]; the last n_buf[b] tokens go to the buffer, the rest is quantized
    on the device with qs_quantize_prefill.  n_buf: int or per-sequence list (T - n_buf[b] multiple of group)."""
    bsz, hkv, t, d = k.shape
    nb = [n_buf] * bsz if np.isscalar(n_buf) else list(n_buf)
    tq = [t - x for x in nb]
    q_cap = -(-max(tq) // 128) * 128 if q_cap is None else q_cap
    buf_cap = max(max(nb), 1) if buf_cap is None else buf_cap
    cache = B.KVCache(bsz, n_q_heads, hkv, q_cap, buf_cap, head_dim=d, group=group, pool_groups=pool_groups)
    if pool_groups is not None:      # a seeded permutation of the pool: every logical group somewhere else
        perm = np.random.default_rng(pool_groups).permutation(pool_groups)[:cache.group_table.numel()]
        cache.group_table.copy_(torch.from_numpy(perm.astype(np.int32)).view_as(cache.group_table))
    kd = torch.from_numpy(k).cuda()
    vd = torch.from_numpy(v).cuda()
    if len(set(tq)) == 1:
        if tq[0]:
            B.qs_quantize_prefill(cache, kd, vd, tq[0])
        cache.n_quant[:] = tq[0]
    else:  # ragged: quantize sequence by sequence through single-sequence views of the same storage
        for b in range(bsz):
            if tq[b]:
                sub = _seq_view(cache, b)
                B.qs_quantize_prefill(sub, kd[b:b + 1].contiguous(), vd[b:b + 1].contiguous(), tq[b])
            cache.n_quant[b] = tq[b]
    for b in range(bsz):
        if nb[b]:
            cache.k_buf[b, :, :nb[b]] = kd[b, :, tq[b]:]
            cache.v_buf[b, :, :nb[b]] = vd[b, :, tq[b]:]
        cache.n_buf[b] = nb[b]
    torch.cuda.synchronize()
    return cache


def _seq_view(cache, b):
    sub = B.KVCache.__new__(B.KVCache)
    sub.batch, sub.n_q_heads, sub.n_kv_heads = 1, cache.n_q_heads, cache.n_kv_heads
    sub.head_dim, sub.group, sub.q_cap, sub.buf_cap = cache.head_dim, cache.group, cache.q_cap, cache.buf_cap
    for name in B.PLANES + ("k_buf", "v_buf"):
        setattr(sub, name, getattr(cache, name)[b:b + 1])
    sub.pool_groups, sub.group_table = cache.pool_groups, None
    sub.compute_units, sub.flags = cache.compute_units, cache.flags
    if cache.group_table is not None:      # paged: the pools are shared, the view selects the table rows
        sub.upper, sub.lower = cache.upper, cache.lower
        sub.group_table = cache.group_table[b:b + 1]
    sub.n_quant = np.zeros(1, np.int32)
    sub.n_buf = np.zeros(1, np.int32)
    return sub


def export_unit(cache, b, h, n_tokens):
    """Plain-order numpy view of one unit's planes and metadata."""
    e = B.qs_export_codes(cache, b, h, n_tokens)
    torch.cuda.synchronize()
    return {k.replace("_", ""): v.cpu().numpy() for k, v in e.items()}


def assert_unit_equals_oracle(cache, oc: O.CacheOracle, b, h, oracle_head=None):
    """Bit-exact comparison of codes, scales and zeros of one unit, plus the buffer contents.  oracle_head: the
    unit's kv-head in the oracle's cache when that holds only some of the heads (default: h)."""
    oh = h if oracle_head is None else oracle_head
    tq = oc.n_quant(b)
    assert cache.n_quant[b] == tq and cache.n_buf[b] == oc.n_buf(b)
    if tq:
        e = export_unit(cache, b, h, tq)
        for name, ref in (("ku", oc.ku[b][oh]), ("kl", oc.kl[b][oh]), ("vu", oc.vu[b][oh]), ("vl", oc.vl[b][oh])):
            assert np.array_equal(e[name], ref), f"{name} differs for unit ({b},{h})"
        for name, ref in (("ks", oc.ks[b][oh]), ("kz", oc.kz[b][oh]), ("vs", oc.vs[b][oh]), ("vz", oc.vz[b][oh])):
            assert np.array_equal(e[name].view(np.uint16).reshape(ref.shape), ref.view(np.uint16)), f"{name} differs for unit ({b},{h})"
    nb = oc.n_buf(b)
    assert np.array_equal(cache.k_buf[b, h, :nb].cpu().numpy().view(np.uint16), oc.kbuf[b][oh].view(np.uint16))
    assert np.array_equal(cache.v_buf[b, h, :nb].cpu().numpy().view(np.uint16), oc.vbuf[b][oh].view(np.uint16))


def rel_err(out_gpu, out_ref):
    """Per output vector: max_d |gpu - ref| / max_d |ref|; returns the maximum over vectors."""
    g = out_gpu.astype(np.float64)
    num = np.abs(g - out_ref).max(axis=-1)
    den = np.abs(out_ref).max(axis=-1)
    return float((num / den).max())
