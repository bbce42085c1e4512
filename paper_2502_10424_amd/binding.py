"""ctypes binding of libquantspec.so: same names as the C ABI, argument marshalling only.

Every step of the hot path runs inside the library's HIP kernels.  PyTorch is used for device
memory and for the current stream handle, nothing else.  There is no fallback: if the shared
library has not been built, loading fails with an error.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libquantspec.so")

QS_MAX_BATCH = 256
QS_MAX_NQ = 16
HEAD_DIM = 128
GROUP = 128
UPPER_BLOCK_BYTES = 4352     # per 32 tokens: key codes, value codes, value S/Z, a quarter of the group's key S/Z
LOWER_BLOCK_BYTES = 4096     # per 32 tokens: key codes, value codes
PLANES = ("upper", "lower")  # the device arrays of the quantized region (C_U and C_L)

QS_OK = 0
QS_ERR_NULL, QS_ERR_SHAPE, QS_ERR_UNSUPPORTED, QS_ERR_ALIGN = -1, -2, -3, -4
QS_ERR_RANGE, QS_ERR_WORKSPACE, QS_ERR_HIP = -5, -6, -7

EXPORTS = ("qs_version", "qs_strerror", "qs_workspace_bytes", "qs_attn_static", "qs_quantize_flush", "qs_quantize_prefill",
           "qs_append", "qs_attn_draft", "qs_attn_verify", "qs_export_codes",
           "qs_w4_bytes", "qs_w4_quantize", "qs_w4_linear", "qs_w4_export")


class qs_cache(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32), ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32), ("group", ctypes.c_int32),
        ("q_cap", ctypes.c_int32), ("buf_cap", ctypes.c_int32),
        ("upper", ctypes.c_void_p), ("lower", ctypes.c_void_p),
        ("k_buf", ctypes.c_void_p), ("v_buf", ctypes.c_void_p),
        ("n_quant", ctypes.POINTER(ctypes.c_int32)), ("n_buf", ctypes.POINTER(ctypes.c_int32)),
        ("group_table", ctypes.c_void_p), ("pool_groups", ctypes.c_int32),
        ("compute_units", ctypes.c_int32), ("flags", ctypes.c_uint32),
    ]


class qs_w4(ctypes.Structure):
    _fields_ = [("n_out", ctypes.c_int32), ("n_in", ctypes.c_int32), ("packed", ctypes.c_void_p)]


class QsError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {qs_strerror(code)} (status {code})")


_lib = None


def lib() -> ctypes.CDLL:
    """Load libquantspec.so (built in-tree by paper_2502_10424_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2502_10424_amd.build` first "
                               "(there is no fallback implementation)")
        l = ctypes.CDLL(LIB_PATH)
        P = ctypes.POINTER(qs_cache)
        vp, i32, i64, f32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float, ctypes.c_size_t
        l.qs_version.restype, l.qs_version.argtypes = ctypes.c_int, []
        l.qs_strerror.restype, l.qs_strerror.argtypes = ctypes.c_char_p, [ctypes.c_int]
        l.qs_workspace_bytes.restype, l.qs_workspace_bytes.argtypes = sz, [P, i32]
        l.qs_quantize_flush.restype, l.qs_quantize_flush.argtypes = ctypes.c_int, [P, i32, vp]
        l.qs_quantize_prefill.restype, l.qs_quantize_prefill.argtypes = ctypes.c_int, [P, vp, vp, i64, i32, vp]
        l.qs_append.restype, l.qs_append.argtypes = ctypes.c_int, [P, vp, vp, i32, vp]
        l.qs_attn_draft.restype = ctypes.c_int
        l.qs_attn_draft.argtypes = [P, vp, vp, f32, vp, sz, vp, vp]
        l.qs_attn_verify.restype = ctypes.c_int
        l.qs_attn_verify.argtypes = [P, vp, i32, vp, f32, vp, sz, vp, vp]
        l.qs_attn_static.restype = ctypes.c_int
        l.qs_attn_static.argtypes = [P, vp, i32, i32, vp, f32, vp, vp]
        l.qs_export_codes.restype = ctypes.c_int
        l.qs_export_codes.argtypes = [P, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp]
        W = ctypes.POINTER(qs_w4)
        l.qs_w4_bytes.restype, l.qs_w4_bytes.argtypes = sz, [i32, i32]
        l.qs_w4_quantize.restype, l.qs_w4_quantize.argtypes = ctypes.c_int, [W, vp, vp]
        l.qs_w4_linear.restype, l.qs_w4_linear.argtypes = ctypes.c_int, [W, vp, i32, vp, vp]
        l.qs_w4_export.restype, l.qs_w4_export.argtypes = ctypes.c_int, [W, vp, vp, vp, vp]
        _lib = l
    return _lib


def qs_version() -> int:
    return lib().qs_version()


def qs_strerror(code: int) -> str:
    return lib().qs_strerror(code).decode()


QS_FLAG_FIXED_RANGES = 1
QS_STATIC_WS_BYTES = 32 << 20


def _ptr(t) -> int | None:
    return None if t is None else t.data_ptr()


def _stream(stream) -> int | None:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream or None
    return getattr(stream, "cuda_stream", stream) or None


def plain_group_bytes(head_dim: int, group: int) -> tuple[int, int]:
    """Bytes of one 128-token group of the upper and of the lower array for shapes other than
    head_dim = group = 128 (the plain layout of include/quantspec.h)."""
    return 128 * head_dim + 1024 * (head_dim // group), 128 * head_dim


class KVCache:
    """Device tensors of one layer's hierarchical cache plus the host-side lengths.

    Pure storage: allocation through torch, layout as documented in include/quantspec.h.
    """

    # what a new cache's planner settings (qs_cache.compute_units, qs_cache.flags) start as
    default_compute_units = 0
    default_flags = 0

    def __init__(self, batch: int, n_q_heads: int, n_kv_heads: int, q_cap: int, buf_cap: int,
                 device="cuda", head_dim: int = HEAD_DIM, group: int = GROUP, pool_groups: int | None = None):
        """pool_groups: None = every unit owns q_cap/128 consecutive groups; a number = paged cache:
        upper / lower are pools of that many 128-token groups and group_table (int32, device,
        [batch][n_kv_heads][q_cap/128], filled by the caller) says where each logical group lives."""
        self.batch, self.n_q_heads, self.n_kv_heads = batch, n_q_heads, n_kv_heads
        self.head_dim, self.group, self.q_cap, self.buf_cap = head_dim, group, q_cap, buf_cap
        u8 = dict(dtype=torch.uint8, device=device)
        f16 = dict(dtype=torch.float16, device=device)
        qc = max(q_cap, 0)
        self.pool_groups, self.group_table = pool_groups, None
        if head_dim == HEAD_DIM and group == GROUP:    # 32-token blocks, four to a 128-token group
            rows, ub, lb = 4, UPPER_BLOCK_BYTES, LOWER_BLOCK_BYTES
        else:                                          # plain layout: one row per 128-token group
            rows, (ub, lb) = 1, plain_group_bytes(head_dim, group)
        if pool_groups is None:
            self.upper = torch.zeros((batch, n_kv_heads, qc // 128 * rows, ub), **u8)
            self.lower = torch.zeros((batch, n_kv_heads, qc // 128 * rows, lb), **u8)
        else:
            self.upper = torch.zeros((pool_groups * rows, ub), **u8)
            self.lower = torch.zeros((pool_groups * rows, lb), **u8)
            self.group_table = torch.zeros((batch, n_kv_heads, qc // 128), dtype=torch.int32, device=device)
        self.k_buf = torch.zeros((batch, n_kv_heads, buf_cap, head_dim), **f16)
        self.v_buf = torch.zeros((batch, n_kv_heads, buf_cap, head_dim), **f16)
        self.n_quant = np.zeros(batch, np.int32)
        self.n_buf = np.zeros(batch, np.int32)
        self.compute_units, self.flags = KVCache.default_compute_units, KVCache.default_flags

    def struct(self) -> qs_cache:
        c = qs_cache()
        c.batch, c.n_q_heads, c.n_kv_heads = self.batch, self.n_q_heads, self.n_kv_heads
        c.head_dim, c.group, c.q_cap, c.buf_cap = self.head_dim, self.group, self.q_cap, self.buf_cap
        for name in ("upper", "lower",
                     "k_buf", "v_buf"):
            setattr(c, name, getattr(self, name).data_ptr())
        c.n_quant = self.n_quant.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))
        c.n_buf = self.n_buf.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))
        if self.group_table is not None:
            c.group_table, c.pool_groups = self.group_table.data_ptr(), self.pool_groups
        c.compute_units, c.flags = self.compute_units, self.flags
        return c

    def plane_bytes(self) -> int:
        return sum(getattr(self, n).numel() * getattr(self, n).element_size()
                   for n in PLANES)


def _as_struct(cache) -> qs_cache:
    return cache.struct() if isinstance(cache, KVCache) else cache


def _check(rc: int, where: str):
    if rc != QS_OK:
        raise QsError(rc, where)


def qs_workspace_bytes(cache, nq: int) -> int:
    c = _as_struct(cache)
    return int(lib().qs_workspace_bytes(ctypes.byref(c), nq))


def qs_quantize_flush(cache, n_tokens: int, stream=None) -> None:
    """Quantize buffer tokens [0, n_tokens) into the planes and move the rest of the buffer to the
    front.  Like the C call it leaves the host lengths alone: the caller updates n_quant / n_buf."""
    c = _as_struct(cache)
    _check(lib().qs_quantize_flush(ctypes.byref(c), n_tokens, _stream(stream)), "qs_quantize_flush")


def qs_quantize_prefill(cache, k_src, v_src, n_tokens: int, stream=None) -> None:
    """k_src, v_src: fp16 device tensors [B, Hkv, T_src, head_dim] (contiguous); quantizes their first n_tokens."""
    c = _as_struct(cache)
    assert k_src.is_contiguous() and v_src.is_contiguous() and k_src.dtype == torch.float16
    _check(lib().qs_quantize_prefill(ctypes.byref(c), k_src.data_ptr(), v_src.data_ptr(), k_src.shape[2],
                                     n_tokens, _stream(stream)), "qs_quantize_prefill")


def qs_append(cache, k_new, v_new, stream=None) -> None:
    """k_new, v_new: fp16 device tensors [B, n_new, Hkv, head_dim] written to buffer rows n_buf[b].. of every
    sequence.  Like the C call it leaves the host lengths alone: the caller adds n_new to n_buf."""
    c = _as_struct(cache)
    assert k_new.dtype == torch.float16 and k_new.is_contiguous() and v_new.is_contiguous()
    _check(lib().qs_append(ctypes.byref(c), k_new.data_ptr(), v_new.data_ptr(), k_new.shape[1], _stream(stream)),
           "qs_append")


def _attn(fn_name, cache, q, nq, out, sm_scale, workspace, lse, stream):
    c = _as_struct(cache)
    assert q.dtype == torch.float16 and q.is_contiguous()
    if out is None:
        out = torch.empty_like(q)
    if workspace is None:
        workspace = torch.empty(qs_workspace_bytes(c, q.shape[1]), dtype=torch.uint8, device=q.device)
    ws_bytes = workspace.numel() * workspace.element_size()
    l = lib()
    if fn_name == "qs_attn_draft":
        rc = l.qs_attn_draft(ctypes.byref(c), q.data_ptr(), out.data_ptr(), sm_scale, workspace.data_ptr(),
                             ws_bytes, _ptr(lse), _stream(stream))
    else:
        rc = l.qs_attn_verify(ctypes.byref(c), q.data_ptr(), nq, out.data_ptr(), sm_scale, workspace.data_ptr(),
                              ws_bytes, _ptr(lse), _stream(stream))
    _check(rc, fn_name)
    return out


def qs_attn_draft(cache, q, sm_scale: float, out=None, workspace=None, lse=None, stream=None):
    """q: fp16 device tensor [B, 1, Hq, head_dim].  Returns out (same shape)."""
    assert q.shape[1] == 1
    return _attn("qs_attn_draft", cache, q, 1, out, sm_scale, workspace, lse, stream)


def qs_attn_verify(cache, q, sm_scale: float, out=None, workspace=None, lse=None, stream=None):
    """q: fp16 device tensor [B, nq, Hq, head_dim], nq = gamma + 1.  Returns out (same shape)."""
    return _attn("qs_attn_verify", cache, q, q.shape[1], out, sm_scale, workspace, lse, stream)


def qs_attn_static(cache, q, sm_scale: float, verify: bool, out=None, lse=None, stream=None):
    """qs_attn_draft (verify=False, one query) or qs_attn_verify (verify=True) with the split-K partials in
    the library's built-in scratch array: no workspace argument, nothing allocated by the call itself
    (pass `out`; without it the binding allocates the result tensor, the library does not)."""
    c = _as_struct(cache)
    assert q.dtype == torch.float16 and q.is_contiguous()
    if out is None:
        out = torch.empty_like(q)
    _check(lib().qs_attn_static(ctypes.byref(c), q.data_ptr(), q.shape[1], int(bool(verify)), out.data_ptr(), sm_scale,
                                _ptr(lse), _stream(stream)), "qs_attn_static")
    return out


def qs_export_codes(cache: KVCache, b: int, kv_head: int, n_tokens: int, stream=None):
    """Plain-order codes and metadata of one unit, as a dict of device tensors (D = head_dim, G = group):
    k_u, v_u uint8 [T,D]; k_l, v_l int8 [T,D]; k_s, k_z fp16 [T/G,D]; v_s, v_z fp16 [T,D/G] ([T] when G = D)."""
    c = cache.struct()
    dev = cache.k_buf.device
    d, g = cache.head_dim, cache.group
    k_u = torch.empty((n_tokens, d), dtype=torch.uint8, device=dev)
    v_u = torch.empty_like(k_u)
    k_l = torch.empty((n_tokens, d), dtype=torch.int8, device=dev)
    v_l = torch.empty_like(k_l)
    v_s = torch.empty(n_tokens if g == d else (n_tokens, d // g), dtype=torch.float16, device=dev)
    v_z = torch.empty_like(v_s)
    k_s = torch.empty((n_tokens // g, d), dtype=torch.float16, device=dev)
    k_z = torch.empty_like(k_s)
    _check(lib().qs_export_codes(ctypes.byref(c), b, kv_head, n_tokens, k_u.data_ptr(), k_l.data_ptr(),
                                 k_s.data_ptr(), k_z.data_ptr(), v_u.data_ptr(), v_l.data_ptr(),
                                 v_s.data_ptr(), v_z.data_ptr(), _stream(stream)),
           "qs_export_codes")
    return dict(k_u=k_u, k_l=k_l, k_s=k_s, k_z=k_z, v_u=v_u, v_l=v_l, v_s=v_s, v_z=v_z)


QS_W4_GROUP = 128
QS_W4_MAX_ROWS = 16


def qs_w4_bytes(n_out: int, n_in: int) -> int:
    return int(lib().qs_w4_bytes(n_out, n_in))


class W4Linear:
    """Device storage of one 4-bit weight matrix W [n_out, n_in] (y = x W^T); memory only, the library fills it."""

    def __init__(self, n_out: int, n_in: int, device="cuda"):
        nbytes = qs_w4_bytes(n_out, n_in)
        if nbytes == 0:
            raise QsError(QS_ERR_SHAPE, "qs_w4_bytes")
        self.n_out, self.n_in = n_out, n_in
        self.packed = torch.zeros(nbytes, dtype=torch.uint8, device=device)

    def struct(self) -> qs_w4:
        return qs_w4(self.n_out, self.n_in, self.packed.data_ptr())


def qs_w4_quantize(layer: W4Linear, w, stream=None) -> None:
    """w: device fp16 [n_out, n_in], contiguous."""
    assert w.dtype == torch.float16 and w.is_contiguous() and tuple(w.shape) == (layer.n_out, layer.n_in)
    c = layer.struct()
    _check(lib().qs_w4_quantize(ctypes.byref(c), w.data_ptr(), _stream(stream)), "qs_w4_quantize")


def qs_w4_linear(layer: W4Linear, x, out=None, stream=None):
    """x: device fp16 [m, n_in], contiguous, m <= QS_W4_MAX_ROWS; returns fp16 [m, n_out]."""
    assert x.dtype == torch.float16 and x.is_contiguous() and x.dim() == 2 and x.shape[1] == layer.n_in
    m = x.shape[0]
    if out is None:
        out = torch.empty((m, layer.n_out), dtype=torch.float16, device=x.device)
    c = layer.struct()
    _check(lib().qs_w4_linear(ctypes.byref(c), x.data_ptr(), m, out.data_ptr(), _stream(stream)), "qs_w4_linear")
    return out


def qs_w4_export(layer: W4Linear, stream=None):
    """Codes uint8 [n_out, n_in], scale and zero fp16 [n_out, n_in / 128] as device tensors."""
    dev = layer.packed.device
    codes = torch.empty((layer.n_out, layer.n_in), dtype=torch.uint8, device=dev)
    scale = torch.empty((layer.n_out, layer.n_in // QS_W4_GROUP), dtype=torch.float16, device=dev)
    zero = torch.empty_like(scale)
    c = layer.struct()
    _check(lib().qs_w4_export(ctypes.byref(c), codes.data_ptr(), scale.data_ptr(), zero.data_ptr(), _stream(stream)),
           "qs_w4_export")
    return codes, scale, zero
