"""Seeded synthetic inputs shaped like the paper's decode workloads.

This module only draws random tensors.  It holds none of the method's
arithmetic (no quantization, no attention) so that both the CPU oracle's tests
and the HIP path's tests can be fed the very same arrays without sharing any
code of the method itself.

Recipe (stands in for the long-context summarisation / language-modelling
prompts the paper evaluates on, Section 5.1, which are not available here):

* K: fp16, i.i.d. N(0,1); then ``n_outlier`` channels per kv-head (indices drawn
  from the unit's seed) are multiplied by ``outlier_gain``.  This models the
  per-channel outlier structure of key caches that motivates quantizing keys
  along the channel axis (Section 4.3.1, Table 5).
* V, Q: fp16, i.i.d. N(0,1).
* Every (config, layer, sequence, kv-head, tensor) gets its own counter-based
  Philox stream, so any single unit can be regenerated on the host without
  generating the rest of the workload.
"""
from __future__ import annotations

import dataclasses
from concurrent.futures import ThreadPoolExecutor

import numpy as np

T_K, T_V, T_Q, T_OUTLIER = 0, 1, 2, 3


@dataclasses.dataclass(frozen=True)
class Workload:
    """Shape of one decode-attention workload (one transformer layer)."""

    name: str
    config_id: int
    batch: int
    n_q_heads: int
    n_kv_heads: int
    ctx: int                 # total context tokens per sequence
    n_buf: int = 256         # tokens held in the fp16 buffer (R = 2G, Section 5.1)
    head_dim: int = 128
    group: int = 128         # G (Section 5.1)
    nq_verify: int = 5       # gamma + 1 with gamma = 4
    n_layers: int = 1

    @property
    def n_quant(self) -> int:
        return self.ctx - self.n_buf

    @property
    def units(self) -> int:
        return self.batch * self.n_kv_heads


# The five workloads of the build's baseline description.
WORKLOADS = {
    "tiny": Workload("tiny", 0, 1, 32, 8, 2048),
    "mha32k": Workload("mha32k", 1, 1, 32, 32, 32768),
    "mha128k": Workload("mha128k", 2, 1, 32, 32, 131072),
    "gqa128k_b4": Workload("gqa128k_b4", 3, 4, 32, 8, 131072),
    "stack64k_b8": Workload("stack64k_b8", 4, 8, 32, 8, 65536, n_layers=32),
}


def _rng(config_id: int, layer: int, seq: int, head: int, tensor: int) -> np.random.Generator:
    ss = np.random.SeedSequence([0x51535043, config_id, layer, seq, head, tensor])
    return np.random.Generator(np.random.Philox(ss))


def outlier_channels(config_id: int, layer: int, seq: int, kv_head: int,
                     head_dim: int = 128, n_outlier: int = 4) -> np.ndarray:
    g = _rng(config_id, layer, seq, kv_head, T_OUTLIER)
    return np.sort(g.choice(head_dim, size=n_outlier, replace=False))


def gen_unit_kv(config_id: int, layer: int, seq: int, kv_head: int, n_tokens: int,
                head_dim: int = 128, n_outlier: int = 4, outlier_gain: float = 10.0):
    """K and V of one (layer, sequence, kv-head) unit: two fp16 [n_tokens, head_dim] arrays.

    Token order is context order: a caller puts the first ctx - n_buf tokens into
    the quantized region and the remaining ones into the full-precision buffer.
    """
    gk = _rng(config_id, layer, seq, kv_head, T_K)
    gv = _rng(config_id, layer, seq, kv_head, T_V)
    k = gk.standard_normal((n_tokens, head_dim), dtype=np.float32)
    if n_outlier > 0:
        ch = outlier_channels(config_id, layer, seq, kv_head, head_dim, n_outlier)
        k[:, ch] *= np.float32(outlier_gain)
    v = gv.standard_normal((n_tokens, head_dim), dtype=np.float32)
    return k.astype(np.float16), v.astype(np.float16)


def gen_q(config_id: int, layer: int, seq: int, nq: int, n_q_heads: int,
          head_dim: int = 128) -> np.ndarray:
    """Queries of one sequence: fp16 [nq, n_q_heads, head_dim]."""
    g = _rng(config_id, layer, seq, 0, T_Q)
    return g.standard_normal((nq, n_q_heads, head_dim), dtype=np.float32).astype(np.float16)


def gen_layer_kv(w: Workload, layer: int = 0, workers: int = 8, n_tokens: int | None = None):
    """K, V for every unit of one layer: fp16 [batch, n_kv_heads, n_tokens, head_dim] (host)."""
    n = w.ctx if n_tokens is None else n_tokens
    k = np.empty((w.batch, w.n_kv_heads, n, w.head_dim), np.float16)
    v = np.empty_like(k)

    def one(bh):
        b, h = bh
        k[b, h], v[b, h] = gen_unit_kv(w.config_id, layer, b, h, n, w.head_dim)

    jobs = [(b, h) for b in range(w.batch) for h in range(w.n_kv_heads)]
    with ThreadPoolExecutor(max_workers=max(1, workers)) as ex:
        list(ex.map(one, jobs))
    return k, v


def gen_layer_q(w: Workload, nq: int, layer: int = 0) -> np.ndarray:
    """Queries for every sequence: fp16 [batch, nq, n_q_heads, head_dim] (host)."""
    return np.stack([gen_q(w.config_id, layer, b, nq, w.n_q_heads, w.head_dim)
                     for b in range(w.batch)])
