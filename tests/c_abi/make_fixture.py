#!/usr/bin/env python3
"""Writes the fixture that tests/c_abi/gpu_run.c checks the library against on a GPU.

Everything expected in the file comes from the CPU oracle (oracle/quantspec_oracle.py); the inputs are
seeded numpy draws.  Nothing here touches the HIP library.  Layout (little endian):
  int32 x 8 : magic 0x51534658, B, Hq, Hkv, Tq, nb, nq, n_flush
  fp16  K, V            [B][Hkv][Tq + nb][128]
  fp16  q_draft         [B][1][Hq][128]
  fp16  q_verify        [B][nq][Hq][128]
  f64   out_draft       [B][1][Hq][128]           oracle, before the flush
  f64   out_verify      [B][nq][Hq][128]
  then for unit (B-1, Hkv-1) after a flush of n_flush tokens, T2 = Tq + n_flush tokens:
  u8 ku [T2][128], i8 kl [T2][128], u8 vu, i8 vl, fp16 ks [T2/128][128], fp16 kz, fp16 vs [T2], fp16 vz [T2]
  f64   out_verify_after [B][nq][Hq][128]         oracle, after the flush
usage: make_fixture.py <output file>"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import quantspec_oracle as O   # noqa: E402


def main(path):
    rng = np.random.default_rng(20250210)
    B, Hq, Hkv, Tq, nb, nq, n_flush = 2, 4, 2, 256, 133, 3, 128
    T = Tq + nb
    k = (rng.standard_normal((B, Hkv, T, 128)) * rng.choice([0.3, 1.0, 8.0], (B, Hkv, 1, 128))).astype(np.float16)
    v = (rng.standard_normal((B, Hkv, T, 128)) + 0.5).astype(np.float16)
    qd = rng.standard_normal((B, 1, Hq, 128)).astype(np.float16)
    qv = rng.standard_normal((B, nq, Hq, 128)).astype(np.float16)
    sm = np.float32(1.0 / np.sqrt(128.0))
    oc = O.build_cache(k, v, Hq, 128, nb)
    out_d, _ = oc.attn_draft(qd, float(sm))
    out_v, _ = oc.attn_verify(qv, float(sm))
    oc.flush(n_flush)
    out_v2, _ = oc.attn_verify(qv, float(sm))
    b, h = B - 1, Hkv - 1
    with open(path, "wb") as f:
        f.write(np.array([0x51534658, B, Hq, Hkv, Tq, nb, nq, n_flush], np.int32).tobytes())
        for a in (k, v, qd, qv, out_d.astype(np.float64), out_v.astype(np.float64),
                  oc.ku[b][h], oc.kl[b][h], oc.vu[b][h], oc.vl[b][h], oc.ks[b][h], oc.kz[b][h],
                  oc.vs[b][h][:, 0], oc.vz[b][h][:, 0], out_v2.astype(np.float64)):
            f.write(np.ascontiguousarray(a).tobytes())


if __name__ == "__main__":
    main(sys.argv[1])
