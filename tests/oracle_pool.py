"""Oracle results for whole (layer, sequence, kv-head) units of the baseline workloads, computed in worker
processes.  A worker regenerates its unit from the seeds (nothing large crosses the process boundary),
runs the float64 oracle on it and returns the attention outputs of all query heads of that kv-head plus
digests of the unit's codes and metadata.  This module imports neither torch nor the HIP binding, so the
spawned workers never touch the GPU."""
import hashlib
import os
from concurrent.futures import ProcessPoolExecutor
import multiprocessing as mp

import numpy as np

PLANE_NAMES = ("ku", "kl", "ks", "kz", "vu", "vl", "vs", "vz")


def digest(a: np.ndarray) -> str:
    return hashlib.blake2b(np.ascontiguousarray(a).view(np.uint8).tobytes(), digest_size=16).hexdigest()


def unit_reference(job):
    """job = (workload name, layer, sequence, kv-head, sm_scale) -> dict with
    draft  float64 [1, rep, D], verify float64 [nq, rep, D] (the kv-head's query heads in order) and
    digests {name: hex} of the unit's eight plane / metadata arrays over the whole quantized length."""
    from oracle import quantspec_oracle as O
    from paper_2502_10424_amd import synth
    name, layer, b, kvh, sm = job
    try:      # one thread per worker: the pool already fills the cores
        from threadpoolctl import threadpool_limits
        threadpool_limits(1)
    except ImportError:
        pass
    w = synth.WORKLOADS[name]
    rep = w.n_q_heads // w.n_kv_heads
    k, v = synth.gen_unit_kv(w.config_id, layer, b, kvh, w.ctx, w.head_dim)
    oc = O.build_cache(k[None, None], v[None, None], rep, w.group, w.n_buf)
    heads = slice(kvh * rep, (kvh + 1) * rep)
    qd = synth.gen_q(w.config_id, layer, b, 1, w.n_q_heads, w.head_dim)[None, :, heads]
    qv = synth.gen_q(w.config_id, layer, b, w.nq_verify, w.n_q_heads, w.head_dim)[None, :, heads]
    out_d, _ = oc.attn_draft(qd, sm)
    out_v, _ = oc.attn_verify(qv, sm)
    arrays = dict(ku=oc.ku[0][0], kl=oc.kl[0][0], ks=oc.ks[0][0], kz=oc.kz[0][0],
                  vu=oc.vu[0][0], vl=oc.vl[0][0], vs=oc.vs[0][0][:, 0], vz=oc.vz[0][0][:, 0])
    return dict(job=job, draft=out_d[0], verify=out_v[0], digests={n: digest(a) for n, a in arrays.items()})


def map_units(jobs, workers=None):
    """Yields unit_reference(job) for every job, in completion order of the pool's chunks."""
    workers = workers or min(16, os.cpu_count() or 8, max(1, len(jobs)))
    with ProcessPoolExecutor(max_workers=workers, mp_context=mp.get_context("spawn")) as ex:
        for res in ex.map(unit_reference, jobs):
            yield res
