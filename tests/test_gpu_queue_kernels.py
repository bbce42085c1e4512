"""GPU parity of the attention kernels under other planner settings, above all of the kernels that deal
128-token groups out through a queue shared by the eight waves of a workgroup: the draft call of 2 - 8 query
rows per kv-head, and that of one row over a paged cache.  The planner takes them when a unit has at least
eight groups per workgroup, i.e. at long contexts; here the caches tell the library to plan for a handful of
compute units (qs_cache.compute_units), so that caches of a few thousand tokens run through exactly that code:
with C compute units and U units the planner wants 8*C/U waves per unit, C/U workgroups of eight, and needs
8*C/U groups or more and at most 4*C/U buffer chunks of 64 tokens.  The other calls of the same cases (one
row per kv-head, verify) run the fixed-range kernels with 4*C/U waves per unit."""
import numpy as np
import pytest

from tests.test_gpu_parity import env, _check_attn, _random_case, _run_attn   # noqa: F401  (env is a fixture)

pytestmark = pytest.mark.gpu


@pytest.fixture()
def few_compute_units(env):
    B = env["B"]

    def plan_for(n):
        B.KVCache.default_compute_units = n      # every cache made from here on carries it

    yield plan_for
    B.KVCache.default_compute_units = 0
    B.KVCache.default_flags = 0


@pytest.mark.parametrize("bsz,hkv,rep,nq,cus", [
    (2, 2, 1, 1, 4),    # one row per kv-head: one token per lane in the softmax; one workgroup per unit
    (2, 2, 1, 5, 8),    # verify, 5 rows, two workgroups per unit
    (1, 2, 4, 1, 2),    # grouped queries, 4 rows, draft
    (1, 2, 4, 2, 4),    # 8 rows, verify, two workgroups per unit
    (3, 1, 2, 3, 3),    # ragged batch, 6 rows
    (1, 8, 1, 1, 24),   # three workgroups per unit
])
def test_queue_kernels_match_oracle(env, few_compute_units, bsz, hkv, rep, nq, cus):
    rng = np.random.default_rng(31 * bsz + 7 * hkv + rep + nq)
    few_compute_units(cus)
    wgs = (8 * cus // (bsz * hkv)) // 8
    assert wgs >= 1
    checked = 0
    for attempt in range(16):
        # ragged lengths: some sequences hold far fewer groups than the planner cut the work for (even none)
        cache, oc, q, tag = _random_case(env, rng, bsz, hkv, rep, nq, max_groups=40, max_buf=4 * 64 * wgs)
        if int(cache.n_quant.max()) // 128 < 8 * wgs:
            continue                       # this draw is too short for the queue kernels
        _check_attn(env, cache, oc, q, 0.09, True, tag=f"queue verify {tag}")
        _check_attn(env, cache, oc, q[:, -1:], 0.09, False, tag=f"queue draft {tag}")
        checked += 1
        if checked == 2:
            break
    assert checked == 2


@pytest.mark.parametrize("hq", [4, 2])   # two rows per kv-head in the draft call, or one (queue-dealt only when paged)
def test_queue_kernels_paged_and_flush(env, few_compute_units, hq):
    """Group-table mode under the queue kernels, before and after a flush."""
    torch, O, U, B = env["torch"], env["O"], env["U"], env["B"]
    rng = np.random.default_rng(77)
    few_compute_units(4)
    bsz, hkv, nq = 2, 2, 5
    tq, nb, q_cap = 20 * 128, 128 + nq + 9, 24 * 128
    n_logical = bsz * hkv * (q_cap // 128)
    pool = n_logical + 5
    cache = B.KVCache(bsz, hq, hkv, q_cap, nb + 8, pool_groups=pool)
    table = rng.permutation(pool)[:n_logical].astype(np.int32).reshape(bsz, hkv, q_cap // 128)
    cache.group_table.copy_(torch.from_numpy(table))
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
    _check_attn(env, cache, oc, q, 0.1, True, tag="queue paged verify")
    _check_attn(env, cache, oc, q[:, -1:], 0.1, False, tag="queue paged draft")
    B.qs_quantize_flush(cache, 128)
    cache.n_quant += 128
    cache.n_buf -= 128
    oc.flush(128)
    _check_attn(env, cache, oc, q, 0.1, True, tag="queue paged verify after flush")
    _check_attn(env, cache, oc, q[:, -1:], 0.1, False, tag="queue paged draft after flush")


def test_calls_that_are_bit_reproducible_without_the_flag(env, few_compute_units):
    """One query row per kv-head over a contiguous cache, and every verify call, run on fixed ranges whatever the
    flag says: repeated calls give identical bits, and identical sequences of a batch identical rows."""
    U = env["U"]
    rng = np.random.default_rng(19)
    few_compute_units(16)
    reps = 3
    for hq, hkv, nq, verify in ((2, 2, 1, False), (2, 2, 5, True), (8, 2, 2, True), (8, 2, 5, True)):
        k1 = rng.standard_normal((1, hkv, 128 * 40 + 64, 128)).astype(np.float16)
        v1 = rng.standard_normal(k1.shape).astype(np.float16)
        q1 = rng.standard_normal((1, nq, hq, 128)).astype(np.float16)
        cache = U.make_device_cache(np.repeat(k1, reps, 0), np.repeat(v1, reps, 0), hq, 64)
        qn = np.repeat(q1, reps, 0)
        first, _ = _run_attn(env, cache, qn, 0.09, verify)
        again, _ = _run_attn(env, cache, qn, 0.09, verify)
        assert np.array_equal(first.view(np.uint16), again.view(np.uint16)), (hq, hkv, nq, verify)
        assert np.abs(first.astype(np.float32) - first[:1].astype(np.float32)).max() == 0.0, (hq, hkv, nq, verify)


def test_deterministic_setting_is_bit_reproducible(env, few_compute_units):
    """With QS_FLAG_FIXED_RANGES every wave gets a fixed range of groups: identical sequences of a batch
    give identical bits, and so do repeated calls.  Without it two results agree to a step or two of the fp16 output."""
    U, B = env["U"], env["B"]
    rng = np.random.default_rng(9)
    few_compute_units(16)
    k1 = rng.standard_normal((1, 2, 128 * 40 + 64, 128)).astype(np.float16)
    v1 = rng.standard_normal(k1.shape).astype(np.float16)
    q1 = rng.standard_normal((1, 3, 2, 128)).astype(np.float16)
    reps = 4
    cache = U.make_device_cache(np.repeat(k1, reps, 0), np.repeat(v1, reps, 0), 2, 64)
    qn = np.repeat(q1, reps, 0)
    free, _ = _run_attn(env, cache, qn, 0.09, True)
    assert U.rel_err(free, np.repeat(free[:1], reps, 0).astype(np.float64)) <= 2e-3
    cache.flags = B.QS_FLAG_FIXED_RANGES
    fixed, _ = _run_attn(env, cache, qn, 0.09, True)
    again, _ = _run_attn(env, cache, qn, 0.09, True)
    assert np.array_equal(fixed.view(np.uint16), again.view(np.uint16))
    assert np.abs(fixed.astype(np.float32) - fixed[:1].astype(np.float32)).max() == 0.0
    assert U.rel_err(free, fixed.astype(np.float64)) <= 2e-3


def test_queue_kernels_in_a_hip_graph(env, few_compute_units):
    """The queue lives in LDS and is set up by every launch itself, so a captured draft + verify pair can
    be replayed any number of times: every replay agrees with the eager result to rounding."""
    torch, U, B = env["torch"], env["U"], env["B"]
    rng = np.random.default_rng(123)
    few_compute_units(8)
    bsz, hkv, hq = 2, 2, 4
    t, nb = 24 * 128, 200
    k = rng.standard_normal((bsz, hkv, t + nb, 128)).astype(np.float16)
    v = rng.standard_normal((bsz, hkv, t + nb, 128)).astype(np.float16)
    cache = U.make_device_cache(k, v, hq, nb, q_cap=t, buf_cap=nb + 8)
    qd = torch.from_numpy(rng.standard_normal((bsz, 1, hq, 128)).astype(np.float16)).cuda()
    qv = torch.from_numpy(rng.standard_normal((bsz, 5, hq, 128)).astype(np.float16)).cuda()
    ws = torch.zeros(B.qs_workspace_bytes(cache, 5), dtype=torch.uint8, device="cuda")
    e_d = B.qs_attn_draft(cache, qd, 0.1, workspace=ws).float().cpu().numpy()
    e_v = B.qs_attn_verify(cache, qv, 0.1, workspace=ws).float().cpu().numpy()
    o_d, o_v = torch.empty_like(qd), torch.empty_like(qv)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        B.qs_attn_draft(cache, qd, 0.1, out=o_d, workspace=ws, stream=side)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        cs = torch.cuda.current_stream()
        B.qs_attn_draft(cache, qd, 0.1, out=o_d, workspace=ws, stream=cs)
        B.qs_attn_verify(cache, qv, 0.1, out=o_v, workspace=ws, stream=cs)
    for rep in range(3):
        o_d.zero_(); o_v.zero_(); ws.fill_(0xFF)
        (torch.ones(1000, device="cuda") * rep).sum().item()
        graph.replay()
        torch.cuda.synchronize()
        assert U.rel_err(o_d.float().cpu().numpy(), e_d.astype(np.float64)) <= 2e-3, f"replay {rep}"
        assert U.rel_err(o_v.float().cpu().numpy(), e_v.astype(np.float64)) <= 2e-3, f"replay {rep}"


@pytest.mark.parametrize("cus", [1, 3, 8, 100, 1024])
def test_random_shapes_under_other_planner_settings(env, few_compute_units, cus):
    """The chunk counts, the kernel variant and the workspace layout all follow from the compute-unit count
    the planner works with: seeded random caches under several counts, with queue and with fixed dealing."""
    B = env["B"]
    rng = np.random.default_rng(500 + cus)
    few_compute_units(cus)
    for det in (0, 1):
        B.KVCache.default_flags = B.QS_FLAG_FIXED_RANGES if det else 0
        for case in range(2):
            bsz, hkv = int(rng.integers(1, 4)), int(rng.choice([1, 2, 3, 8]))
            rep, nq = int(rng.choice([1, 2, 4, 8])), int(rng.integers(1, 9))
            cache, oc, q, tag = _random_case(env, rng, bsz, hkv, rep, nq, max_groups=int(rng.choice([3, 12, 40])),
                                             max_buf=int(rng.choice([40, 140, 600])))
            _check_attn(env, cache, oc, q, 0.09, True, tag=f"cus{cus} det{det} verify {tag}")
            _check_attn(env, cache, oc, q[:, -1:], 0.09, False, tag=f"cus{cus} det{det} draft {tag}")


@pytest.mark.parametrize("bsz,hkv,rep,nq,tq,nb,cus", [
    (1, 1, 1, 1, [8 * 128], [1], 1),                                  # one group per wave, one buffer token
    (1, 1, 1, 1, [9 * 128], [256], 1),                                # nine groups for eight waves, four buffer items
    (2, 1, 1, 1, [8 * 128, 0], [1, 5], 2),                            # a sequence without quantized tokens
    (2, 1, 2, 4, [16 * 128, 128], [4, 200], 2),                       # one group against sixteen
    (1, 2, 1, 5, [24 * 128], [5], 6),                                 # three workgroups, the buffer holds just the queries
    (3, 1, 1, 1, [40 * 128, 17 * 128, 3 * 128], [64, 65, 63], 3),     # buffers that end at tile edges
    (1, 1, 8, 1, [8 * 128], [256], 1),                                # eight rows
])
def test_queue_kernels_edge_lengths(env, few_compute_units, bsz, hkv, rep, nq, tq, nb, cus):
    torch, O, U, B = env["torch"], env["O"], env["U"], env["B"]
    rng = np.random.default_rng(7 + sum(tq) // 128 + sum(nb))
    few_compute_units(cus)
    hq = hkv * rep
    cache = B.KVCache(bsz, hq, hkv, max(max(tq), 128), max(nb) + 3)
    oc = O.CacheOracle(bsz, hq, hkv, 128, 128)
    for b in range(bsz):
        n = tq[b] + nb[b]
        k = rng.standard_normal((1, hkv, n, 128)).astype(np.float16)
        v = rng.standard_normal((1, hkv, n, 128)).astype(np.float16)
        kd, vd = torch.from_numpy(k).cuda(), torch.from_numpy(v).cuda()
        if tq[b]:
            B.qs_quantize_prefill(U._seq_view(cache, b), kd, vd, tq[b])
        cache.n_quant[b], cache.n_buf[b] = tq[b], nb[b]
        cache.k_buf[b, :, :nb[b]] = kd[0, :, tq[b]:]
        cache.v_buf[b, :, :nb[b]] = vd[0, :, tq[b]:]
        ob = O.build_cache(k, v, hq, 128, nb[b])
        for name in ("ku", "kl", "ks", "kz", "vu", "vl", "vs", "vz", "kbuf", "vbuf"):
            getattr(oc, name)[b] = getattr(ob, name)[0]
    q = rng.standard_normal((bsz, nq, hq, 128)).astype(np.float16)
    _check_attn(env, cache, oc, q, 0.09, True, tag=f"edge verify tq{tq} nb{nb}")
    _check_attn(env, cache, oc, q[:, -1:], 0.09, False, tag=f"edge draft tq{tq} nb{nb}")
