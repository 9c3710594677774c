"""GPU-segment priority assignment (Sec. 4.3 / 5.4) on the GPU against the CPU oracle, bit for
bit: every assigned level (int32), every response time (int64, sentinels included), every
verdict, through the C ABI."""
import numpy as np
import pytest

from test_gpu_parity import few_gpu_tasks_workload, gpu, relaxed_workload  # noqa: F401 (fixture)

pytestmark = pytest.mark.gpu

GCAPS, BUSY, SUSPEND = 1, 0, 1


def compare(oracle, B, ctx, batch, skip=None, waits=(BUSY, SUSPEND)):
    found = 0
    for wait in waits:
        want_g, want_r, want_s, _ = oracle.gprio_assign_batch(batch, wait, skip=skip, threads=16)
        got_g, got_r, got_s = B.gcaps_gprio_assign_batch(ctx, batch, wait, skip)
        bad = np.argwhere(got_g != want_g)
        assert bad.size == 0, (wait, bad[:5], got_g[bad[0][0]], want_g[bad[0][0]])
        bad = np.argwhere(got_r != want_r)
        assert bad.size == 0, (wait, bad[:5], got_r[bad[0][0]], want_r[bad[0][0]])
        assert (got_s == want_s).all()
        found += int(want_s.sum())
    return found


@pytest.mark.parametrize("k,N", [(1, None), (2, None), (3, 20_000), (4, 2_000), (5, 21_600)])
def test_named_workloads(oracle, gpu, k, N):
    from paper_2406_05221_amd import taskgen
    B, ctx, _ = gpu
    print(f"workload {k} N={N}", flush=True)
    compare(oracle, B, ctx, taskgen.config(k, N))
    # shapes up to 32 tasks with these magnitudes stay in the quad-lane kernel; workload 4 (80 tasks) does not
    wide = B.gcaps_last_wide_count(ctx)
    assert wide == (0 if k != 4 else 2_000)


def test_only_the_tasksets_that_fail_with_equal_priorities(oracle, gpu):
    """The procedure of Sec. 6.1: separate priorities are searched for the tasksets that fail the
    test with GPU priority = CPU priority; some of them are rescued."""
    B, ctx, _ = gpu
    batch = relaxed_workload(6_001, seed=4)
    for wait in (BUSY, SUSPEND):
        _, sched = B.gcaps_rta_batch(ctx, batch, GCAPS, wait)
        skip = sched[0]
        assert 0.05 < skip.mean() < 0.95
        want_g, want_r, want_s, _ = oracle.gprio_assign_batch(batch, wait, skip=skip, threads=16)
        got_g, got_r, got_s = B.gcaps_gprio_assign_batch(ctx, batch, wait, skip)
        assert (got_g == want_g).all() and (got_r == want_r).all() and (got_s == want_s).all()
        rescued = int((got_s.astype(bool) & ~skip.astype(bool)).sum())
        assert rescued > 0
        # an assignment that was found passes the analysis for given priorities, with the same bounds
        for s in np.flatnonzero(got_s.astype(bool) & ~skip.astype(bool))[:40]:
            r, ok, _ = oracle.gprio_rta_taskset(batch["cpu_us"][s], batch["period_us"][s], batch["deadline_us"][s],
                                                batch["prio"][s], batch["core"][s], batch["n_gseg"][s],
                                                batch["gm_us"][s], batch["ge_us"][s], got_g[s],
                                                eps_us=batch["eps_us"][s], wait_mode=wait)
            assert ok == 1 and (r == got_r[s]).all()


def test_mostly_schedulable_tasksets(oracle, gpu):
    B, ctx, _ = gpu
    for batch in (relaxed_workload(5_003, seed=2), few_gpu_tasks_workload(5_003, seed=2)):
        found = compare(oracle, B, ctx, batch)
        assert 0.1 * 2 * 5_003 < found < 0.99 * 2 * 5_003


def test_two_launch_route_of_the_search(oracle, monkeypatch):
    """GCAPS_GPRIO_KERNEL=list: the first launch only settles and lists, the second searches sixteen listed
    tasksets per wavefront (the faster route when most tasksets are searched deeply); same results."""
    import torch
    from paper_2406_05221_amd import binding as B, taskgen
    monkeypatch.setenv("GCAPS_GPRIO_KERNEL", "list")
    ctx = B.gcaps_create(0, torch.cuda.Stream().cuda_stream)
    try:
        for batch in (taskgen.config(3, 6_000), relaxed_workload(4_001, seed=8), few_gpu_tasks_workload(1_037, seed=3),
                      relaxed_workload(515, seed=9, n_cores=4, per_core=8, S=2)):
            compare(oracle, B, ctx, batch)
            _, sched = B.gcaps_rta_batch(ctx, batch, GCAPS, BUSY)
            compare(oracle, B, ctx, batch, skip=sched[0], waits=(BUSY,))
    finally:
        B.gcaps_destroy(ctx)


@pytest.mark.parametrize("shape", [(1, 1, 0), (1, 1, 1), (2, 1, 2), (3, 7, 1), (8, 4, 5), (4, 8, 2), (5, 13, 2),
                                   (2, 3, 11), (2, 17, 4), (16, 2, 3)])
def test_shapes_and_ragged_batches(oracle, gpu, shape):
    B, ctx, _ = gpu
    cores, per_core, S = shape
    for N in (1, 15, 16, 17, 257):
        compare(oracle, B, ctx, relaxed_workload(N, seed=N, n_cores=cores, per_core=per_core, S=S))


def test_priority_ties_cpu_only_tasks_and_constrained_deadlines(oracle, gpu):
    B, ctx, _ = gpu
    rng = np.random.default_rng(5)
    batch = few_gpu_tasks_workload(3_000, seed=9)
    batch["prio"] = rng.integers(-3, 4, batch["prio"].shape).astype(np.int32)
    batch["n_gseg"] = np.where(rng.random(batch["n_gseg"].shape) < 0.4, 0, batch["n_gseg"]).astype(np.uint8)
    batch["deadline_us"] = (batch["period_us"] * rng.uniform(0.6, 1.0, batch["period_us"].shape)).astype(np.uint32)
    batch["core"] = rng.integers(0, 5, batch["core"].shape).astype(np.uint8)
    found = compare(oracle, B, ctx, batch)
    assert found > 300


def test_values_beyond_24_bits(oracle, gpu):
    B, ctx, _ = gpu
    rng = np.random.default_rng(6)
    batch = relaxed_workload(1_500, seed=3, n_cores=2, per_core=4, S=2)
    scale = rng.choice([1, 1, 300, 4000], size=(1500, 1)).astype(np.uint64)
    for key in ("cpu_us", "period_us", "deadline_us"):
        batch[key] = np.minimum(batch[key].astype(np.uint64) * scale, 2**32 - 1).astype(np.uint32)
    for key in ("gm_us", "ge_us"):
        batch[key] = np.minimum(batch[key].astype(np.uint64) * scale[:, :, None], 2**32 - 1).astype(np.uint32)
    batch["eps_us"] = rng.choice([0, 200, 70_000, 2**31], size=1500).astype(np.uint32)
    batch["prio"] = (batch["prio"].astype(np.int64) * rng.choice([1, 2**26], size=(1500, 1))).astype(np.int32)
    found = compare(oracle, B, ctx, batch)
    assert found > 100
    assert 100 < B.gcaps_last_wide_count(ctx) < 1500  # both kernels took part
    big = 2**32 - 1
    one = dict(theta_us=[big], eps_us=[big], slice_us=[1], cpu_us=[[big, 5]], period_us=[[big, big]],
               deadline_us=[[big, big]], prio=[[2, 1]], core=[[0, 0]], n_gseg=[[3, 3]],
               gm_us=[[[big] * 3] * 2], ge_us=[[[big] * 3] * 2])
    compare(oracle, B, ctx, {k: np.array(v) for k, v in one.items()})
    one.update(eps_us=[0], cpu_us=[[5, 5]], gm_us=[[[1] * 3] * 2], ge_us=[[[2**30] * 3, [7] * 3]], core=[[0, 1]])
    assert compare(oracle, B, ctx, {k: np.array(v) for k, v in one.items()}) == 2


def test_invalid_taskset_is_reported(gpu):
    B, ctx, _ = gpu
    batch = relaxed_workload(300, seed=1)
    for key, value in (("period_us", 0), ("deadline_us", 0), ("n_gseg", 200)):
        bad = {k: v.copy() for k, v in batch.items()}
        bad[key][137, 2] = value
        with pytest.raises(B.GcapsError) as e:
            B.gcaps_gprio_assign_batch(ctx, bad, BUSY)
        assert e.value.code == B.GCAPS_ETASK and e.value.first_bad == 137
    bad = {k: v.copy() for k, v in batch.items()}
    bad["deadline_us"][5, 0] = bad["period_us"][5, 0] + 1
    with pytest.raises(B.GcapsError) as e:
        B.gcaps_gprio_assign_batch(ctx, bad, SUSPEND)
    assert e.value.first_bad == 5
    # a skipped taskset is not looked at
    skip = np.zeros(300, np.uint8)
    skip[5] = 1
    B.gcaps_gprio_assign_batch(ctx, bad, SUSPEND, skip)


def test_device_entry_point_and_chunked_calls(oracle, gpu, monkeypatch):
    import torch
    B, ctx, stream = gpu
    batch = relaxed_workload(3_001, seed=12)
    d = B.to_device(batch)
    N, n = batch["cpu_us"].shape
    skip = (np.arange(N) % 5 == 0).astype(np.uint8)
    want_g, want_r, want_s, _ = oracle.gprio_assign_batch(batch, SUSPEND, skip=skip, threads=16)
    monkeypatch.setenv("GCAPS_CHUNK_TASKSETS", "640")
    ctx2 = B.gcaps_create(0, stream.cuda_stream)
    try:
        for c in (ctx, ctx2):
            g = torch.full((N, n), -7, dtype=torch.int32, device="cuda:0")
            r = torch.full((N, n), -7, dtype=torch.int64, device="cuda:0")
            s = torch.full((N,), 9, dtype=torch.uint8, device="cuda:0")
            torch.cuda.synchronize()
            B.gcaps_gprio_assign_batch_device(c, d, SUSPEND, torch.from_numpy(skip).to("cuda:0"), g, r, s)
            B.gcaps_status(c)
            assert (g.cpu().numpy() == want_g).all() and (r.cpu().numpy() == want_r).all()
            assert (s.cpu().numpy() == want_s).all()
    finally:
        B.gcaps_destroy(ctx2)


# ---- full sizes, in the launch configuration the benchmark times (device entry point, skip flags from the
# ---- response-time analysis with equal priorities) ----
@pytest.mark.parametrize("k,first,N", [(3, 0, 1_000_000), (4, 0, 100_000), (5, 0, 1_000_000), (5, 7_000_000, 1_000_000),
                                       (0, 0, 300_000)])
def test_full_size_workloads_device_entry(oracle, gpu, k, first, N):
    import torch
    from paper_2406_05221_amd import taskgen
    B, ctx, _ = gpu
    print(f"workload {k} tasksets [{first}, {first + N})", flush=True)
    batch = relaxed_workload(N, seed=21) if k == 0 else taskgen.config(k, N, first_index=first)
    d = B.to_device(batch)
    n = batch["cpu_us"].shape[1]
    d_r1 = torch.empty((1, N, n), dtype=torch.int64, device="cuda:0")
    d_flags = torch.empty((1, N), dtype=torch.uint8, device="cuda:0")
    d_gprio = torch.empty((N, n), dtype=torch.int32, device="cuda:0")
    d_resp = torch.empty((N, n), dtype=torch.int64, device="cuda:0")
    d_sched = torch.empty((N,), dtype=torch.uint8, device="cuda:0")
    for wait in (BUSY, SUSPEND):
        B.gcaps_rta_batch_device(ctx, d, GCAPS, wait, d_r1, d_flags)
        B.gcaps_status(ctx)
        d_skip = d_flags[0].clone()
        d_gprio.fill_(-7)
        d_resp.fill_(-7)
        d_sched.fill_(9)
        torch.cuda.synchronize()
        B.gcaps_gprio_assign_batch_device(ctx, d, wait, d_skip, d_gprio, d_resp, d_sched)
        B.gcaps_status(ctx)
        skip = d_skip.cpu().numpy()
        want_g, want_r, want_s, _ = oracle.gprio_assign_batch(batch, wait, skip=skip, threads=16)
        got_g, got_r, got_s = d_gprio.cpu().numpy(), d_resp.cpu().numpy(), d_sched.cpu().numpy()
        assert np.array_equal(got_g, want_g), np.argwhere(got_g != want_g)[:5]
        assert np.array_equal(got_r, want_r), np.argwhere(got_r != want_r)[:5]
        assert np.array_equal(got_s, want_s)
        # properties that hold at any size: a found assignment is a permutation of the levels 1..n and
        # every bound is within its deadline; everything else is all-zero / not analysed
        found = (got_s == 1) & (skip == 0)
        assert (np.sort(got_g[found], axis=1) == np.arange(1, n + 1)).all()
        assert (got_r[found] <= batch["deadline_us"][found]).all() and (got_r[found] > 0).all()
        assert (got_g[~found] == 0).all() and (got_r[~found] == -2).all()


def test_maximum_shapes(oracle, gpu):
    """255 GPU segments per task; 255 tasks per taskset (the general kernel); 32 tasks (the widest the quad-lane
    kernel takes) and 33 (the narrowest it does not)."""
    from paper_2406_05221_amd import taskgen
    B, ctx, _ = gpu
    rng = np.random.default_rng(8)
    batch = taskgen.generate(40, n_cores=2, tasks_per_core=1, max_gseg=255, util=(0.2, 0.5), eta=(0, 255),
                             share=(0.3, 0.6), period=(200_000, 1_000_000), overhead=(0, 3), slice_us=64, seed=2,
                             stream=90)
    assert compare(oracle, B, ctx, batch) > 0
    batch = relaxed_workload(33, seed=4, n_cores=5, per_core=51, S=1)
    compare(oracle, B, ctx, batch)
    for per_core, wide in ((8, 0), (11, 64)):  # 4 x 8 = 32 tasks, 3 x 11 = 33 tasks
        cores = 4 if per_core == 8 else 3
        batch = taskgen.generate(64, n_cores=cores, tasks_per_core=per_core, max_gseg=2, util=(0.1, 0.4), eta=(0, 2),
                                 share=(0.05, 0.4), period=(50_000, 1_000_000), overhead=(0, 20), slice_us=1024,
                                 seed=int(rng.integers(1, 99)), stream=91)
        assert compare(oracle, B, ctx, batch) > 0
        assert B.gcaps_last_wide_count(ctx) == wide


# ---- the analysis of Sec. 5.4 for priorities given by the caller ----
def admissible_levels(batch, rng):
    """Random GPU priority levels that agree with the CPU priority order on every core."""
    N, n = batch["prio"].shape
    levels = np.argsort(rng.random((N, n)), axis=1).astype(np.int32) + 1
    for s in range(N):
        for c in np.unique(batch["core"][s]):
            on = np.flatnonzero(batch["core"][s] == c)
            by_cpu = on[np.argsort(-batch["prio"][s, on], kind="stable")]  # highest CPU priority first
            levels[s, by_cpu] = np.sort(levels[s, on])[::-1]
    return levels


def test_analysis_for_given_priorities(oracle, gpu):
    from paper_2406_05221_amd import taskgen
    B, ctx, _ = gpu
    rng = np.random.default_rng(12)
    cases = [relaxed_workload(1_500, seed=6), few_gpu_tasks_workload(1_500, seed=6), taskgen.config(3, 1_000),
             taskgen.config(4, 300), relaxed_workload(257, seed=3, n_cores=1, per_core=1, S=0)]
    passing = 0
    for batch in cases:
        for wait in (BUSY, SUSPEND):
            for gprio in (batch["prio"], admissible_levels(batch, rng)):
                want_r, want_s = oracle.gprio_rta_batch(batch, gprio, wait)
                got_r, got_s = B.gcaps_gprio_rta_batch(ctx, batch, wait, gprio)
                assert np.array_equal(got_r, want_r), np.argwhere(got_r != want_r)[:5]
                assert np.array_equal(got_s, want_s) and (got_r != -2).all()
                passing += int(want_s.sum())
    assert passing > 500
    # what the search assigns passes here with the same bounds
    batch = cases[0]
    g, r, s = B.gcaps_gprio_assign_batch(ctx, batch, SUSPEND)
    found = np.flatnonzero(s)
    sub = {k: v[found] for k, v in batch.items()}
    got_r, got_s = B.gcaps_gprio_rta_batch(ctx, sub, SUSPEND, g[found])
    assert len(found) > 100 and (got_s == 1).all() and np.array_equal(got_r, r[found])


def test_given_priorities_ties_big_values_and_rejections(oracle, gpu):
    B, ctx, _ = gpu
    rng = np.random.default_rng(13)
    batch = relaxed_workload(1_200, seed=8, n_cores=2, per_core=4, S=2)
    scale = rng.choice([1, 1, 300, 4000], size=(1200, 1)).astype(np.uint64)
    for key in ("cpu_us", "period_us", "deadline_us"):
        batch[key] = np.minimum(batch[key].astype(np.uint64) * scale, 2**32 - 1).astype(np.uint32)
    for key in ("gm_us", "ge_us"):
        batch[key] = np.minimum(batch[key].astype(np.uint64) * scale[:, :, None], 2**32 - 1).astype(np.uint32)
    batch["eps_us"] = rng.choice([0, 200, 70_000, 2**31], size=1200).astype(np.uint32)
    tight = rng.random(batch["deadline_us"].shape) < 0.1  # own demand beyond the deadline: jitters at zero
    batch["deadline_us"] = np.where(tight, np.maximum(1, batch["deadline_us"] // 50), batch["deadline_us"]).astype(np.uint32)
    levels = admissible_levels(batch, rng)
    coarse = (levels + 1) // 2 * np.int32(-2**30 // 4)  # ties and large negative values; order kept up to ties
    for gprio in (levels, np.zeros_like(levels), -coarse):
        try:
            want = oracle.gprio_rta_batch(batch, gprio, BUSY)
        except oracle.OracleError as e:
            assert e.code == oracle.EORDER
            with pytest.raises(B.GcapsError) as g:
                B.gcaps_gprio_rta_batch(ctx, batch, BUSY, gprio)
            assert g.value.code == B.GCAPS_ETASK and g.value.first_bad == e.first_bad
            continue
        got = B.gcaps_gprio_rta_batch(ctx, batch, BUSY, gprio)
        assert np.array_equal(got[0], want[0]) and np.array_equal(got[1], want[1])
    # an order that inverts two tasks of one core
    bad = levels.copy()
    s = 77
    on = np.flatnonzero(batch["core"][s] == batch["core"][s, 0])
    assert len(on) >= 2
    a, b = on[0], on[1]
    bad[s, a], bad[s, b] = bad[s, b], bad[s, a]
    with pytest.raises(B.GcapsError) as e:
        B.gcaps_gprio_rta_batch(ctx, batch, SUSPEND, bad)
    assert e.value.code == B.GCAPS_ETASK and e.value.first_bad == s


def test_given_priorities_device_entry_point_chunked(oracle, gpu, monkeypatch):
    import torch
    B, ctx, stream = gpu
    batch = relaxed_workload(2_001, seed=14)
    levels = admissible_levels(batch, np.random.default_rng(1))
    want_r, want_s = oracle.gprio_rta_batch(batch, levels, SUSPEND)
    d = B.to_device(batch)
    monkeypatch.setenv("GCAPS_CHUNK_TASKSETS", "640")
    ctx2 = B.gcaps_create(0, stream.cuda_stream)
    try:
        for c in (ctx, ctx2):
            r = torch.full(want_r.shape, -7, dtype=torch.int64, device="cuda:0")
            s = torch.full(want_s.shape, 9, dtype=torch.uint8, device="cuda:0")
            torch.cuda.synchronize()
            B.gcaps_gprio_rta_batch_device(c, d, SUSPEND, torch.from_numpy(levels).to("cuda:0"), r, s)
            B.gcaps_status(c)
            assert np.array_equal(r.cpu().numpy(), want_r) and np.array_equal(s.cpu().numpy(), want_s)
    finally:
        B.gcaps_destroy(ctx2)


def test_calls_of_every_kind_interleaved_on_one_context(oracle, gpu, monkeypatch):
    """The per-call device words (invalid-taskset index, hand-over counts, list and tile counters) are
    prepared for the next call by the last kernel of the one before it, whatever kind either is, also
    after a call that reported an invalid taskset and with calls split into chunks."""
    import torch
    B, _, stream = gpu
    monkeypatch.setenv("GCAPS_CHUNK_TASKSETS", "448")
    ctx = B.gcaps_create(0, stream.cuda_stream)
    try:
        small = relaxed_workload(300, seed=41)          # one chunk
        large = relaxed_workload(1_500, seed=42)        # four chunks
        wide = relaxed_workload(400, seed=43, n_cores=2, per_core=4, S=2)
        wide["period_us"] = (wide["period_us"].astype(np.uint64) * 3000).astype(np.uint32)  # beyond 24 bits
        wide["deadline_us"] = wide["period_us"].copy()
        bad = {k: v.copy() for k, v in small.items()}
        bad["period_us"][123, 1] = 0
        want = {}
        for name, b in (("small", small), ("large", large), ("wide", wide)):
            want[name] = (oracle.rta_batch(b, 3, SUSPEND, threads=16)[:2],
                          oracle.gprio_assign_batch(b, SUSPEND, threads=16)[:3],
                          oracle.gprio_rta_batch(b, b["prio"], SUSPEND))
        batches = dict(small=small, large=large, wide=wide)
        for round_ in range(2):
            for name in ("small", "wide", "large", "small"):
                b = batches[name]
                got = B.gcaps_rta_batch(ctx, b, 3, SUSPEND)
                assert all(np.array_equal(x, y) for x, y in zip(got, want[name][0])), (round_, name, "rta")
                assert (B.gcaps_last_wide_count(ctx) > 0) == (name == "wide")
                with pytest.raises(B.GcapsError) as e:
                    B.gcaps_gprio_assign_batch(ctx, bad, SUSPEND)
                assert e.value.first_bad == 123
                got = B.gcaps_gprio_assign_batch(ctx, b, SUSPEND)
                assert all(np.array_equal(x, y) for x, y in zip(got, want[name][1])), (round_, name, "assign")
                got = B.gcaps_gprio_rta_batch(ctx, b, SUSPEND, b["prio"])
                assert all(np.array_equal(x, y) for x, y in zip(got, want[name][2])), (round_, name, "given")
                with pytest.raises(B.GcapsError):
                    B.gcaps_rta_batch(ctx, bad, 3, SUSPEND)
    finally:
        B.gcaps_destroy(ctx)


def test_captured_search_replays(oracle):
    """The device entry point of the priority search recorded into a HIP graph (after a warm-up call that made the
    context's allocations) and replayed, with eager calls of other sizes between the replays."""
    import torch
    from paper_2406_05221_amd import binding as B
    stream = torch.cuda.Stream()
    ctx = B.gcaps_create(0, stream.cuda_stream)
    try:
        batch, other = relaxed_workload(3_000, seed=61), relaxed_workload(555, seed=62)
        want = oracle.gprio_assign_batch(batch, SUSPEND, threads=16)[:3]
        ref = oracle.gprio_assign_batch(other, BUSY, threads=16)[:3]
        d = B.to_device(batch)
        N, n = batch["cpu_us"].shape
        d_gprio = torch.empty((N, n), dtype=torch.int32, device="cuda:0")
        d_resp = torch.empty((N, n), dtype=torch.int64, device="cuda:0")
        d_sched = torch.empty((N,), dtype=torch.uint8, device="cuda:0")
        B.gcaps_gprio_assign_batch_device(ctx, d, SUSPEND, None, d_gprio, d_resp, d_sched)  # warm-up
        B.gcaps_status(ctx)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            B.gcaps_gprio_assign_batch_device(ctx, d, SUSPEND, None, d_gprio, d_resp, d_sched)
        for k in range(3):
            d_gprio.fill_(-7)
            d_resp.fill_(-7)
            d_sched.fill_(9)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert np.array_equal(d_gprio.cpu().numpy(), want[0]) and np.array_equal(d_resp.cpu().numpy(), want[1]), k
            assert np.array_equal(d_sched.cpu().numpy(), want[2]), k
            got = B.gcaps_gprio_assign_batch(ctx, other, BUSY)
            assert all(np.array_equal(g, w) for g, w in zip(got, ref)), k
        B.gcaps_status(ctx)
        # the analysis for given priorities, recorded and replayed likewise
        given = np.where(want[2][:, None].astype(bool), want[0], batch["prio"]).astype(np.int32)
        want_r, want_s = oracle.gprio_rta_batch(batch, given, SUSPEND)
        d_given = torch.from_numpy(given).cuda()
        B.gcaps_gprio_rta_batch_device(ctx, d, SUSPEND, d_given, d_resp, d_sched)  # warm-up
        B.gcaps_status(ctx)
        graph2 = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph2, stream=stream):
            B.gcaps_gprio_rta_batch_device(ctx, d, SUSPEND, d_given, d_resp, d_sched)
        for k in range(2):
            d_resp.fill_(-7)
            d_sched.fill_(9)
            torch.cuda.synchronize()
            graph2.replay()
            torch.cuda.synchronize()
            assert np.array_equal(d_resp.cpu().numpy(), want_r) and np.array_equal(d_sched.cpu().numpy(), want_s), k
            got = B.gcaps_gprio_assign_batch(ctx, other, BUSY)
            assert all(np.array_equal(g, w) for g, w in zip(got, ref)), k
        B.gcaps_status(ctx)
    finally:
        B.gcaps_destroy(ctx)
