"""GPU library against the CPU oracle, bit for bit: every response time (int64 microseconds,
sentinels included) and every schedulable flag, through the C ABI."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

GCAPS, RR, BOTH, BUSY, SUSPEND = 1, 2, 3, 0, 1


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2406_05221_amd import binding as B
    stream = torch.cuda.Stream()
    ctx = B.gcaps_create(0, stream.cuda_stream)
    yield B, ctx, stream
    B.gcaps_destroy(ctx)


def compare(oracle, B, ctx, batch, policy=BOTH, waits=(BUSY, SUSPEND)):
    for wait in waits:
        want_r, want_s, _ = oracle.rta_batch(batch, policy, wait, threads=16)
        got_r, got_s = B.gcaps_rta_batch(ctx, batch, policy, wait)
        bad = np.argwhere(got_r != want_r)
        assert bad.size == 0, (wait, bad[:5], got_r[tuple(bad[0])], want_r[tuple(bad[0])])
        assert (got_s == want_s).all()


@pytest.mark.parametrize("k,N", [(1, None), (2, None), (3, 20_000), (4, 3_000), (5, 21_600)])
def test_named_workloads(oracle, gpu, k, N):
    from paper_2406_05221_amd import taskgen
    B, ctx, _ = gpu
    print(f"workload {k} N={N}", flush=True)
    compare(oracle, B, ctx, taskgen.config(k, N))
    # the named workloads fit the 24-bit fast kernel entirely
    assert B.gcaps_last_wide_count(ctx) == 0


def relaxed_workload(N, seed, n_cores=4, per_core=5, S=3):
    """Like workload 3 but with long periods and small overheads, so that a good part of the
    tasksets is schedulable under GCAPS and the fixed-point iterations run long."""
    from paper_2406_05221_amd import taskgen
    return taskgen.generate(N, n_cores=n_cores, tasks_per_core=per_core, max_gseg=S, util=(0.25, 0.85), eta=(0, S),
                            share=(0.05, 0.5), period=(20_000, 1_000_000), overhead=(0, 40), slice_us=1024,
                            seed=seed, stream=77)


def few_gpu_tasks_workload(N, seed):
    """Few GPU-using tasks and long periods: mostly schedulable under round-robin as well."""
    from paper_2406_05221_amd import taskgen
    return taskgen.generate(N, n_cores=4, tasks_per_core=4, max_gseg=2, util=(0.2, 0.7), eta=(0, 1),
                            share=(0.05, 0.3), period=(50_000, 1_000_000), overhead=(0, 20), slice_us=256,
                            seed=seed, stream=78)


@pytest.mark.parametrize("policy", [GCAPS, RR, BOTH])
def test_mostly_schedulable_tasksets(oracle, gpu, policy):
    B, ctx, _ = gpu
    batch = relaxed_workload(5_003, seed=policy)
    want_s = oracle.rta_batch(batch, GCAPS, SUSPEND, threads=16)[1]
    assert 0.2 < want_s.mean() < 0.98
    compare(oracle, B, ctx, batch, policy)
    assert B.gcaps_last_wide_count(ctx) == 0
    batch = few_gpu_tasks_workload(5_003, seed=policy)
    want_s = oracle.rta_batch(batch, RR, BUSY, threads=16)[1]
    assert 0.2 < want_s.mean() < 0.98
    compare(oracle, B, ctx, batch, policy)


@pytest.mark.parametrize("shape", [(1, 1, 0), (1, 1, 1), (2, 1, 2), (3, 7, 1), (8, 10, 5), (5, 51, 2), (2, 3, 11),
                                   (3, 11, 7), (2, 17, 4), (4, 16, 3)])
def test_shapes_and_ragged_batches(oracle, gpu, shape):
    B, ctx, _ = gpu
    cores, per_core, S = shape
    for N in (1, 63, 64, 65, 257):
        batch = relaxed_workload(N, seed=N, n_cores=cores, per_core=per_core, S=S)
        compare(oracle, B, ctx, batch)


def test_priority_ties_and_cpu_only_tasks(oracle, gpu):
    B, ctx, _ = gpu
    rng = np.random.default_rng(5)
    batch = relaxed_workload(2_000, seed=9)
    batch["prio"] = rng.integers(-3, 4, batch["prio"].shape).astype(np.int32)
    batch["n_gseg"] = np.where(rng.random(batch["n_gseg"].shape) < 0.4, 0, batch["n_gseg"]).astype(np.uint8)
    batch["deadline_us"] = (batch["period_us"] * rng.uniform(0.5, 1.0, batch["period_us"].shape)).astype(np.uint32)
    batch["core"] = rng.integers(0, 3, batch["core"].shape).astype(np.uint8)
    compare(oracle, B, ctx, batch)


def test_values_beyond_24_bits(oracle, gpu):
    """Periods of hours, nanosecond-like slices, overheads near 2^32: exact all the same."""
    B, ctx, _ = gpu
    rng = np.random.default_rng(6)
    batch = relaxed_workload(1_500, seed=3, n_cores=2, per_core=4, S=2)
    scale = rng.choice([1, 1, 300, 4000], size=(1500, 1)).astype(np.uint64)
    for key in ("cpu_us", "period_us", "deadline_us"):
        batch[key] = np.minimum(batch[key].astype(np.uint64) * scale, 2**32 - 1).astype(np.uint32)
    for key in ("gm_us", "ge_us"):
        batch[key] = np.minimum(batch[key].astype(np.uint64) * scale[:, :, None], 2**32 - 1).astype(np.uint32)
    batch["slice_us"] = rng.choice([1, 7, 1024, 2**31], size=1500).astype(np.uint32)
    batch["theta_us"] = rng.choice([0, 200, 2**32 - 1], size=1500).astype(np.uint32)
    batch["eps_us"] = rng.choice([0, 200, 2**31], size=1500).astype(np.uint32)
    compare(oracle, B, ctx, batch)
    assert 100 < B.gcaps_last_wide_count(ctx) < 1500  # both kernels took part
    big = 2**32 - 1
    one = dict(theta_us=[big], eps_us=[big], slice_us=[1], cpu_us=[[big, 5]], period_us=[[big, big]],
               deadline_us=[[big, big]], prio=[[2, 1]], core=[[0, 0]], n_gseg=[[3, 3]],
               gm_us=[[[big] * 3] * 2], ge_us=[[[big] * 3] * 2])
    one = {k: np.array(v) for k, v in one.items()}
    compare(oracle, B, ctx, one)


def test_invalid_taskset_is_reported(gpu):
    B, ctx, _ = gpu
    batch = relaxed_workload(300, seed=1)
    for key, value in (("period_us", 0), ("deadline_us", 0), ("slice_us", 0), ("n_gseg", 200)):
        bad = {k: v.copy() for k, v in batch.items()}
        if key == "slice_us":
            bad[key][211] = value
            bad[key][250] = value
        else:
            bad[key][211, 3] = value
            bad[key][250, 0] = value
        with pytest.raises(B.GcapsError) as e:
            B.gcaps_rta_batch(ctx, bad, BOTH, BUSY)
        assert e.value.code == B.GCAPS_ETASK and e.value.first_bad == 211
    bad = {k: v.copy() for k, v in batch.items()}
    bad["deadline_us"][7, 2] = bad["period_us"][7, 2] + 1
    with pytest.raises(B.GcapsError) as e:
        B.gcaps_rta_batch(ctx, bad, GCAPS, SUSPEND)
    assert e.value.first_bad == 7
    # the context stays usable
    B.gcaps_rta_batch(ctx, batch, BOTH, BUSY)


def test_device_entry_point_matches_host_entry_point(oracle, gpu):
    import torch
    from paper_2406_05221_amd import taskgen
    B, ctx, stream = gpu
    batch = taskgen.config(3, 10_000, first_index=500_000)
    d = B.to_device(batch)
    N, n = batch["cpu_us"].shape
    for policy in (GCAPS, RR, BOTH):
        P = B.npol(policy)
        d_resp = torch.full((P, N, n), -7, dtype=torch.int64, device="cuda:0")
        d_sched = torch.full((P, N), 9, dtype=torch.uint8, device="cuda:0")
        torch.cuda.synchronize()
        B.gcaps_rta_batch_device(ctx, d, policy, SUSPEND, d_resp, d_sched)
        B.gcaps_status(ctx)
        want_r, want_s, _ = oracle.rta_batch(batch, policy, SUSPEND, threads=16)
        assert (d_resp.cpu().numpy() == want_r).all() and (d_sched.cpu().numpy() == want_s).all()


# ---- full sizes, in the launch configuration the benchmark times (device entry point, both policies) ----
def full_size_cases():
    from paper_2406_05221_amd import taskgen
    cases = [(1, 0, 1000), (2, 0, 9000), (3, 0, 1_000_000), (4, 0, 100_000)]
    cases += [(5, k * 1_000_000, 1_000_000) for k in range(10)]  # workload 5 streamed in 1M batches
    return cases


@pytest.mark.parametrize("k,first,N", full_size_cases())
def test_full_size_workloads_device_entry(oracle, gpu, k, first, N):
    """Every response time and flag of every taskset of the five workloads, both waiting modes."""
    import torch
    from paper_2406_05221_amd import taskgen
    B, ctx, _ = gpu
    print(f"workload {k} tasksets [{first}, {first + N})", flush=True)
    batch = taskgen.config(k, N, first_index=first)
    d = B.to_device(batch)
    n = batch["cpu_us"].shape[1]
    d_resp = torch.empty((2, N, n), dtype=torch.int64, device="cuda:0")
    d_sched = torch.empty((2, N), dtype=torch.uint8, device="cuda:0")
    for wait in (BUSY, SUSPEND):
        d_resp.fill_(-7)
        d_sched.fill_(9)
        torch.cuda.synchronize()
        B.gcaps_rta_batch_device(ctx, d, BOTH, wait, d_resp, d_sched)
        B.gcaps_status(ctx)
        assert B.gcaps_last_wide_count(ctx) == 0
        want_r, want_s, _ = oracle.rta_batch(batch, BOTH, wait, threads=16)
        got_r = d_resp.cpu().numpy()
        assert np.array_equal(got_r, want_r), np.argwhere(got_r != want_r)[:5]
        assert np.array_equal(d_sched.cpu().numpy(), want_s)
        # properties that hold at any size: sentinels are consistent with the flags
        miss = (got_r == -1).sum(axis=2)
        assert ((miss == 0) == (d_sched.cpu().numpy() == 1)).all() and miss.max() <= 1


def test_binning_does_not_change_results(oracle, gpu):
    from paper_2406_05221_amd import taskgen
    B, ctx, _ = gpu
    batch = taskgen.config(5, 50_000, first_index=123_456)
    want = oracle.rta_batch(batch, BOTH, SUSPEND, threads=16)
    try:
        B.gcaps_set_binning(ctx, 1)
        got_r, got_s = B.gcaps_rta_batch(ctx, batch, BOTH, SUSPEND)
        assert np.array_equal(got_r, want[0]) and np.array_equal(got_s, want[1])
        compare(oracle, B, ctx, relaxed_workload(7_001, seed=11))
    finally:
        B.gcaps_set_binning(ctx, 0)
    got_r, got_s = B.gcaps_rta_batch(ctx, batch, BOTH, SUSPEND)
    assert np.array_equal(got_r, want[0]) and np.array_equal(got_s, want[1])


def test_chunked_calls(oracle, monkeypatch):
    """Calls too large for 32-bit byte offsets are split into chunks of tasksets; forced here with
    a small chunk size.  Policy strides, the invalid-taskset index and the 64-bit hand-over count
    must all refer to the whole call."""
    import torch
    from paper_2406_05221_amd import binding as B
    monkeypatch.setenv("GCAPS_CHUNK_TASKSETS", "1000")
    monkeypatch.setenv("GCAPS_SCREEN_TASKS", "2")
    ctx = B.gcaps_create(0, torch.cuda.Stream().cuda_stream)
    try:
        batch = relaxed_workload(4_321, seed=21)
        batch["period_us"][[5, 1500, 4000], 0] = 2**23  # beyond the fast kernel's range: three chunks hand over
        batch["deadline_us"][[5, 1500, 4000], 0] = 2**23
        compare(oracle, B, ctx, batch)
        assert B.gcaps_last_wide_count(ctx) == 3
        compare(oracle, B, ctx, batch, policy=RR, waits=(BUSY,))
        bad = {k: v.copy() for k, v in batch.items()}
        bad["period_us"][3456, 7] = 0
        with pytest.raises(B.GcapsError) as e:
            B.gcaps_rta_batch(ctx, bad, BOTH, BUSY)
        assert e.value.first_bad == 3456
    finally:
        B.gcaps_destroy(ctx)


@pytest.mark.parametrize("screen_tasks,deep_lanes,deep_kernel", [(1, 4, ""), (3, 8, ""), (4, 8, ""), (6, 4, ""), (6, 8, ""),
                                                                  (9, 4, ""), (64, 4, ""), (4, 4, "lds"), (2, 4, "lds"),
                                                                  (7, 4, "lds")])
def test_launch_split_knobs(oracle, monkeypatch, screen_tasks, deep_lanes, deep_kernel):
    """How many ranks the first launch analyses and how many lanes share a taskset in the second
    are tuning knobs: results are the same for every setting, also where the second launch resumes
    from more ranks than it has lanes per taskset, and where the first launch settles everything."""
    import torch
    from paper_2406_05221_amd import binding as B
    monkeypatch.setenv("GCAPS_SCREEN_TASKS", str(screen_tasks))
    monkeypatch.setenv("GCAPS_DEEP_LANES", str(deep_lanes))
    if deep_kernel:
        monkeypatch.setenv("GCAPS_DEEP_KERNEL", deep_kernel)  # the LDS-record form of the second launch for every shape
    ctx = B.gcaps_create(0, torch.cuda.Stream().cuda_stream)
    try:
        compare(oracle, B, ctx, relaxed_workload(3_001, seed=31))
        compare(oracle, B, ctx, relaxed_workload(517, seed=32, n_cores=3, per_core=11, S=5))
        compare(oracle, B, ctx, few_gpu_tasks_workload(1_003, seed=33), policy=RR)
        from paper_2406_05221_amd import taskgen
        compare(oracle, B, ctx, taskgen.config(3, 10_000, first_index=500_000))
    finally:
        B.gcaps_destroy(ctx)


def test_out_of_range_values_below_the_screened_ranks(oracle, gpu):
    """Values outside the fast kernels' range in LOW-priority tasks only: the first launch does not
    look at them, the second hands the taskset over to the 64-bit kernel when it gets there."""
    B, ctx, _ = gpu
    rng = np.random.default_rng(8)
    batch = relaxed_workload(2_000, seed=41, n_cores=4, per_core=10, S=2)
    order = np.argsort(-batch["prio"], axis=1, kind="stable")
    rows = np.arange(2_000)
    low = order[rows, rng.integers(8, 40, 2_000)]
    pick = rng.random(2_000) < 0.3
    batch["prio"][rows[pick], low[pick]] = -(2**30)           # far below the 24-bit key range
    pick2 = rng.random(2_000) < 0.2
    batch["period_us"][rows[pick2], low[pick2]] = 2**24       # beyond the reciprocal's range
    batch["deadline_us"][rows[pick2], low[pick2]] = 2**24
    compare(oracle, B, ctx, batch)
    assert B.gcaps_last_wide_count(ctx) > 0


def test_outputs_at_8_byte_alignment_only(oracle, gpu):
    """Response buffers that are 8- but not 16-byte aligned (a view into a larger buffer), with
    even and odd task counts: the kernels may use wider stores only where they are aligned."""
    import torch
    B, ctx, _ = gpu
    for per_core in (5, 3):  # n = 20, n = 9
        batch = relaxed_workload(1_111, seed=51, n_cores=4 if per_core == 5 else 3, per_core=per_core, S=3)
        d = B.to_device(batch)
        N, n = batch["cpu_us"].shape
        want_r, want_s, _ = oracle.rta_batch(batch, BOTH, BUSY, threads=16)
        for shift in (0, 1):
            raw = torch.full((2 * N * n + 2,), -7, dtype=torch.int64, device="cuda:0")
            d_resp = raw[shift:shift + 2 * N * n].view(2, N, n)
            assert d_resp.data_ptr() % 16 == 8 * shift
            d_sched = torch.full((2, N), 9, dtype=torch.uint8, device="cuda:0")
            torch.cuda.synchronize()
            B.gcaps_rta_batch_device(ctx, d, BOTH, BUSY, d_resp, d_sched)
            B.gcaps_status(ctx)
            assert (d_resp.cpu().numpy() == want_r).all() and (d_sched.cpu().numpy() == want_s).all()
            assert (raw[:shift] == -7).all() and (raw[shift + 2 * N * n:] == -7).all()  # nothing outside the view


def test_inputs_at_element_alignment_only(oracle, gpu):
    """Every input array starts one element into a larger buffer: 4-byte aligned words, 1-byte aligned bytes.  The
    kernels load several segment slots of a task with one instruction and stream arrays with wide accesses; none of
    it may assume more than the element's own alignment.  Shapes with 1 to 5 segment slots, both entry points of the
    analysis and the priority search."""
    import torch
    B, ctx, _ = gpu

    def shifted(batch):
        out = {}
        for name, t in B.to_device(batch).items():
            raw = torch.empty(t.numel() + 1, dtype=t.dtype, device="cuda:0")
            raw[1:] = t.flatten()
            out[name] = raw[1:].view(t.shape)
            assert out[name].data_ptr() % 16 == t.element_size() and out[name].is_contiguous()
        return out

    for S in (1, 2, 3, 4, 5):
        batch = relaxed_workload(1_037, seed=80 + S, n_cores=4, per_core=5, S=S)
        N, n = batch["cpu_us"].shape
        d = shifted(batch)
        d_resp = torch.empty((2, N, n), dtype=torch.int64, device="cuda:0")
        d_sched = torch.empty((2, N), dtype=torch.uint8, device="cuda:0")
        for wait in (BUSY, SUSPEND):
            torch.cuda.synchronize()
            B.gcaps_rta_batch_device(ctx, d, BOTH, wait, d_resp, d_sched)
            B.gcaps_status(ctx)
            want_r, want_s, _ = oracle.rta_batch(batch, BOTH, wait, threads=16)
            assert (d_resp.cpu().numpy() == want_r).all() and (d_sched.cpu().numpy() == want_s).all(), (S, wait)
            d_gprio = torch.empty((N, n), dtype=torch.int32, device="cuda:0")
            g_resp = torch.empty((N, n), dtype=torch.int64, device="cuda:0")
            g_sched = torch.empty((N,), dtype=torch.uint8, device="cuda:0")
            B.gcaps_gprio_assign_batch_device(ctx, d, wait, None, d_gprio, g_resp, g_sched)
            B.gcaps_status(ctx)
            wg, wr, ws, _ = oracle.gprio_assign_batch(batch, wait, threads=16)
            assert (d_gprio.cpu().numpy() == wg).all() and (g_resp.cpu().numpy() == wr).all()
            assert (g_sched.cpu().numpy() == ws).all(), (S, wait)


def test_priorities_that_look_like_internal_marks(oracle, gpu):
    """Any int32 is a legal priority.  Values around 2^30 (the first launch marks looked-up tasks
    with such words in the priority column) and the extremes must not confuse anything."""
    B, ctx, _ = gpu
    rng = np.random.default_rng(12)
    batch = relaxed_workload(3_000, seed=61)
    odd = rng.choice([2**30, 2**30 + 1, 2**30 + 2, 2**30 + 3, -(2**31), 2**31 - 1, 2**22, -(2**22) - 1],
                     size=batch["prio"].shape)
    hit = rng.random(batch["prio"].shape) < 0.05
    batch["prio"] = np.where(hit, odd, batch["prio"]).astype(np.int32)
    compare(oracle, B, ctx, batch)
    assert B.gcaps_last_wide_count(ctx) > 0


# ---- continue-after-miss: every task analysed, D_h for the unknown R_h below a miss ----
def compare_continue(oracle, B, batch, policy=BOTH, waits=(BUSY, SUSPEND), env=None):
    import torch
    ctx = B.gcaps_create(0, torch.cuda.Stream().cuda_stream)
    B.gcaps_set_continue_after_miss(ctx, 1)
    try:
        for wait in waits:
            want_r, want_s, _ = oracle.rta_batch(batch, policy, wait, threads=16,
                                                 options=oracle.OPT_CONTINUE_AFTER_MISS)
            got_r, got_s = B.gcaps_rta_batch(ctx, batch, policy, wait)
            bad = np.argwhere(got_r != want_r)
            assert bad.size == 0, (wait, bad[:5], got_r[tuple(bad[0])], want_r[tuple(bad[0])])
            assert (got_s == want_s).all() and (got_r != -2).all()
        wide = B.gcaps_last_wide_count(ctx)
        # switching the option off again restores the default analysis
        B.gcaps_set_continue_after_miss(ctx, 0)
        want_r, want_s, _ = oracle.rta_batch(batch, policy, BUSY, threads=16)
        got_r, got_s = B.gcaps_rta_batch(ctx, batch, policy, BUSY)
        assert (got_r == want_r).all() and (got_s == want_s).all()
        return wide
    finally:
        B.gcaps_destroy(ctx)


@pytest.mark.parametrize("k,N", [(1, None), (2, None), (3, 20_000), (4, 3_000), (5, 21_600)])
def test_continue_after_miss_named_workloads(oracle, gpu, k, N):
    from paper_2406_05221_amd import taskgen
    B, _, _ = gpu
    print(f"workload {k} N={N}", flush=True)
    batch = taskgen.config(k, N)
    # a task that cannot meet its deadline may cost more than a few periods, which the 24-bit terms do not
    # hold: once such a task is committed the taskset goes to the 64-bit kernel (nearly all of workload 4 with
    # its 80 tasks per taskset)
    wide = compare_continue(oracle, B, batch)
    assert k == 4 or wide <= 0.2 * batch["cpu_us"].shape[0]


@pytest.mark.parametrize("k,N", [(3, 100_000), (5, 64_800)])
def test_continue_after_miss_busy_waiting_stays_in_the_fast_kernel(oracle, gpu, k, N):
    """Under round-robin with busy-waiting a task that cannot meet its deadline costs cgm + nu (L + theta) K (Lemma 4),
    many periods' worth.  The fast kernel caps such a cost at a few periods, which changes no result (a task that
    faces a cost above one period has no fixed point either way), instead of sending the taskset to the 64-bit
    kernel."""
    from paper_2406_05221_amd import taskgen
    B, _, _ = gpu
    wide = compare_continue(oracle, B, taskgen.config(k, N), waits=(BUSY,))
    assert wide <= N // 100


@pytest.mark.parametrize("shape", [(1, 1, 0), (2, 1, 2), (3, 7, 1), (8, 10, 5), (5, 51, 2), (2, 3, 11), (4, 16, 3)])
def test_continue_after_miss_shapes(oracle, gpu, shape):
    B, _, _ = gpu
    cores, per_core, S = shape
    for N in (1, 17, 257):
        compare_continue(oracle, B, relaxed_workload(N, seed=N, n_cores=cores, per_core=per_core, S=S))


def test_continue_after_miss_mixed_cases(oracle, gpu):
    B, _, _ = gpu
    rng = np.random.default_rng(15)
    batch = relaxed_workload(4_000, seed=19)
    # tight deadlines in the middle of many tasksets: misses with tasks below them
    tight = rng.random(batch["deadline_us"].shape) < 0.08
    batch["deadline_us"] = np.where(tight, np.maximum(1, batch["period_us"] // rng.integers(3, 40, tight.shape)),
                                    batch["deadline_us"]).astype(np.uint32)
    batch["prio"] = rng.integers(-3, 4, batch["prio"].shape).astype(np.int32)
    batch["n_gseg"] = np.where(rng.random(batch["n_gseg"].shape) < 0.3, 0, batch["n_gseg"]).astype(np.uint8)
    for policy in (GCAPS, RR, BOTH):
        compare_continue(oracle, B, batch, policy)
    # values beyond 24 bits: the 64-bit kernel in the same mode
    scale = rng.choice([1, 1, 300, 4000], size=(4000, 1)).astype(np.uint64)
    for key in ("cpu_us", "period_us", "deadline_us"):
        batch[key] = np.minimum(batch[key].astype(np.uint64) * scale, 2**32 - 1).astype(np.uint32)
    for key in ("gm_us", "ge_us"):
        batch[key] = np.minimum(batch[key].astype(np.uint64) * scale[:, :, None], 2**32 - 1).astype(np.uint32)
    assert 500 < compare_continue(oracle, B, batch) < 4000


def test_continue_after_miss_reports_invalid_tasksets(gpu):
    import torch
    B, _, _ = gpu
    ctx = B.gcaps_create(0, torch.cuda.Stream().cuda_stream)
    B.gcaps_set_continue_after_miss(ctx, 1)
    try:
        batch = relaxed_workload(300, seed=1)
        for key, value in (("period_us", 0), ("deadline_us", 0), ("slice_us", 0), ("n_gseg", 200)):
            bad = {k: v.copy() for k, v in batch.items()}
            if key == "slice_us":
                bad[key][137] = value
            else:
                bad[key][137, 2] = value
            with pytest.raises(B.GcapsError) as e:
                B.gcaps_rta_batch(ctx, bad, BOTH, BUSY)
            assert e.value.code == B.GCAPS_ETASK and e.value.first_bad == 137
    finally:
        B.gcaps_destroy(ctx)


def test_captured_call_replays(oracle, gpu):
    """One device-entry call recorded into a HIP graph (after a warm-up call that made the context's
    allocations) and replayed, with eager calls of other sizes in between: every replay gives the eager result."""
    import torch
    B, _, _ = gpu
    stream = torch.cuda.Stream()
    ctx = B.gcaps_create(0, stream.cuda_stream)
    try:
        batch, other = relaxed_workload(3_000, seed=51), relaxed_workload(777, seed=52)
        want_r, want_s, _ = oracle.rta_batch(batch, BOTH, SUSPEND, threads=16)
        d = B.to_device(batch)
        N, n = batch["cpu_us"].shape
        d_resp = torch.empty((2, N, n), dtype=torch.int64, device="cuda:0")
        d_sched = torch.empty((2, N), dtype=torch.uint8, device="cuda:0")
        B.gcaps_rta_batch_device(ctx, d, BOTH, SUSPEND, d_resp, d_sched)  # warm-up: allocations happen here
        B.gcaps_status(ctx)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            B.gcaps_rta_batch_device(ctx, d, BOTH, SUSPEND, d_resp, d_sched)
        for k in range(4):
            d_resp.fill_(-7)
            d_sched.fill_(9)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert np.array_equal(d_resp.cpu().numpy(), want_r) and np.array_equal(d_sched.cpu().numpy(), want_s), k
            # eager work of the same context between the replays
            got = B.gcaps_rta_batch(ctx, other, BOTH, BUSY)
            ref = oracle.rta_batch(other, BOTH, BUSY, threads=16)
            assert np.array_equal(got[0], ref[0]) and np.array_equal(got[1], ref[1])
            if k % 2:
                B.gcaps_gprio_assign_batch(ctx, other, BUSY)
        B.gcaps_status(ctx)
    finally:
        B.gcaps_destroy(ctx)


def test_recorded_call_that_would_have_to_allocate_is_refused(oracle, gpu):
    """A call that the stream is recording into a HIP graph makes no device allocation: when it needs
    more scratch than every direct call before it, it returns GCAPS_ESIZE and leaves the context's
    buffers alone (a direct call afterwards works)."""
    import torch
    B, _, _ = gpu
    stream = torch.cuda.Stream()
    ctx = B.gcaps_create(0, stream.cuda_stream)
    try:
        small, large = relaxed_workload(500, seed=61), relaxed_workload(9_000, seed=62)
        assert np.array_equal(B.gcaps_rta_batch(ctx, small, BOTH, BUSY)[0], oracle.rta_batch(small, BOTH, BUSY)[0])
        d = B.to_device(large)
        N, n = large["cpu_us"].shape
        d_resp = torch.empty((2, N, n), dtype=torch.int64, device="cuda:0")
        d_sched = torch.empty((2, N), dtype=torch.uint8, device="cuda:0")
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        code = None
        with torch.cuda.graph(graph, stream=stream):
            try:
                B.gcaps_rta_batch_device(ctx, d, BOTH, BUSY, d_resp, d_sched)
            except B.GcapsError as e:
                code = e.code
        assert code == B.GCAPS_ESIZE
        del graph  # holds at most the status reset; never replayed
        torch.cuda.synchronize()
        B.gcaps_rta_batch_device(ctx, d, BOTH, BUSY, d_resp, d_sched)
        B.gcaps_status(ctx)
        want_r, want_s, _ = oracle.rta_batch(large, BOTH, BUSY, threads=16)
        assert np.array_equal(d_resp.cpu().numpy(), want_r) and np.array_equal(d_sched.cpu().numpy(), want_s)
    finally:
        B.gcaps_destroy(ctx)


def test_argument_and_allocation_failures_leave_the_context_usable(oracle, gpu):
    """Failures forced from the host: an empty batch (GCAPS_EINVAL) and a batch whose device copy cannot be
    allocated (GCAPS_ENOMEM: the sizes ask for petabytes; no array is touched before the allocation fails)."""
    import ctypes
    B, ctx, _ = gpu
    good = relaxed_workload(300, seed=71)
    keep = {name: np.ascontiguousarray(good[name], dtype=dtype) for name, dtype, _ in B._FIELDS}
    resp = np.empty((2, 300, 20), np.int64)
    sched = np.empty((2, 300), np.uint8)
    bad = ctypes.c_uint32(0)

    def call(n_tasksets, n_tasks, max_gseg):
        b = B.gcaps_batch(n_tasksets=n_tasksets, n_tasks=n_tasks, max_gseg=max_gseg)
        for name in keep:
            setattr(b, name, keep[name].ctypes.data)
        return B._lib.gcaps_rta_batch(ctx, ctypes.byref(b), BOTH, BUSY, resp.ctypes.data, sched.ctypes.data,
                                      ctypes.byref(bad))

    assert call(0, 20, 3) == B.GCAPS_EINVAL
    assert call(300, 0, 3) == B.GCAPS_EINVAL
    assert call(300, 256, 3) == B.GCAPS_EINVAL
    assert call(0xFFFFFFFF, 255, 255) == B.GCAPS_ENOMEM
    assert "allocation" in B.gcaps_strerror(B.GCAPS_ENOMEM)
    assert call(300, 20, 3) == B.GCAPS_OK
    want_r, want_s, _ = oracle.rta_batch(good, BOTH, BUSY)
    assert np.array_equal(resp, want_r) and np.array_equal(sched, want_s)


def test_rate_probes_report_plausible_rates(gpu):
    """The denominators the benchmark prints: integer VALU rates by instruction kind and HBM rates of plain
    streaming kernels.  Loose physical limits only (a rate of zero means a launch failed); the context goes on
    working afterwards, and arguments the probe cannot use are refused."""
    import ctypes
    B, ctx, _ = gpu
    valu = B.gcaps_valu_probe(ctx)
    assert valu["cu_count"] > 0 and valu["wavefront_size"] == 64
    for kind, rate in valu["lane_ops_per_s"].items():
        assert 0.2 * valu["spec_lane_ops_per_s"] < rate < 2.5 * valu["spec_lane_ops_per_s"], (kind, rate)
    hbm = B.gcaps_hbm_probe(ctx, 1 << 28)
    assert set(hbm) == set(B.HBM_KINDS)
    for kind, rate in hbm.items():
        assert 0.5e12 < rate < 30e12, (kind, rate)  # 256 MiB may sit in the memory-side cache: above the HBM peak
    r = B.gcaps_hbm_rates()
    assert B._lib.gcaps_hbm_probe(ctx, 1000, ctypes.byref(r)) == B.GCAPS_EINVAL
    assert B._lib.gcaps_hbm_probe(ctx, (1 << 20) + 8, ctypes.byref(r)) == B.GCAPS_EINVAL
    assert B._lib.gcaps_hbm_probe(ctx, 1 << 50, ctypes.byref(r)) == B.GCAPS_ENOMEM
    B.gcaps_status(ctx)
