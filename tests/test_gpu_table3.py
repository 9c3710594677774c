"""Tasksets drawn by the recipe of Sec. 6.1 / Table 3 (task counts 12..24 per taskset, CPU-only tasks,
worst-fit-decreasing allocation): every analysis and the priority search against the oracle, and the
sweep module's shares against the same shares computed with the oracle."""
import numpy as np
import pytest

from test_gpu_parity import gpu  # noqa: F401 (fixture)

pytestmark = pytest.mark.gpu

GCAPS, RR, BOTH, BUSY, SUSPEND = 1, 2, 3, 0, 1


def oracle_verdicts(oracle, groups):
    total = sum(len(idx) for idx, _ in groups.values())
    cols = ["tsg_rr_busy", "tsg_rr_suspend", "gcaps_busy", "gcaps_suspend", "gcaps_busy+prio", "gcaps_suspend+prio"]
    out = {c: np.zeros(total, np.uint8) for c in cols}
    from paper_2406_05221_amd import taskgen
    for idx, batch in groups.values():
        be = batch.get("best_effort")
        fields = {k: v for k, v in batch.items() if k != "best_effort"}
        for wait, name in ((BUSY, "busy"), (SUSPEND, "suspend")):
            if be is None:
                _, sched, _ = oracle.rta_batch(fields, BOTH, wait, threads=16)
                gcaps, rr, real_time = sched[0], sched[1], fields
            else:
                # best-effort tasks: in the round-robin taskset but untested; not in the GCAPS taskset
                resp, _, _ = oracle.rta_batch(fields, RR, wait, threads=16)
                rr = np.array([all(r >= 0 for r, b in zip(row, flags) if not b) for row, flags in zip(resp[0], be)])
                real_time = taskgen.without_tasks(fields, be != 0)
                gcaps = oracle.rta_batch(real_time, GCAPS, wait, threads=16)[1][0]
            out[f"gcaps_{name}"][idx] = gcaps
            out[f"tsg_rr_{name}"][idx] = rr
            out[f"gcaps_{name}+prio"][idx] = oracle.gprio_assign_batch(real_time, wait, skip=gcaps, threads=16)[2]
    return out


def test_every_analysis_on_table3_tasksets(oracle, gpu):
    from paper_2406_05221_amd import taskgen
    B, ctx, _ = gpu
    for overrides in ({}, dict(util=(0.3, 0.3), eps_us=200)):
        groups = taskgen.table3(4000, seed=3, **overrides)
        rescued = 0
        for n, (idx, batch) in groups.items():
            print(f"n={n} tasksets={len(idx)}", flush=True)
            for wait in (BUSY, SUSPEND):
                want_r, want_s, _ = oracle.rta_batch(batch, BOTH, wait, threads=16)
                got_r, got_s = B.gcaps_rta_batch(ctx, batch, BOTH, wait)
                assert np.array_equal(got_r, want_r) and np.array_equal(got_s, want_s)
                want = oracle.gprio_assign_batch(batch, wait, skip=want_s[0], threads=16)[:3]
                got = B.gcaps_gprio_assign_batch(ctx, batch, wait, got_s[0])
                assert all(np.array_equal(x, y) for x, y in zip(got, want))
                rescued += int((got[2].astype(bool) & ~got_s[0].astype(bool)).sum())
        assert rescued > 0


@pytest.mark.parametrize("overrides", [{}, dict(util=(0.3, 0.35), eps_us=200), dict(n_cpus=2, tasks_per_cpu=(1, 9), eta=(2, 4)),
                                       dict(n_cpus=8, tasks_per_cpu=(2, 3), gpu_ratio=(0.0, 1.0), period=(5_000, 9_000))])
def test_table3_tasksets_generated_on_the_device_are_the_hosts(gpu, overrides):
    """gcaps_table3_count_device / gcaps_table3_generate_device against the host generator: the same grouping by
    task count and the same batches, every field, bit for bit."""
    from paper_2406_05221_amd import taskgen
    B, ctx, _ = gpu
    N = 6_000
    host = taskgen.table3(N, seed=11, stream=301, first_index=77_000, **overrides)
    dev = B.gcaps_table3_device(ctx, N, seed=11, stream=301, first_index=77_000, **overrides)
    assert sorted(dev) == sorted(host)
    for n in host:
        idx, batch = host[n]
        d_idx, d_batch = dev[n]
        assert np.array_equal(d_idx.cpu().numpy(), idx)
        got = B.to_host(d_batch)
        for name in batch:
            assert np.array_equal(got[name], batch[name]), (n, name)


def test_table3_generation_rejects_a_wrong_task_count(gpu):
    import ctypes
    import torch
    from paper_2406_05221_amd import taskgen
    B, ctx, _ = gpu
    host = taskgen.table3(300, seed=1)
    by_size = sorted(host, key=lambda m: len(host[m][0]))
    n, other = by_size[-1], by_size[-2]  # the two most frequent task counts
    assert len(host[n][0]) >= 20 and len(host[other][0]) >= 5
    wrong = host[other][0][:5]  # tasksets of another count
    idx = torch.from_numpy(np.concatenate([host[n][0][:20], wrong]).astype(np.int32)).cuda()
    assert idx.numel() == 25
    q = taskgen.TABLE3
    spec = B.gcaps_table3_spec(seed=1, stream=300, first_index=0, n_cpus=q["n_cpus"], per_cpu_lo=q["tasks_per_cpu"][0],
                               per_cpu_hi=q["tasks_per_cpu"][1], gpu_ratio_lo=q["gpu_ratio"][0],
                               gpu_ratio_hi=q["gpu_ratio"][1], util_lo=q["util"][0], util_hi=q["util"][1],
                               period_lo=q["period"][0], period_hi=q["period"][1], eta_lo=q["eta"][0], eta_hi=q["eta"][1],
                               gc_lo=q["g_over_c"][0], gc_hi=q["g_over_c"][1], gm_lo=q["gm_over_g"][0],
                               gm_hi=q["gm_over_g"][1], theta_us=200, eps_us=1000, slice_us=1024)
    M, S = 25, 3
    kinds = {np.uint32: torch.int32, np.int32: torch.int32, np.uint8: torch.uint8}
    shapes = {1: (M,), 2: (M, n), 3: (M, n, S)}
    batch = {name: torch.zeros(shapes[ndim], dtype=kinds[dtype], device="cuda:0") for name, dtype, ndim in B._FIELDS}
    b = B.gcaps_batch(n_tasksets=M, n_tasks=n, max_gseg=S)
    for name, _, _ in B._FIELDS:
        setattr(b, name, batch[name].data_ptr())
    torch.cuda.synchronize()
    assert B._lib.gcaps_table3_generate_device(ctx, ctypes.byref(spec), idx.data_ptr(), ctypes.byref(b)) == B.GCAPS_OK
    with pytest.raises(B.GcapsError) as e:
        B.gcaps_status(ctx)
    assert e.value.code == B.GCAPS_ETASK and e.value.first_bad == 20
    got = B.to_host(batch)
    assert (got["period_us"][20:] == 0).all() and (got["period_us"][:20] > 0).all()
    spec.n_cpus = 9
    assert B._lib.gcaps_table3_generate_device(ctx, ctypes.byref(spec), idx.data_ptr(), ctypes.byref(b)) == B.GCAPS_EINVAL


def test_sweep_matches_the_oracle(oracle, gpu):
    from paper_2406_05221_amd import sweep, taskgen
    B, ctx, _ = gpu
    rows = sweep.sweep(ctx, "util", [0.2, 0.4], 600, seed=5)
    assert rows == sweep.sweep(ctx, "util", [0.2, 0.4], 600, seed=5, host_inputs=True)
    for k, (value, shares) in enumerate(rows):
        groups = taskgen.table3(600, seed=5, stream=300 + k, util=(value, value))
        want = oracle_verdicts(oracle, groups)
        for c in sweep.COLUMNS:
            assert shares[c] == float(want[c].mean()), (value, c)
    # lighter CPUs: more tasksets pass; the priority search never loses a taskset
    for c in sweep.COLUMNS:
        assert rows[0][1][c] >= rows[1][1][c]
    for _, shares in rows:
        assert shares["gcaps_busy+prio"] >= shares["gcaps_busy"]
        assert shares["gcaps_suspend+prio"] >= shares["gcaps_suspend"]


def test_sweep_with_best_effort_tasks_matches_the_oracle(oracle, gpu):
    from paper_2406_05221_amd import sweep, taskgen
    B, ctx, _ = gpu
    rows = sweep.sweep(ctx, "be_ratio", [0.0, 0.3], 600, seed=6, util=(0.45, 0.45))
    for k, (value, shares) in enumerate(rows):
        groups = taskgen.table3(600, seed=6, stream=300 + k, be_ratio=value, util=(0.45, 0.45))
        want = oracle_verdicts(oracle, groups)
        for c in sweep.COLUMNS:
            assert shares[c] == float(want[c].mean()), (value, c)
    # turning tasks into best-effort ones helps GCAPS (they no longer preempt anyone) more than round-robin
    # (their GPU segments still take their time slices)
    gain = {c: rows[1][1][c] - rows[0][1][c] for c in sweep.COLUMNS}
    assert gain["gcaps_suspend"] > 0 and gain["gcaps_busy"] > 0
