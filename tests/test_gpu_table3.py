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


def test_sweep_matches_the_oracle(oracle, gpu):
    from paper_2406_05221_amd import sweep, taskgen
    B, ctx, _ = gpu
    rows = sweep.sweep(ctx, "util", [0.2, 0.4], 600, seed=5)
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
