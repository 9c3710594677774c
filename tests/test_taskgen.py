"""The synthetic generator: determinism, shapes and the structure the workloads promise."""
import numpy as np
import pytest

from paper_2406_05221_amd import taskgen


@pytest.mark.parametrize("k,N", [(1, 1000), (2, 9000), (3, 5000), (4, 500), (5, 2160)])
def test_workload_structure(k, N):
    b = taskgen.config(k, N)
    cores, per_core, S = taskgen.CONFIG_SHAPES[k]
    n = cores * per_core
    assert b["cpu_us"].shape == (N, n) and b["gm_us"].shape == (N, n, S)
    assert (b["deadline_us"] == b["period_us"]).all()
    assert (b["n_gseg"] >= 1).all() and (b["n_gseg"] <= S).all()
    # unused slots are zero; used slots split a segment into launch/copy and kernel halves
    used = np.arange(S)[None, None, :] < b["n_gseg"][:, :, None]
    assert (b["gm_us"][~used] == 0).all() and (b["ge_us"][~used] == 0).all()
    assert ((b["ge_us"] - b["gm_us"])[used] <= 1).all() and (b["ge_us"][used] >= 1).all()
    # rate-monotonic, unique ranks 1..n
    assert (np.sort(b["prio"], axis=1) == np.arange(1, n + 1)).all()
    order = np.argsort(-b["prio"], axis=1)
    assert (np.diff(np.take_along_axis(b["period_us"], order, 1).astype(np.int64), axis=1) >= 0).all()
    # tasks_per_core tasks on each core
    assert (b["core"] == np.repeat(np.arange(cores), per_core)[None, :]).all()
    assert (b["theta_us"] == b["eps_us"]).all()


def test_utilisation_per_core_matches_request():
    b = taskgen.config(1)
    w = b["cpu_us"].astype(np.float64) + b["gm_us"].sum(2) + b["ge_us"].sum(2)
    u = (w / b["period_us"]).reshape(1000, 2, 3).sum(2)
    assert abs(u.mean() - 0.4) < 0.005 and u.max() < 0.42
    b = taskgen.config(2)
    w = b["cpu_us"].astype(np.float64) + b["gm_us"].sum(2) + b["ge_us"].sum(2)
    u = (w / b["period_us"]).reshape(9, 1000, 4, 4).sum(3).mean((1, 2))
    assert np.allclose(u, 0.1 * np.arange(1, 10), atol=0.01)


def test_any_taskset_can_be_regenerated_alone():
    full = taskgen.config(3, 3000, threads=3)
    part = taskgen.config(3, 100, first_index=1234, threads=1)
    for key in full:
        assert (full[key][1234:1334] == part[key]).all(), key
    five = taskgen.config(5, 400)
    tail = taskgen.config(5, 100, first_index=300)
    for key in five:
        assert (five[key][300:] == tail[key]).all(), key
    # grid cell of workload 5 follows the taskset index
    assert set(np.unique(five["slice_us"])) == {512, 1024, 2048}
    assert set(np.unique(five["theta_us"])) == {50, 200, 500}


def test_seed_changes_the_draw():
    a, b = taskgen.config(1, 50, seed=0), taskgen.config(1, 50, seed=1)
    assert (a["period_us"] != b["period_us"]).any()


def test_table3_recipe_structure():
    """Sec. 6.1 / Table 3: ranges, rate-monotonic priorities, worst-fit-decreasing allocation."""
    groups = taskgen.table3(3000, seed=1)
    assert sum(len(idx) for idx, _ in groups.values()) == 3000
    assert min(groups) >= 12 and max(groups) <= 24 and len(groups) >= 10
    seen = np.zeros(3000, bool)
    for n, (idx, b) in groups.items():
        assert not seen[idx].any()
        seen[idx] = True
        N = len(idx)
        assert b["cpu_us"].shape == (N, n) and b["gm_us"].shape == (N, n, 3)
        assert (b["theta_us"] == 200).all() and (b["eps_us"] == 1000).all() and (b["slice_us"] == 1024).all()
        assert (b["period_us"] >= 30_000).all() and (b["period_us"] <= 500_000).all()
        assert (b["deadline_us"] == b["period_us"]).all() and (b["core"] < 4).all()
        gpu = b["n_gseg"] > 0
        share = gpu.mean(axis=1)
        assert (share >= 0.4 - 0.5 / n - 1e-9).all() and (share <= 0.6 + 0.5 / n + 1e-9).all()
        assert (b["n_gseg"][gpu] >= 1).all() and (b["n_gseg"][gpu] <= 3).all()
        used = np.arange(3)[None, None, :] < b["n_gseg"][:, :, None]
        assert (b["gm_us"][~used] == 0).all() and (b["ge_us"][~used] == 0).all() and (b["ge_us"][used] >= 1).all()
        Gm, Ge = b["gm_us"].sum(axis=2).astype(float), b["ge_us"].sum(axis=2).astype(float)
        G, C = Gm + Ge, b["cpu_us"].astype(float)
        big = gpu & (G + C > 2000)  # rounding to whole microseconds matters for tiny tasks only
        assert (G[big] / C[big] > 0.19).all() and (G[big] / C[big] < 2.05).all()
        assert (Gm[big] / G[big] > 0.09).all() and (Gm[big] / G[big] < 0.31).all()
        assert (np.sort(b["prio"], axis=1) == np.arange(1, n + 1)).all()
        order = np.argsort(-b["prio"], axis=1)
        assert (np.diff(np.take_along_axis(b["period_us"], order, 1).astype(np.int64), axis=1) >= 0).all()
        # total utilisation: 4 CPUs x [0.4, 0.6]; worst-fit decreasing leaves the CPUs balanced: no CPU
        # exceeds the lightest one by more than the largest task placed after it, i.e. by more than its own
        # smallest task would explain; the cheap check: max - min load <= largest task utilisation
        u = (C + G) / b["period_us"]
        assert (u.sum(axis=1) > 1.55).all() and (u.sum(axis=1) < 2.45).all()
        load = np.stack([(u * (b["core"] == c)).sum(axis=1) for c in range(4)], axis=1)
        assert (load.max(axis=1) - load.min(axis=1) <= u.max(axis=1) + 1e-3).all()
    assert seen.all()
    again = taskgen.table3(3000, seed=1, threads=3)
    assert all((again[n][1]["cpu_us"] == groups[n][1]["cpu_us"]).all() for n in groups)
    one = taskgen.table3(50, seed=1, util=(0.5, 0.5), tasks_per_cpu=(4, 4))
    assert list(one) == [16]


def test_table3_best_effort_tasks():
    groups = taskgen.table3(800, seed=2, be_ratio=0.25)
    for n, (idx, b) in groups.items():
        be = b["best_effort"] != 0
        assert (be.sum(axis=1) == int(np.floor(0.25 * n + 0.5))).all()
        # below every real-time task, order among themselves and among the real-time tasks kept
        assert (np.where(be, b["prio"], -10**9).max(axis=1) < np.where(~be, b["prio"], 10**9).min(axis=1)).all()
        plain = taskgen.table3(800, seed=2)[n][1]
        assert (np.where(be, b["prio"] + n, b["prio"]) == plain["prio"]).all()
        assert all((b[k] == plain[k]).all() for k in plain if k != "prio")
        rt = taskgen.without_tasks({k: v for k, v in b.items() if k != "best_effort"}, be)
        m = n - int(be[0].sum())
        assert rt["cpu_us"].shape == (len(idx), m) and rt["ge_us"].shape == (len(idx), m, 3)
        last = len(idx) - 1
        assert (rt["cpu_us"][0] == b["cpu_us"][0][~be[0]]).all() and (rt["gm_us"][last] == b["gm_us"][last][~be[last]]).all()
        assert (rt["eps_us"] == b["eps_us"]).all()


def test_cpu_only_tasks_keep_their_whole_demand():
    """eta = 0 is drawn for some tasks: nothing of their demand is set aside for GPU segments that are not there,
    so the demand per core is the utilisation that was asked for (up to the rounding to whole microseconds)."""
    from paper_2406_05221_amd import taskgen
    b = taskgen.generate(4000, n_cores=3, tasks_per_core=4, max_gseg=2, util=(0.6, 0.6), eta=(0, 2), share=(0.5, 0.5),
                         period=(50_000, 500_000), overhead=(0, 0), slice_us=1024, seed=9, stream=9)
    demand = b["cpu_us"].astype(np.float64) + b["gm_us"].sum(2) + b["ge_us"].sum(2)
    per_core = (demand / b["period_us"]).reshape(4000, 3, 4).sum(axis=2)
    assert np.abs(per_core - 0.6).max() < 1e-3
    cpu_only = b["n_gseg"] == 0
    assert cpu_only.mean() > 0.2 and (b["gm_us"].sum(2)[cpu_only] == 0).all() and (b["ge_us"].sum(2)[cpu_only] == 0).all()


def test_periods_are_log_uniform_and_splits_sum_to_the_core_utilisation():
    """The generator's own logarithm and power routines (no math library: the device generator must match bit for
    bit) are checked through what they produce: log2 of the periods is uniform over the range, and the
    UUniFast shares of a core have the known mean U / m each."""
    from paper_2406_05221_amd import taskgen
    b = taskgen.generate(20_000, n_cores=2, tasks_per_core=5, max_gseg=1, util=(0.5, 0.5), eta=(1, 1), share=(0.1, 0.1),
                         period=(1_000, 1_000_000), overhead=(0, 0), slice_us=1024, seed=1, stream=2)
    x = np.log2(b["period_us"].astype(np.float64)).ravel()
    lo, hi = np.log2(1_000), np.log2(1_000_000)
    hist, _ = np.histogram(x, bins=20, range=(lo, hi))
    assert np.abs(hist / x.size - 0.05).max() < 0.004
    assert b["period_us"].min() >= 1_000 and b["period_us"].max() <= 1_000_000
    u = (b["cpu_us"].astype(np.float64) + b["gm_us"].sum(2) + b["ge_us"].sum(2)) / b["period_us"]
    assert np.abs(u.reshape(-1, 2, 5).mean(axis=0) - 0.1).max() < 0.003
    # the first share of a core is U (1 - r^(1/4)) with r uniform: mean 0.1, second moment 2 U^2 / 30
    first = u.reshape(-1, 2, 5)[:, :, 0].ravel()
    assert abs((first ** 2).mean() - 2 * 0.25 / 30) < 6e-4


def test_tasks_clear_of_delayed_updates_by_hand():
    """The study module's mask of tasks that no delayed closing update can reach: task k is clear when every
    GPU-using task of higher priority is the highest-priority task of its core."""
    from paper_2406_05221_amd import pessimism
    # priorities 6..1; cores 0,1,0,1,0,1; GPU segments: tasks 0 (leads core 0), 2 (second on core 0), 5 (last on core 1)
    fields = dict(prio=np.array([[6, 5, 4, 3, 2, 1]], np.int32), core=np.array([[0, 1, 0, 1, 0, 1]], np.uint8),
                  n_gseg=np.array([[1, 0, 2, 0, 0, 1]], np.uint8))
    # tasks 0..2 have only task 0 as a GPU-using task above them; below task 2 its update can wait for task 0's CPU work
    assert pessimism.clear_of_delayed_updates(fields).tolist() == [[True, True, True, False, False, False]]
    # the order of the columns does not matter, only the priorities
    perm = [3, 5, 0, 2, 4, 1]
    shuffled = {k: v[:, perm] for k, v in fields.items()}
    assert pessimism.clear_of_delayed_updates(shuffled).tolist() == [[False, False, True, True, False, True]]


def test_tasks_clear_of_delayed_updates_against_the_loop_form():
    from paper_2406_05221_amd import pessimism
    from test_oracle_sim import tasks_no_delayed_update_reaches
    b = taskgen.generate(200, n_cores=3, tasks_per_core=3, max_gseg=2, util=(0.2, 0.5), eta=(0, 2), share=(0.1, 0.5),
                         period=(40, 400), overhead=(1, 3), slice_us=8, seed=4, stream=5)
    mask = pessimism.clear_of_delayed_updates(b)
    assert (mask == tasks_no_delayed_update_reaches(b)).all() and 0.2 < mask.mean() < 0.9
