"""Pins of the oracle's GPU-segment priority assignment (Sec. 4.3) and of the analysis it uses
(Sec. 5.4): the verdicts the paper prints for the taskset of Table 2, bounds worked by hand,
agreement with the analysis of Sec. 5.3 where Sec. 5.4 changes nothing, an exhaustive search
over all admissible priority orders, and a unit-tick simulation run with the assigned priorities."""
import itertools

import numpy as np
import pytest

import des_harness as des
from helpers import load_table2, oracle_bound, seg_arrays
from test_oracle_des import random_tiny_taskset

GCAPS, BUSY, SUSPEND = 1, 0, 1


def _args(tasks):
    gm, ge, eta = seg_arrays(tasks)
    C = [t["C"] if "C" in t else sum(t["c"]) for t in tasks]
    return (C, [t["T"] for t in tasks], [t["D"] for t in tasks], [t["prio"] for t in tasks],
            [t["core"] for t in tasks], eta, gm, ge)


def bound_with(o, tasks, gprio, wait, eps, options=0):
    return o.gprio_rta_taskset(*_args(tasks), gprio, eps_us=eps, wait_mode=wait, options=options)


def assign(o, tasks, wait, eps, options=0):
    return o.gprio_assign_taskset(*_args(tasks), eps_us=eps, wait_mode=wait, options=options)


# ---- the paper's example ----------------------------------------------------------------------
def test_table2_printed_verdicts(oracle):
    g, tasks = load_table2()
    v = g["printed_verdict_separate_gpu_priority"]
    assert v["wait_mode"] == "suspend" and v["schedulable"] is True
    names = [t["name"] for t in g["tasks"]]
    order = v["gpu_priority_order"]
    swapped = [len(order) - order.index(nm) for nm in names]  # larger = higher
    assert swapped == [4, 3, 1, 2]
    for eps in (0, 1):
        _, sched, _ = bound_with(oracle, tasks, swapped, SUSPEND, eps)
        assert sched == 1
        # GPU priority = CPU priority: fails here as well (D_h >= R_h in the jitters)
        _, sched, _ = bound_with(oracle, tasks, [t["prio"] for t in tasks], SUSPEND, eps)
        assert sched == 0
        # and the search of Sec. 4.3 arrives at the order of Fig. 4(b)
        gp, _, sched, _ = assign(oracle, tasks, SUSPEND, eps)
        assert sched == 1 and list(gp) == swapped


def test_table2_hand_worked_values(oracle):
    """eps = 0, jitters with D_h: J^c_1 = 80-13 = 67, J^g_1 = 80-6 = 74, J^g_3 = 190-80 = 110,
    J^g_4 = 200-10 = 190.
    GPU order tau1 > tau2 > tau4 > tau3, self-suspension:
      tau1 = 9+10 = 19;  tau2 = 40 + ceil((R+67)/80)*13: 40 -> 66 -> 66;
      tau3 (alone on its core; tau1, tau4 above it on the GPU):
        119 + ceil((R+74)/80)*6 + ceil((R+190)/200)*10: 119 -> 157 -> 157;
      tau4 (tau3 now below it): 30 + ceil(R/150)*40 + ceil((R+67)/80)*13 + ceil((R+74)/80)*6:
        30 -> 108 -> 127 -> 127.
    Same order, busy-waiting: tau2 = 40 + ceil(R/80)*(13+6) = 59; tau3 = 157;
      tau4 = 30 + ceil(R/150)*40 + ceil(R/80)*19: 30 -> 89 -> 108 -> 108.
    GPU order = CPU order, self-suspension: tau3 = 119 + ceil((R+74)/80)*6: 119 -> 137 -> 137;
      tau4 = 30 + ceil(R/150)*40 + ceil((R+67)/80)*13 + ceil((R+74)/80)*6 + ceil((R+110)/190)*80:
        30 -> 188 -> 346 > 200: miss."""
    _, tasks = load_table2()
    resp, sched, _ = bound_with(oracle, tasks, [4, 3, 1, 2], SUSPEND, 0)
    assert list(resp) == [19, 66, 157, 127] and sched == 1
    resp, sched, _ = bound_with(oracle, tasks, [4, 3, 1, 2], BUSY, 0)
    assert list(resp) == [19, 59, 157, 108] and sched == 1
    resp, sched, _ = bound_with(oracle, tasks, [4, 3, 2, 1], SUSPEND, 0)
    assert list(resp) == [19, 66, 137, -1] and sched == 0
    for wait, want in ((SUSPEND, [19, 66, 157, 127]), (BUSY, [19, 59, 157, 108])):
        gp, resp, sched, _ = assign(oracle, tasks, wait, 0)
        assert list(gp) == [4, 3, 1, 2] and list(resp) == want and sched == 1


def test_runlist_update_cost_hand_worked(oracle):
    """Two GPU-using tasks on different cores, eps = 3, busy-waiting.  tau_b below tau_a:
    base_b = 5+(2+20) + 2*3*1 + (1+1)*3 = 39;  G^{e*}_a = 10 + 2*3*2 = 22;  J^g_a = 100 - 10 = 90:
    39 + ceil((R+90)/100)*22: 39 -> 83 -> 83.  tau_b above tau_a: tau_b = 39 and, with
    base_a = 4+(2+10) + 2*3*2 + (2+1)*3 = 37, G^{e*}_b = 26, J^g_b = 180:
    tau_a = 37 + ceil((R+180)/200)*26: 37 -> 89 -> 89."""
    a = dict(C=4, T=100, D=100, prio=2, core=0, gm=[1, 1], ge=[6, 4])
    b = dict(C=5, T=200, D=200, prio=1, core=1, gm=[2], ge=[20])
    resp, _, _ = bound_with(oracle, [a, b], [2, 1], BUSY, 3)
    assert list(resp) == [37, 83]
    resp, _, _ = bound_with(oracle, [a, b], [1, 2], BUSY, 3)
    assert list(resp) == [89, 39]


def test_same_core_self_suspension_with_update_cost_hand_worked(oracle):
    """Two GPU-using tasks on one core, eps = 2, self-suspension.  tau_a = 3+6 + 2*2 + 2*2 = 17.
    tau_b: base = 28+8 + 4 + 4 = 44; Lemma 15: ceil((R+J^c_a)/40)*(C_a + G^{m*}_a) with
    J^c_a = 40-4 = 36 and cost 3+1+4 = 8; Lemma 13, same core: ceil((R+J^g_a)/40)*G^e_a with
    J^g_a = 40-5 = 35 and cost 5 (no update cost in this sum): 44 -> 70 -> 83 -> 83
    (83+36 = 119 and 83+35 = 118 stay just inside three periods of tau_a)."""
    a = dict(C=3, T=40, D=40, prio=2, core=0, gm=[1], ge=[5])
    b = dict(C=28, T=100, D=100, prio=1, core=0, gm=[2], ge=[6])
    resp, sched, _ = bound_with(oracle, [a, b], [2, 1], SUSPEND, 2)
    assert list(resp) == [17, 83] and sched == 1
    # a CPU-only tau_b sees the CPU part only (Lemma 13 applies to GPU-using tasks)
    b2 = dict(C=12, T=100, D=100, prio=1, core=0, gm=[], ge=[])
    resp, _, _ = bound_with(oracle, [a, b2], [2, 1], SUSPEND, 2)
    assert list(resp) == [17, 12 + 2 + 2 * 8]  # 14 -> ceil(50/40)*8 = 16 -> 30 -> 30


def test_carry_in_jitter_is_deadline_minus_gpu_time(oracle):
    """Busy-waiting, eps = 0, two cores.  tau_b (T = D = 200, G^e = 20) above tau_a on the GPU:
    J^g_b = 200-20 = 180.  tau_a: 170 + ceil((R+180)/200)*20: 170 -> 210 -> 210, because
    210+180 = 390 is still inside two periods (a jitter of D_b alone would reach a third)."""
    a = dict(C=165, T=1000, D=1000, prio=2, core=0, gm=[0], ge=[5])
    b = dict(C=10, T=200, D=200, prio=1, core=1, gm=[0], ge=[20])
    resp, _, _ = bound_with(oracle, [a, b], [1, 2], BUSY, 0)
    assert list(resp) == [210, 30]
    a["ge"], a["gm"], a["C"] = [], [], 170  # Lemma 11: the same for a CPU-only tau_a
    resp, _, _ = bound_with(oracle, [a, b], [1, 2], BUSY, 0)
    assert list(resp) == [210, 30]
    resp, _, _ = bound_with(oracle, [a, b], [1, 2], SUSPEND, 0)  # Lemma 14: nothing under self-suspension
    assert list(resp) == [170, 30]


# ---- relations with the analysis of Sec. 5.3 -----------------------------------------------------
def random_taskset(rng, n, n_cores, scale=1):
    tasks = random_tiny_taskset(rng, n, n_cores, max_eta=2, t_lo=30 * scale, t_hi=90 * scale)
    for t in tasks:
        t["C"] = sum(t["c"])
    return tasks


def test_single_core_busy_waiting_equals_sec_5_3(oracle):
    """One core, busy-waiting: no sum of Lemmas 10-12 carries a jitter and no task of another core
    exists, so Sec. 5.4 changes nothing up to the first miss."""
    rng = np.random.default_rng(5)
    seen = 0
    for _ in range(200):
        tasks = random_taskset(rng, int(rng.integers(2, 7)), 1)
        eps = int(rng.integers(0, 3))
        ref, _, _ = oracle_bound(oracle, tasks, GCAPS, BUSY, 0, eps, 1)
        got, _, _ = bound_with(oracle, tasks, [t["prio"] for t in tasks], BUSY, eps)
        for r, g in zip(ref, got):
            if r == -2:
                break
            assert r == g
            seen += 1
    assert seen > 300


@pytest.mark.parametrize("wait", [BUSY, SUSPEND])
def test_bounds_with_deadline_jitters_dominate_sec_5_3(oracle, wait):
    """GPU priority = CPU priority: the only difference is D_h >= R_h inside the jitters, so no
    bound may be smaller than that of Sec. 5.3, and a taskset that passes here passes there."""
    rng = np.random.default_rng(11 + wait)
    strictly = 0
    for _ in range(300):
        tasks = random_taskset(rng, int(rng.integers(2, 7)), int(rng.integers(1, 4)))
        eps = int(rng.integers(0, 3))
        ref, ref_sched, _ = oracle_bound(oracle, tasks, GCAPS, wait, 0, eps, 1)
        got, got_sched, _ = bound_with(oracle, tasks, [t["prio"] for t in tasks], wait, eps)
        assert not (got_sched and not ref_sched)
        for r, g in zip(ref, got):
            if r < 0:
                break
            assert g == -1 or g >= r
            strictly += g > r
    assert strictly > 50


def test_moving_a_task_up_never_hurts_it(oracle):
    """What Audsley's scheme relies on: the bound of a task depends on the set of tasks above it
    on the GPU only, and shrinking that set cannot raise it."""
    rng = np.random.default_rng(3)
    for _ in range(150):
        n = int(rng.integers(3, 7))
        tasks = random_taskset(rng, n, n)  # one task per core at most is not forced: cores drawn at random
        for k, t in enumerate(tasks):
            t["core"] = k  # all on different cores: every GPU order is admissible
        wait = int(rng.integers(0, 2))
        order = list(rng.permutation(n))
        gp = [0] * n
        for lvl, i in enumerate(order):
            gp[i] = lvl + 1
        base, _, _ = bound_with(oracle, tasks, gp, wait, 1)
        i, j = order[0], order[-1]  # lowest and highest
        # reorder the tasks above the lowest one: its bound stays
        gp2 = list(gp)
        a, b = order[1], order[2]
        gp2[a], gp2[b] = gp2[b], gp2[a]
        again, _, _ = bound_with(oracle, tasks, gp2, wait, 1)
        assert again[i] == base[i]
        # lift the lowest task to the top: its own bound cannot grow
        gp3 = [g - 1 if g > 1 else n for g in gp]
        lifted, _, _ = bound_with(oracle, tasks, gp3, wait, 1)
        assert base[i] == -1 or (0 <= lifted[i] <= base[i])
        assert j != i


def test_orders_that_disagree_on_a_core_are_rejected(oracle):
    a = dict(C=2, T=50, D=50, prio=2, core=0, gm=[1], ge=[3])
    b = dict(C=2, T=60, D=60, prio=1, core=0, gm=[1], ge=[3])
    with pytest.raises(oracle.OracleError) as e:
        bound_with(oracle, [a, b], [1, 2], SUSPEND, 0)
    assert e.value.code == oracle.EORDER
    b["core"] = 1
    bound_with(oracle, [a, b], [1, 2], SUSPEND, 0)


# ---- the search ------------------------------------------------------------------------------
def admissible_orders(tasks):
    """Every GPU priority order (as levels, larger = higher) that agrees with the CPU priority
    order among the tasks of each core."""
    n = len(tasks)
    by_prio = sorted(range(n), key=lambda i: -tasks[i]["prio"])
    for perm in itertools.permutations(range(n)):  # perm[0] = highest GPU priority
        pos = {i: k for k, i in enumerate(perm)}
        ok = all(pos[a] < pos[b] for x, a in enumerate(by_prio) for b in by_prio[x + 1:]
                 if tasks[a]["core"] == tasks[b]["core"])
        if ok:
            yield [n - pos[i] for i in range(n)]


@pytest.mark.parametrize("wait", [BUSY, SUSPEND])
def test_search_finds_an_order_iff_one_exists(oracle, wait):
    rng = np.random.default_rng(17 + wait)
    found = rescued = hopeless = 0
    for trial in range(500):
        n = int(rng.integers(3, 6))
        tasks = random_taskset(rng, n, int(rng.integers(2, 4)), scale=1)
        for t in tasks:  # heavier GPU parts: orders matter
            t["ge"] = [g * 3 for g in t["ge"]]
        eps = int(rng.integers(0, 2))
        gp, resp, sched, _ = assign(oracle, tasks, wait, eps)
        passing = []
        for levels in admissible_orders(tasks):
            r, s, _ = bound_with(oracle, tasks, levels, wait, eps)
            if s:
                passing.append((levels, list(r)))
        assert bool(sched) == bool(passing), (tasks, eps, gp, passing[:1])
        if sched:
            found += 1
            assert sorted(gp) == list(range(1, n + 1))
            assert (list(gp), list(resp)) in passing
            _, default_ok, _ = bound_with(oracle, tasks, [t["prio"] for t in tasks], wait, eps)
            rescued += not default_ok
        else:
            hopeless += 1
            assert list(gp) == [0] * n and list(resp) == [-2] * n
    assert found > 40 and hopeless > 40 and rescued > 5, (found, hopeless, rescued)


def test_search_prefers_the_lowest_cpu_priority_candidate(oracle):
    """Two independent tasks on two cores, both able to take the lowest level: the one with the
    lower CPU priority gets it (candidates are tried from the lowest CPU priority upwards)."""
    a = dict(C=2, T=100, D=100, prio=2, core=0, gm=[1], ge=[3])
    b = dict(C=2, T=100, D=100, prio=1, core=1, gm=[1], ge=[3])
    gp, _, sched, _ = assign(oracle, [a, b], SUSPEND, 0)
    assert sched == 1 and list(gp) == [2, 1]


def test_own_demand_beyond_deadline_fails_the_search(oracle):
    a = dict(C=2, T=100, D=100, prio=2, core=0, gm=[1], ge=[3])
    b = dict(C=50, T=60, D=60, prio=1, core=1, gm=[1], ge=[10])  # 61 > 60
    gp, resp, sched, _ = assign(oracle, [a, b], BUSY, 0)
    assert sched == 0 and list(gp) == [0, 0] and list(resp) == [-2, -2]


def test_batch_matches_single_calls_and_honours_skip(oracle):
    from paper_2406_05221_amd import taskgen
    batch = taskgen.config(2, 300)
    for wait in (BUSY, SUSPEND):
        skip = (np.arange(300) % 3 == 0).astype(np.uint8)
        gp, resp, sched, terms = oracle.gprio_assign_batch(batch, wait, skip=skip, threads=3)
        assert terms > 0
        for s in range(300):
            if skip[s]:
                assert sched[s] == 1 and (gp[s] == 0).all() and (resp[s] == -2).all()
                continue
            g1, r1, s1, _ = oracle.gprio_assign_taskset(
                batch["cpu_us"][s], batch["period_us"][s], batch["deadline_us"][s], batch["prio"][s],
                batch["core"][s], batch["n_gseg"][s], batch["gm_us"][s], batch["ge_us"][s],
                eps_us=batch["eps_us"][s], wait_mode=wait)
            assert (g1 == gp[s]).all() and (r1 == resp[s]).all() and s1 == sched[s]


def admissible_levels(rng, prio, core):
    """GPU priority levels 1..n drawn at random among those that keep, on every core, the order of
    the CPU priorities (Sec. 4.3): the levels that fall on a core are dealt to its tasks by CPU priority."""
    n = len(prio)
    levels = rng.permutation(n) + 1
    out = np.zeros(n, np.int32)
    for c in set(core.tolist()):
        on = [i for i in range(n) if core[i] == c]
        by_cpu = sorted(on, key=lambda i: (-int(prio[i]), i))
        for i, lv in zip(by_cpu, sorted((int(levels[j]) for j in on), reverse=True)):
            out[i] = lv
    return out


def test_given_priorities_batch_matches_single_calls(oracle):
    """oracle_gprio_rta_batch is the per-taskset analysis of Sec. 5.4 applied to every taskset of a batch:
    its indexing of the per-task, per-segment and priority arrays, its outputs and its error reporting are
    checked against single calls on the slices."""
    from paper_2406_05221_amd import taskgen
    rng = np.random.default_rng(11)
    N = 48
    batch = taskgen.generate(N, n_cores=3, tasks_per_core=3, max_gseg=3, util=(0.1, 0.5), eta=(0, 3),
                             share=(0.1, 0.5), period=(5_000, 200_000), overhead=(0, 300), slice_us=1024,
                             seed=5, stream=41)
    gprio = np.stack([admissible_levels(rng, batch["prio"][s], batch["core"][s]) for s in range(N)])
    assert (gprio != batch["prio"]).any(axis=1).sum() > N // 2  # orders that differ from the CPU order
    for wait in (BUSY, SUSPEND):
        resp, sched = oracle.gprio_rta_batch(batch, gprio, wait)
        assert resp.shape == (N, 9) and sched.shape == (N,)
        assert 0 < sched.sum() < N  # both verdicts occur
        for s in range(N):
            r1, s1, _ = oracle.gprio_rta_taskset(
                batch["cpu_us"][s], batch["period_us"][s], batch["deadline_us"][s], batch["prio"][s],
                batch["core"][s], batch["n_gseg"][s], batch["gm_us"][s], batch["ge_us"][s], gprio[s],
                eps_us=batch["eps_us"][s], wait_mode=wait)
            assert (r1 == resp[s]).all() and s1 == sched[s], s


def test_given_priorities_batch_reports_the_first_bad_taskset(oracle):
    from paper_2406_05221_amd import taskgen
    rng = np.random.default_rng(12)
    N = 40
    batch = taskgen.generate(N, n_cores=2, tasks_per_core=3, max_gseg=2, util=(0.1, 0.4), eta=(1, 2),
                             share=(0.1, 0.5), period=(5_000, 200_000), overhead=(0, 100), slice_us=1024,
                             seed=6, stream=42)
    gprio = np.stack([admissible_levels(rng, batch["prio"][s], batch["core"][s]) for s in range(N)])
    oracle.gprio_rta_batch(batch, gprio, SUSPEND)
    # a period of zero: task-model violation, smallest index reported
    bad = {k: v.copy() for k, v in batch.items()}
    bad["period_us"][29, 4] = 0
    bad["period_us"][17, 1] = 0
    with pytest.raises(oracle.OracleError) as e:
        oracle.gprio_rta_batch(bad, gprio, SUSPEND)
    assert e.value.code == oracle.ETASK and e.value.first_bad == 17
    # two tasks of one core in the opposite order on the GPU (Sec. 4.3 forbids it)
    g2 = gprio.copy()
    for s in (33, 21):
        on0 = [i for i in range(6) if batch["core"][s, i] == 0]
        a, b = on0[0], on0[1]
        g2[s, a], g2[s, b] = g2[s, b], g2[s, a]
    with pytest.raises(oracle.OracleError) as e:
        oracle.gprio_rta_batch(batch, g2, BUSY)
    assert e.value.code == oracle.EORDER and e.value.first_bad == 21
    # the violation with the smaller index wins, whatever its kind
    with pytest.raises(oracle.OracleError) as e:
        oracle.gprio_rta_batch(bad, g2, BUSY)
    assert e.value.code == oracle.ETASK and e.value.first_bad == 17


# ---- concrete schedules under separate GPU priorities -------------------------------------------
@pytest.mark.parametrize("wait", [BUSY, SUSPEND])
def test_simulated_response_never_exceeds_bound_under_separate_priorities(oracle, wait):
    """The simulator takes its runlist decisions by GPU priority and everything else by CPU
    priority.  Orders tried per taskset: the one the search assigns, and admissible orders drawn
    at random; whenever Sec. 5.4 calls the taskset schedulable no job may exceed its bound."""
    rng = np.random.default_rng(23 + wait)
    checked = reordered = 0
    for trial in range(400):
        n = int(rng.integers(2, 6))
        tasks = random_tiny_taskset(rng, n, n_cores=int(rng.integers(2, 4)), max_eta=2, rm=bool(trial % 2))
        for t in tasks:
            t["ge"] = [g * 2 for g in t["ge"]]
        eps = int(rng.integers(0, 3))
        orders = []
        gp, R, sched, _ = assign(oracle, tasks, wait, eps)
        if sched:
            orders.append((list(gp), R))
        every = list(admissible_orders(tasks))
        for k in rng.permutation(len(every))[:3]:
            R2, s2, _ = bound_with(oracle, tasks, every[k], wait, eps)
            if s2:
                orders.append((every[k], R2))
        cpu_order = sorted(range(n), key=lambda i: tasks[i]["prio"])
        offs = [[0] * n] + [[int(x) for x in rng.integers(0, 25, n)] for _ in range(16)]
        for levels, bound in orders:
            checked += 1
            reordered += sorted(range(n), key=lambda i: levels[i]) != cpu_order
            for o in offs:
                rc, mr, _ = des.run(tasks, policy=GCAPS, wait_mode=wait, theta=0, eps=eps, L=1, offsets=o,
                                    horizon=500, gprio=levels)
                assert rc == 0 and (mr <= bound).all(), (tasks, eps, levels, o, mr, bound)
    assert checked > 200 and reordered > 60, (checked, reordered)
