"""Structural properties of the bounds, the exhaustive least-fixed-point search, output
conventions and argument checking of the CPU oracle."""
import numpy as np
import pytest

from helpers import VARIANTS, oracle_bound
from rta_spec import Spec

GCAPS, RR, BUSY, SUSPEND = 1, 2, 0, 1


def random_taskset(rng, n, n_cores, max_eta, t_lo, t_hi, util):
    T = sorted(int(x) for x in rng.integers(t_lo, t_hi + 1, n))
    tasks = []
    for i in range(n):
        eta = int(rng.integers(0, max_eta + 1))
        w = max(1 + 2 * eta, int(T[i] * rng.uniform(0.3, 1.0) * util))
        g = int(w * rng.uniform(0.1, 0.6)) if eta else 0
        ge = [max(1, g // (2 * eta))] * eta if eta else []
        gm = [max(0, g // (4 * eta))] * eta if eta else []
        tasks.append(dict(C=max(1, w - sum(ge) - sum(gm)), T=T[i], D=T[i], prio=n - i,
                          core=int(rng.integers(0, n_cores)), gm=gm, ge=ge))
    return tasks


@pytest.mark.parametrize("policy,wait", VARIANTS)
def test_matches_exhaustive_least_fixed_point(oracle, policy, wait):
    rng = np.random.default_rng(17 * policy + wait)
    n_sched = 0
    for _ in range(150):
        n = int(rng.integers(1, 7))
        tasks = random_taskset(rng, n, int(rng.integers(1, 4)), 3, 30, 400, rng.uniform(0.05, 0.35))
        theta, eps, L = int(rng.integers(0, 5)), int(rng.integers(0, 5)), int(rng.integers(1, 12))
        resp, sched, _ = oracle_bound(oracle, tasks, policy, wait, theta, eps, L)
        want = Spec(tasks, theta, eps, L).least_fixed_points(policy, wait)
        assert [int(x) for x in resp] == want
        n_sched += sched
    assert 20 < n_sched < 150  # both outcomes are exercised


@pytest.mark.parametrize("policy,wait", VARIANTS)
def test_structure_of_the_bound(oracle, policy, wait):
    rng = np.random.default_rng(policy + 2 * wait)
    for _ in range(150):
        n = int(rng.integers(2, 8))
        tasks = random_taskset(rng, n, 2, 2, 50, 600, 0.15)
        theta, eps, L = 2, 3, 7
        resp, sched, _ = oracle_bound(oracle, tasks, policy, wait, theta, eps, L)
        # never below the task's own demand; the top task has no R-dependent term
        for i, t in enumerate(tasks):
            if resp[i] >= 0:
                assert resp[i] >= t["C"] + sum(t["gm"]) + sum(t["ge"])
                assert resp[i] <= t["D"]
        # sentinels: one -1, then only -2, and the flag agrees
        r = [int(x) for x in resp]
        if sched:
            assert min(r) >= 0
        else:
            k = r.index(-1)
            assert all(x >= 0 for x in r[:k]) and all(x == -2 for x in r[k + 1:])
        # a prefix of the priority order is analysed identically on its own under GCAPS
        # (lower-priority tasks only matter to round-robin, through the TSG count)
        if policy == GCAPS and n > 2:
            sub, _, _ = oracle_bound(oracle, tasks[:-1], policy, wait, theta, eps, L)
            assert [int(x) for x in sub] == r[:-1] or -1 in r[:-1]


@pytest.mark.parametrize("policy,wait", VARIANTS)
def test_monotone_in_load_and_overheads(oracle, policy, wait):
    """More higher-priority demand, a larger theta or a larger eps never shrinks a bound."""
    rng = np.random.default_rng(40 + policy + 2 * wait)

    def leq(a, b):  # bound a <= bound b, where a miss counts as infinity
        for x, y in zip(a, b):
            if y < 0:
                return True  # everything from here on is a miss / not analysed in b
            if x < 0 or x > y:
                return False
        return True

    for _ in range(120):
        n = int(rng.integers(2, 7))
        tasks = random_taskset(rng, n, 2, 2, 50, 600, 0.12)
        theta, eps, L = int(rng.integers(0, 4)), int(rng.integers(0, 4)), int(rng.integers(2, 9))
        base = [int(x) for x in oracle_bound(oracle, tasks, policy, wait, theta, eps, L)[0]]
        # grow one higher-priority task's CPU demand
        k = int(rng.integers(0, n - 1))
        grown = [dict(t) for t in tasks]
        grown[k]["C"] += int(rng.integers(1, 6))
        assert leq(base, [int(x) for x in oracle_bound(oracle, grown, policy, wait, theta, eps, L)[0]])
        # grow one pure GPU segment
        gk = [i for i in range(n) if tasks[i]["ge"]]
        if gk:
            grown = [dict(t, ge=list(t["ge"])) for t in tasks]
            grown[gk[0]]["ge"][0] += int(rng.integers(1, 9))
            assert leq(base, [int(x) for x in oracle_bound(oracle, grown, policy, wait, theta, eps, L)[0]])
        # overheads
        assert leq(base, [int(x) for x in oracle_bound(oracle, tasks, policy, wait, theta + 1, eps, L)[0]])
        assert leq(base, [int(x) for x in oracle_bound(oracle, tasks, policy, wait, theta, eps + 1, L)[0]])
        # add a new top-priority GPU-using task on a random core
        extra = dict(C=2, T=40, D=40, prio=n + 5, core=int(rng.integers(0, 2)), gm=[1], ge=[3])
        more = [int(x) for x in oracle_bound(oracle, [extra] + tasks, policy, wait, theta, eps, L)[0]]
        assert leq(base, more[1:])


@pytest.mark.parametrize("policy,wait", VARIANTS)
def test_caller_order_and_priority_ties(oracle, policy, wait):
    rng = np.random.default_rng(9)
    for _ in range(60):
        n = int(rng.integers(2, 8))
        tasks = random_taskset(rng, n, 2, 2, 50, 600, 0.15)
        ref = oracle_bound(oracle, tasks, policy, wait, 1, 2, 5)[0]
        perm = rng.permutation(n)
        shuffled = [tasks[p] for p in perm]
        got = oracle_bound(oracle, shuffled, policy, wait, 1, 2, 5)[0]
        assert [int(got[k]) for k in range(n)] == [int(ref[perm[k]]) for k in range(n)]
        # equal priorities: the lower caller index ranks higher
        tied = [dict(t, prio=7) for t in tasks]
        assert list(oracle_bound(oracle, tied, policy, wait, 1, 2, 5)[0]) == list(ref)


def test_round_robin_counts_lower_priority_tsgs(oracle):
    top = dict(C=1, T=100, D=100, prio=5, core=0, gm=[0], ge=[4])
    low = [dict(C=1, T=100, D=100, prio=4 - k, core=1, gm=[0], ge=[1]) for k in range(3)]
    r = [int(oracle_bound(oracle, [top] + low[:k], RR, BUSY, 1, 0, 2)[0][0]) for k in range(4)]
    assert r == [5, 5 + 3 * 1 * 2, 5 + 3 * 2 * 2, 5 + 3 * 3 * 2]
    # GCAPS ignores them
    r = [int(oracle_bound(oracle, [top] + low[:k], GCAPS, BUSY, 1, 0, 2)[0][0]) for k in range(4)]
    assert r == [5] * 4


def test_unused_segment_slots_are_ignored(oracle):
    a = oracle.rta_taskset([3, 4], [50, 60], [50, 60], [2, 1], [0, 0], [1, 0], [[1, 9], [9, 9]], [[5, 9], [9, 9]],
                           theta_us=1, eps_us=1, slice_us=2, policy=GCAPS, wait_mode=BUSY)
    b = oracle.rta_taskset([3, 4], [50, 60], [50, 60], [2, 1], [0, 0], [1, 0], [[1, 0], [0, 0]], [[5, 0], [0, 0]],
                           theta_us=1, eps_us=1, slice_us=2, policy=GCAPS, wait_mode=BUSY)
    assert list(a[0]) == list(b[0])


def test_large_values_saturate_to_a_miss(oracle):
    big = 2**32 - 1
    resp, sched, _ = oracle.rta_taskset([big, 5], [big, big], [big, big], [2, 1], [0, 0], [3, 3],
                                        [[big] * 3] * 2, [[big] * 3] * 2, theta_us=big, eps_us=big,
                                        slice_us=1, policy=RR, wait_mode=BUSY)
    assert list(resp) == [-1, -2] and sched == 0


def test_argument_checks(oracle):
    ok = dict(theta_us=1, eps_us=1, slice_us=2, policy=GCAPS, wait_mode=BUSY)
    with pytest.raises(oracle.OracleError) as e:
        oracle.rta_taskset([1], [0], [1], [1], [0], [0], [], [], **ok)  # T = 0
    assert e.value.code == oracle.ETASK
    with pytest.raises(oracle.OracleError):
        oracle.rta_taskset([1], [5], [6], [1], [0], [0], [], [], **ok)  # D > T
    with pytest.raises(oracle.OracleError):
        oracle.rta_taskset([1], [5], [0], [1], [0], [0], [], [], **ok)  # D = 0
    with pytest.raises(oracle.OracleError):
        oracle.rta_taskset([1], [5], [5], [1], [0], [2], [[1]], [[1]], **ok)  # eta > S
    with pytest.raises(oracle.OracleError):
        oracle.rta_taskset([1], [5], [5], [1], [0], [0], [], [], **dict(ok, slice_us=0))  # L = 0
    with pytest.raises(oracle.OracleError) as e:
        oracle.rta_taskset([1], [5], [5], [1], [0], [0], [], [], **dict(ok, policy=3))
    assert e.value.code == oracle.EINVAL


def test_batch_matches_single_calls_and_threads(oracle):
    rng = np.random.default_rng(2)
    N, n, S = 37, 5, 2
    b = dict(theta_us=rng.integers(0, 4, N), eps_us=rng.integers(0, 4, N), slice_us=rng.integers(1, 9, N),
             cpu_us=rng.integers(1, 9, (N, n)), period_us=rng.integers(60, 300, (N, n)),
             prio=rng.integers(0, 4, (N, n)), core=rng.integers(0, 2, (N, n)), n_gseg=rng.integers(0, S + 1, (N, n)),
             gm_us=rng.integers(0, 3, (N, n, S)), ge_us=rng.integers(1, 9, (N, n, S)))
    b["deadline_us"] = b["period_us"] - rng.integers(0, 20, (N, n))
    for wait in (BUSY, SUSPEND):
        resp, sched, terms = oracle.rta_batch(b, 3, wait, threads=1)
        resp4, sched4, terms4 = oracle.rta_batch(b, 3, wait, threads=4)
        assert (resp == resp4).all() and (sched == sched4).all() and terms == terms4
        tot = 0
        for s in range(N):
            for p, pol in enumerate((GCAPS, RR)):
                r, sc, t = oracle.rta_taskset(b["cpu_us"][s], b["period_us"][s], b["deadline_us"][s], b["prio"][s],
                                              b["core"][s], b["n_gseg"][s], b["gm_us"][s], b["ge_us"][s],
                                              theta_us=b["theta_us"][s], eps_us=b["eps_us"][s],
                                              slice_us=b["slice_us"][s], policy=pol, wait_mode=wait)
                assert (resp[p, s] == r).all() and sched[p, s] == sc
                tot += t
        assert tot == terms
    bad = dict(b, period_us=b["period_us"].copy())
    bad["period_us"][21, 3] = 0
    with pytest.raises(oracle.OracleError) as e:
        oracle.rta_batch(bad, 3, BUSY, threads=3)
    assert e.value.code == oracle.ETASK and e.value.first_bad == 21


def test_an_empty_lowest_priority_task_changes_no_bound(oracle):
    """A task with C = 0 and no GPU segment below every other task (what padding a taskset to a fixed task
    count would add) leaves every other bound as it was, in all four analyses, and never improves a verdict.
    Its own bound is the blocking of Lemma 8 plus, under GCAPS with busy-waiting, the GPU work of the tasks
    above it on other cores (Lemma 11); under round-robin and under self-suspension nothing is charged to a
    CPU-only task alone on its core, and it always passes."""
    from paper_2406_05221_amd import taskgen
    groups = taskgen.table3(1500, seed=2, util=(0.3, 0.3), eps_us=300)
    for n, (idx, batch) in groups.items():
        N = len(idx)
        padded = {}
        for k, v in batch.items():
            if v.ndim == 1:
                padded[k] = v
            else:
                pad = np.zeros((N, 1) + v.shape[2:], v.dtype)
                if k in ("period_us", "deadline_us"):
                    pad[:] = 500_000
                if k == "core":
                    pad[:] = 7  # a core of its own
                padded[k] = np.concatenate([v, pad], axis=1)  # prio 0: below the real tasks' 1..n
        for policy in (1, 2):
            for wait in (0, 1):
                r0, s0, _ = oracle.rta_batch(batch, policy, wait, threads=8)
                r1, s1, _ = oracle.rta_batch(padded, policy, wait, threads=8)
                assert np.array_equal(r1[0][:, :n], r0[0])
                assert (s1[0] <= s0[0]).all()
                passed = s0[0] == 1
                own = r1[0][:, n][passed]
                if policy == 2:
                    assert (own == 0).all()  # Lemma 1 with C = G = 0, no same-core task above
                elif wait == 1:
                    assert (own == batch["eps_us"][passed]).all()  # Lemma 8 alone
                else:
                    assert ((own >= batch["eps_us"][passed]) | (own == -1)).all()
                    assert (own > batch["eps_us"][passed]).any()  # Lemma 11: GPU work of the other cores
