"""The analytic bounds must dominate every response time a concrete schedule produces.
A unit-tick simulator (oracle/sim_oracle.cpp, independent of the analysis oracle) runs tiny tasksets
under both GPU policies and both waiting modes; for tasksets the oracle calls schedulable no
job may respond later than its bound.

Round-robin and theta: Eq. 3 charges theta once per slice of each *other* TSG.  A schedule in
which every slice, the task's own included, is followed by a switch therefore pays one more
theta per own slice than Eq. 3 counts.  The simulator is compared (a) with theta = 0, where Eq. 3
is exact for it, and (b) with theta > 0 against the bound evaluated at 2*theta, which covers the
own-slice switches whenever another TSG exists (and no switch happens when none does)."""
import itertools

import numpy as np
import pytest

import des_harness as des
from helpers import VARIANTS, oracle_bound

GCAPS, RR, BUSY, SUSPEND = 1, 2, 0, 1


def random_tiny_taskset(rng, n, n_cores, max_eta, t_lo=10, t_hi=40, rm=True):
    tasks = []
    for _ in range(n):
        T = int(rng.integers(t_lo, t_hi + 1))
        eta = int(rng.integers(0, max_eta + 1))
        c = [int(rng.integers(0, 4)) for _ in range(eta + 1)]
        if sum(c) == 0:
            c[0] = 1
        tasks.append(dict(core=int(rng.integers(0, n_cores)), T=T, D=T, c=c,
                          gm=[int(rng.integers(0, 2)) for _ in range(eta)],
                          ge=[int(rng.integers(1, 6)) for _ in range(eta)]))
    if rm:
        tasks.sort(key=lambda t: t["T"])
    else:
        rng.shuffle(tasks)
    for i, t in enumerate(tasks):
        t["prio"] = n - i
    return tasks


def check(oracle, tasks, policy, wait, theta, eps, L, offsets_list, horizon, bound_theta=None):
    R, sched, _ = oracle_bound(oracle, tasks, policy, wait, theta if bound_theta is None else bound_theta, eps, L)
    if not sched:
        return None
    worst = np.zeros(len(tasks), int)
    for offs in offsets_list:
        rc, mr, jd = des.run(tasks, policy=policy, wait_mode=wait, theta=theta, eps=eps, L=L,
                             offsets=offs, horizon=horizon)
        assert rc == 0, (tasks, policy, wait, theta, eps, L, offs)
        assert (mr <= R).all(), (tasks, policy, wait, theta, eps, L, offs, mr, R)
        worst = np.maximum(worst, mr)
    return worst, R


@pytest.mark.parametrize("policy,wait", VARIANTS)
def test_simulated_response_never_exceeds_bound(oracle, policy, wait):
    rng = np.random.default_rng(100 * policy + wait)
    checked = 0
    for trial in range(220):
        n = int(rng.integers(2, 6))
        tasks = random_tiny_taskset(rng, n, n_cores=int(rng.integers(1, 4)), max_eta=2, rm=bool(trial % 2))
        eps = int(rng.integers(0, 3))
        L = int(rng.integers(1, 4))
        offs = [[0] * n] + [[int(x) for x in rng.integers(0, 25, n)] for _ in range(24)]
        if check(oracle, tasks, policy, wait, 0, eps, L, offs, 500) is not None:
            checked += 1
    assert checked > 60


@pytest.mark.parametrize("wait", [BUSY, SUSPEND])
def test_round_robin_with_switch_cost(oracle, wait):
    rng = np.random.default_rng(7 + wait)
    checked = 0
    for trial in range(200):
        n = int(rng.integers(2, 6))
        tasks = random_tiny_taskset(rng, n, n_cores=int(rng.integers(1, 4)), max_eta=2, t_lo=20, t_hi=60,
                                    rm=bool(trial % 2))
        theta = int(rng.integers(1, 3))
        L = int(rng.integers(1, 4))
        offs = [[0] * n] + [[int(x) for x in rng.integers(0, 30, n)] for _ in range(24)]
        if check(oracle, tasks, RR, wait, theta, 0, L, offs, 600, bound_theta=2 * theta) is not None:
            checked += 1
    assert checked > 40


def test_directed_carry_in_other_core(oracle):
    """The GPU work of a higher-priority task on another core lands late in its first job (delayed
    on its own core) and early in the second: two preemptions inside one window shorter than
    T_h.  The schedule reaches the bound of Lemma 10 / 13 exactly (19), which the same sums
    without the jitter J^g_h (15) would not cover."""
    tasks = [dict(core=0, prio=3, T=40, D=40, c=[8], gm=[], ge=[]),
             dict(core=0, prio=2, T=20, D=20, c=[1, 0], gm=[0], ge=[4]),
             dict(core=1, prio=1, T=40, D=40, c=[1, 0], gm=[0], ge=[10])]
    for wait in (BUSY, SUSPEND):
        worst, R = check(oracle, tasks, GCAPS, wait, 0, 0, 1, [[0, 0, 8]], 200)
        assert worst[2] == 19 and R[2] == 19


def test_directed_self_suspension_same_core(oracle):
    """A self-suspending higher-priority task whose first job is stretched by GPU preemption from
    another core executes its last CPU part late and the first CPU part of its next job on time:
    the lower-priority task on its core sees more than ceil(R/T_h) jobs' worth (16 > 13); the
    jitter J^c_h of Lemma 15 covers it (17)."""
    tasks = [dict(core=1, prio=3, T=40, D=40, c=[1, 0], gm=[0], ge=[8]),
             dict(core=0, prio=2, T=20, D=20, c=[1, 3], gm=[0], ge=[5]),
             dict(core=0, prio=1, T=40, D=40, c=[9], gm=[], ge=[])]
    worst, R = check(oracle, tasks, GCAPS, SUSPEND, 0, 0, 1, [[0, 0, 14], [0, 0, 13], [0, 0, 15]], 200)
    assert worst[2] == 16 and R[2] == 17


@pytest.mark.parametrize("policy,wait", VARIANTS)
def test_exhaustive_offsets_on_three_tasks(oracle, policy, wait):
    rng = np.random.default_rng(31 * policy + wait)
    checked = 0
    for trial in range(40):
        tasks = random_tiny_taskset(rng, 3, n_cores=2, max_eta=1, t_lo=6, t_hi=14, rm=bool(trial % 2))
        eps, L = int(rng.integers(0, 2)), int(rng.integers(1, 4))
        offs = [list(o) + [0] for o in itertools.product(range(tasks[0]["T"]), range(tasks[1]["T"]))]
        if check(oracle, tasks, policy, wait, 0, eps, L, offs, 160) is not None:
            checked += 1
    assert checked > 5
