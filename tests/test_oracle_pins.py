"""Pins of the CPU oracle that do not go through the oracle's own code:
hand-worked fixed points, the textbook uniprocessor special case, closed forms
of Eq. 3, the verdict the paper prints for Table 2."""
import numpy as np
import pytest

from helpers import VARIANTS, classic_rta, load_table2, oracle_bound

GCAPS, RR, BUSY, SUSPEND = 1, 2, 0, 1


def cpu_only(C, T, core=None, D=None):
    n = len(C)
    return [dict(C=C[i], T=T[i], D=(D or T)[i], prio=n - i, core=(core or [0] * n)[i], gm=[], ge=[])
            for i in range(n)]


# ---- classic response-time analysis, hand-worked ------------------------------------------
# (C,T) = (1,4),(2,6),(3,13): R1 = 1; R2: 2 -> 2+1 = 3 -> 3; R3: 3 -> 3+1+2 = 6 -> 3+2+2 = 7
# -> 3+2+4 = 9 -> 3+3+4 = 10 -> 3+3+4 = 10.
# (C,T) = (3,7),(3,12),(5,20): R = 3, 6, 20 (5 -> 11 -> 14 -> 17 -> 20 -> 20).
@pytest.mark.parametrize("C,T,R", [([1, 2, 3], [4, 6, 13], [1, 3, 10]), ([3, 3, 5], [7, 12, 20], [3, 6, 20])])
@pytest.mark.parametrize("policy,wait", VARIANTS)
def test_classic_hand_examples(oracle, C, T, R, policy, wait):
    resp, sched, _ = oracle_bound(oracle, cpu_only(C, T), policy, wait, theta=7, eps=0, L=5)
    assert list(resp) == R and sched == 1


@pytest.mark.parametrize("policy,wait", VARIANTS)
def test_cpu_only_reduces_to_textbook_rta(oracle, policy, wait):
    """Without GPU segments every analysis is the uniprocessor RTA per core; under GCAPS each
    task under analysis additionally carries the one blocking term eps of Lemma 8."""
    rng = np.random.default_rng(11)
    for _ in range(200):
        n = int(rng.integers(1, 7))
        T = sorted(int(x) for x in rng.integers(5, 200, n))
        C = [max(1, int(t * rng.uniform(0.02, 0.45))) for t in T]
        eps = int(rng.integers(0, 4))
        resp, sched, _ = oracle_bound(oracle, cpu_only(C, T), policy, wait, theta=3, eps=eps, L=4)
        blocking = eps if policy == GCAPS else 0
        # textbook routine with the blocking added to the task under analysis only
        want = []
        for i in range(n):
            r = classic_rta(C[:i] + [C[i] + blocking], T[: i + 1], T[: i + 1])[-1]
            if r is None:
                break
            want.append(r)
        got = [int(x) for x in resp]
        assert got[: len(want)] == want
        if len(want) < n:
            assert got[len(want)] == -1 and all(x == -2 for x in got[len(want) + 1:]) and sched == 0
        else:
            assert sched == 1


@pytest.mark.parametrize("policy,wait", VARIANTS)
def test_two_cores_are_independent_without_gpu(oracle, policy, wait):
    C, T = [1, 2, 2, 3, 3, 5], [4, 7, 6, 12, 13, 20]
    core = [0, 1, 0, 1, 0, 1]
    resp, _, _ = oracle_bound(oracle, cpu_only(C, T, core), policy, wait, theta=1, eps=0, L=3)
    a = classic_rta(C[0::2], T[0::2], T[0::2])
    b = classic_rta(C[1::2], T[1::2], T[1::2])
    assert list(resp[0::2]) == a and list(resp[1::2]) == b


def test_single_core_gcaps_busy_is_classic_rta_on_inflated_wcet(oracle):
    """One core, eps = 0, busy-waiting: a task holds its core for C + G^m + G^e, so the bound is
    the textbook RTA with that demand (Lemma 12 plus the same-core sum of Lemma 10)."""
    rng = np.random.default_rng(5)
    for _ in range(200):
        n = int(rng.integers(1, 6))
        T = sorted(int(x) for x in rng.integers(20, 300, n))
        tasks, W = [], []
        for i in range(n):
            eta = int(rng.integers(0, 3))
            gm = [int(x) for x in rng.integers(0, 3, eta)]
            ge = [int(x) for x in rng.integers(1, 8, eta)]
            C = int(rng.integers(1, 8))
            tasks.append(dict(C=C, T=T[i], D=T[i], prio=n - i, core=0, gm=gm, ge=ge))
            W.append(C + sum(gm) + sum(ge))
        resp, _, _ = oracle_bound(oracle, tasks, GCAPS, BUSY, theta=0, eps=0, L=1)
        want = classic_rta(W, T, T)
        got = [int(x) if x >= 0 else None for x in resp]
        assert got == want


# ---- Eq. 3 closed forms ---------------------------------------------------------------------
def test_round_robin_interleave_closed_form(oracle):
    """Highest-priority task, alone on its core: R = C + G + (L+theta) * nu * sum_j ceil(Ge_j / L)
    with nu = number of other GPU-using tasks (Lemma 1, Eq. 3); no R-dependent term."""
    L, theta = 10, 3
    t1 = dict(C=4, T=1000, D=1000, prio=9, core=0, gm=[1, 2], ge=[25, 10])       # ceil: 3 + 1 = 4
    others = [dict(C=1, T=2000, D=2000, prio=5 - k, core=1 + k, gm=[0], ge=[5]) for k in range(3)]
    cpu = dict(C=1, T=3000, D=3000, prio=1, core=5, gm=[], ge=[])
    for wait in (BUSY, SUSPEND):
        resp, _, _ = oracle_bound(oracle, [t1] + others + [cpu], RR, wait, theta=theta, eps=99, L=L)
        assert resp[0] == 4 + (3 + 35) + (L + theta) * 3 * 4
        # the CPU-only task has no interleaved execution and nobody above it on its core
        assert resp[4] == 1
    # a lone GPU-using task is never interleaved
    resp, _, _ = oracle_bound(oracle, [t1, cpu], RR, BUSY, theta=theta, eps=0, L=L)
    assert resp[0] == 4 + 38


def test_gcaps_top_task_closed_form(oracle):
    """Highest-priority task: R = C + G + 2*eps*eta + (eta+1)*eps (Sec. 5.3, Lemma 8)."""
    t1 = dict(C=4, T=1000, D=1000, prio=9, core=0, gm=[1, 2], ge=[25, 10])
    for wait in (BUSY, SUSPEND):
        resp, _, _ = oracle_bound(oracle, [t1], GCAPS, wait, theta=50, eps=7, L=1)
        assert resp[0] == 4 + 38 + 2 * 7 * 2 + 3 * 7


# ---- the paper's own example ----------------------------------------------------------------
def test_table2_printed_verdict(oracle):
    g, tasks = load_table2()
    v = g["printed_verdict"]
    assert v["policy"] == "gcaps" and v["wait_mode"] == "suspend" and v["schedulable"] is False
    for eps in (0, 1):
        _, sched, _ = oracle_bound(oracle, tasks, GCAPS, SUSPEND, theta=0, eps=eps, L=1)
        assert sched == 0


def test_table2_hand_worked_values(oracle):
    """eps = 0.  tau1: 9+10 = 19.  tau2 (CPU-only, core of tau1): 40 + ceil((R+6)/80)*13 -> 53
    (J^c_1 = 19-13 = 6).  tau3 (other core): 119 + ceil((R+13)/80)*6 -> 131 (J^g_1 = 19-6).
    tau4: 30 + ceil(R/150)*40 + ceil((R+6)/80)*13 + ceil((R+13)/80)*6 + ceil((R+51)/190)*80:
    30 -> 169 -> 327 > 200: miss.  Busy-waiting: tau2 = 40 + ceil(R/80)*(13+6) -> 59 (53 with the
    literal guard of Lemma 10), tau3 = 131, tau4: 30 -> 169 -> 327: miss."""
    _, tasks = load_table2()
    resp, sched, _ = oracle_bound(oracle, tasks, GCAPS, SUSPEND, theta=0, eps=0, L=1)
    assert list(resp) == [19, 53, 131, -1] and sched == 0
    resp, _, _ = oracle_bound(oracle, tasks, GCAPS, BUSY, theta=0, eps=0, L=1)
    assert list(resp) == [19, 59, 131, -1]
    resp, _, _ = oracle_bound(oracle, tasks, GCAPS, BUSY, theta=0, eps=0, L=1, options=oracle.OPT_LITERAL_LEMMA10)
    assert list(resp) == [19, 53, 131, -1]


# ---- a three-task example with every overhead non-zero, worked by hand -------------------------
def three_task_example():
    return [dict(C=5, T=100, D=100, prio=3, core=0, gm=[1], ge=[8]),
            dict(C=20, T=200, D=200, prio=2, core=0, gm=[], ge=[]),
            dict(C=10, T=300, D=300, prio=1, core=1, gm=[2], ge=[25])]


@pytest.mark.parametrize("policy,wait,want", [
    # L = 10, theta = 2, eps = 3; two GPU-using tasks.
    # RR: tau1 = 5+9 + 12*1*ceil(8/10) = 26; tau3 = 10+27 + 12*1*ceil(25/10) = 73.
    #   suspend: tau2 = 20 + ceil((R+20)/100)*6 -> 26   (J^c_1 = 26-6)
    #   busy:    tau2 = 20 + ceil(R/100)*6 + ceil(R/100)*12*2*1 -> 50   (nu = {tau3} + tau_h = 2)
    (RR, SUSPEND, [26, 26, 73]), (RR, BUSY, [26, 50, 73]),
    # GCAPS: tau1 = 14 + 2*3 + 2*3 = 26; tau3 = 37+6+6 = 49, + ceil((R+18)/100)*14 -> 63 (J^g_1 = 26-8)
    #   suspend: tau2 = 20+3 + ceil((R+20)/100)*(5+1+6) -> 35
    #   busy:    tau2 = 23 + ceil(R/100)*6 + ceil(R/100)*14 -> 43
    (GCAPS, SUSPEND, [26, 35, 63]), (GCAPS, BUSY, [26, 43, 63])])
def test_three_task_example(oracle, policy, wait, want):
    resp, sched, _ = oracle_bound(oracle, three_task_example(), policy, wait, theta=2, eps=3, L=10)
    assert list(resp) == want and sched == 1


def test_literal_lemma10_switch(oracle):
    resp, _, _ = oracle_bound(oracle, three_task_example(), GCAPS, BUSY, theta=2, eps=3, L=10,
                              options=oracle.OPT_LITERAL_LEMMA10)
    assert list(resp) == [26, 29, 63]


# ---- jitter terms, worked by hand ---------------------------------------------------------------
def test_carry_in_jitter_other_core(oracle):
    """eps = 0.  core 0: a (C=8, T=40, top), h (C=1, Ge=4, T=20); core 1: i (C=1, Ge=10, T=40, lowest).
    R_h = 5 + 8 = 13, J^g_h = 13-4 = 9.  R_i = 11 + ceil((R+9)/20)*4: 11 -> 15 -> 19 -> 19."""
    tasks = [dict(C=8, T=40, D=40, prio=3, core=0, gm=[], ge=[]),
             dict(C=1, T=20, D=20, prio=2, core=0, gm=[0], ge=[4]),
             dict(C=1, T=40, D=40, prio=1, core=1, gm=[0], ge=[10])]
    for wait in (BUSY, SUSPEND):
        resp, _, _ = oracle_bound(oracle, tasks, GCAPS, wait, theta=0, eps=0, L=1)
        assert list(resp) == [8, 13, 19]


def test_self_suspension_jitter_same_core(oracle):
    """eps = 0, suspend.  core 1: g (C=0.. Ge=8, T=40, top).  core 0: h (C=4, Ge=5, T=20), i (C=9, T=40, CPU-only).
    R_g = 9.  R_h = 9 + ceil((R+1)/40)*8 = 17 (J^g_g = 9-8 = 1), J^c_h = 17-4 = 13.
    R_i = 9 + ceil((R+13)/20)*4: 9 -> 17 -> 17 (ceil(30/20) = 2)."""
    tasks = [dict(C=1, T=40, D=40, prio=3, core=1, gm=[0], ge=[8]),
             dict(C=4, T=20, D=20, prio=2, core=0, gm=[0], ge=[5]),
             dict(C=9, T=40, D=40, prio=1, core=0, gm=[], ge=[])]
    resp, _, _ = oracle_bound(oracle, tasks, GCAPS, SUSPEND, theta=0, eps=0, L=1)
    assert list(resp) == [9, 17, 17]
    # round-robin, suspend: tau_h's interleave with g: (1+0)*1*ceil(5/1) = 5 -> R_h = 9+5 = 14, J^c_h = 10;
    # R_i = 9 + ceil((R+10)/20)*4: 9 -> 13 -> 17 -> 17.
    resp, _, _ = oracle_bound(oracle, tasks, RR, SUSPEND, theta=0, eps=0, L=1)
    assert list(resp) == [9 + 8, 14, 17]


# ---- theta enters only through (L + theta) when every pure GPU segment fits one slice -----------
def test_theta_slice_identity(oracle):
    rng = np.random.default_rng(3)
    for _ in range(100):
        n = int(rng.integers(2, 6))
        L, theta = int(rng.integers(4, 9)), int(rng.integers(1, 5))
        T = sorted(int(x) for x in rng.integers(60, 400, n))
        tasks = []
        for i in range(n):
            eta = int(rng.integers(0, 3))
            tasks.append(dict(C=int(rng.integers(1, 6)), T=T[i], D=T[i], prio=n - i, core=int(rng.integers(0, 2)),
                              gm=[int(x) for x in rng.integers(0, 2, eta)],
                              ge=[int(x) for x in rng.integers(1, L + 1, eta)]))
        for wait in (BUSY, SUSPEND):
            a = oracle_bound(oracle, tasks, RR, wait, theta=theta, eps=0, L=L)
            b = oracle_bound(oracle, tasks, RR, wait, theta=0, eps=0, L=L + theta)
            assert list(a[0]) == list(b[0]) and a[1] == b[1]
