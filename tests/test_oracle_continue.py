"""Pins of the oracle's continue-after-miss option: the analysis goes on below a task whose bound
exceeds its deadline, with D_h in place of the unknown R_h in the jitters (proof of Lemma 10)."""
import numpy as np
import pytest

from helpers import VARIANTS, oracle_bound, seg_arrays
from test_oracle_des import random_tiny_taskset

GCAPS, RR, BUSY, SUSPEND = 1, 2, 0, 1


def four_tasks():
    return [dict(C=2, T=20, D=20, prio=3, core=0, gm=[0], ge=[8]),
            dict(C=12, T=25, D=25, prio=2, core=0, gm=[0], ge=[4]),
            dict(C=5, T=100, D=100, prio=1, core=1, gm=[0], ge=[10]),
            dict(C=3, T=200, D=200, prio=0, core=0, gm=[], ge=[])]


def test_hand_worked_example(oracle):
    """GCAPS, self-suspension, eps = 0.  tau1 = 2+8 = 10.  tau2 (same core): 16 + ceil((R+8)/20)*2 +
    ceil((R+2)/20)*8 with J^c_1 = 10-2, J^g_1 = 10-8: 16 -> 28 > 25: miss.  From here on R_2 is unknown:
    J^g_2 = D_2 - G^e_2 = 21, J^c_2 = D_2 - (C_2 + G^m_2) = 13.
    tau3 (other core, GPU-using): 15 + ceil((R+2)/20)*8 + ceil((R+21)/25)*4: 15 -> 31 -> 43 -> 51 -> 51
    (51+21 = 72 stays inside three periods of tau2; D_2 alone would reach a fourth).
    tau4 (CPU-only, core of tau1 and tau2): 3 + ceil((R+8)/20)*2 + ceil((R+13)/25)*12: 3 -> 17 -> 31 -> 31."""
    tasks = four_tasks()
    resp, sched, _ = oracle_bound(oracle, tasks, GCAPS, SUSPEND, 0, 0, 1)
    assert list(resp) == [10, -1, -2, -2] and sched == 0
    resp, sched, _ = oracle_bound(oracle, tasks, GCAPS, SUSPEND, 0, 0, 1, options=oracle.OPT_CONTINUE_AFTER_MISS)
    assert list(resp) == [10, -1, 51, 31] and sched == 0


def test_jitter_is_not_taken_below_zero(oracle):
    """tau_a's own GPU time alone exceeds its deadline: D_a - G^e_a < 0, the jitter is 0.  GCAPS,
    busy-waiting, eps = 0, other core: tau_b = 10 + ceil(R/100)*40: 10 -> 50 -> 50 (with a jitter of
    30-40 = -10 the window would shrink; with |.| or D_a it would not change here, so the deadline
    of tau_b is set to make one more arrival visible: R = 50+J crosses 100 only for J > 50)."""
    a = dict(C=1, T=100, D=30, prio=2, core=0, gm=[0], ge=[40])
    b = dict(C=4, T=500, D=500, prio=1, core=1, gm=[0], ge=[6])
    resp, _, _ = oracle_bound(oracle, [a, b], GCAPS, BUSY, 0, 0, 1, options=oracle.OPT_CONTINUE_AFTER_MISS)
    assert list(resp) == [-1, 50]
    # ceil((R + J)/100) with J = -10 and R = 10 would be ceil(0/100) = 0 arrivals: 10, not 50
    b2 = dict(b, C=0, ge=[10])
    resp, _, _ = oracle_bound(oracle, [a, b2], GCAPS, BUSY, 0, 0, 1, options=oracle.OPT_CONTINUE_AFTER_MISS)
    assert list(resp) == [-1, 50]


def test_round_robin_busy_has_no_jitter_to_replace(oracle):
    """Lemmas 4 and 5 use no response time of another task: below a miss every bound is what it
    would be had the task above met its deadline.  tau_b misses (1 > its deadline is forced by D = 1)."""
    a = dict(C=2, T=50, D=50, prio=3, core=0, gm=[1], ge=[3])
    b = dict(C=2, T=60, D=1, prio=2, core=0, gm=[1], ge=[3])
    c = dict(C=4, T=400, D=400, prio=1, core=0, gm=[1], ge=[3])
    resp, _, _ = oracle_bound(oracle, [a, b, c], RR, BUSY, 1, 0, 2, options=oracle.OPT_CONTINUE_AFTER_MISS)
    b_ok = dict(b, D=60)
    ref, _, _ = oracle_bound(oracle, [a, b_ok, c], RR, BUSY, 1, 0, 2)
    assert resp[1] == -1 and ref[1] > 1 and resp[0] == ref[0] and resp[2] == ref[2]


@pytest.mark.parametrize("policy,wait", VARIANTS)
def test_relations_with_the_default_and_with_deadline_jitters(oracle, policy, wait):
    rng = np.random.default_rng(41 + 10 * policy + wait)
    later = 0
    for _ in range(300):
        n = int(rng.integers(2, 7))
        tasks = random_tiny_taskset(rng, n, int(rng.integers(1, 4)), max_eta=2, t_lo=20, t_hi=60)
        for t in tasks:
            t["C"] = sum(t["c"])
            t["ge"] = [g * 2 for g in t["ge"]]
        victim = tasks[int(rng.integers(0, n - 1))]  # a tight deadline somewhere above the lowest task
        victim["D"] = max(1, victim["T"] // 5)
        eps, L = int(rng.integers(0, 3)), int(rng.integers(1, 4))
        ref, ref_s, _ = oracle_bound(oracle, tasks, policy, wait, 1, eps, L)
        got, got_s, _ = oracle_bound(oracle, tasks, policy, wait, 1, eps, L, options=oracle.OPT_CONTINUE_AFTER_MISS)
        assert ref_s == got_s and (got != -2).all()
        order = sorted(range(n), key=lambda i: -tasks[i]["prio"])
        first_miss = next((k for k, i in enumerate(order) if ref[i] == -1), n)
        for k, i in enumerate(order):
            if k <= first_miss:
                assert got[i] == ref[i]
            else:
                assert ref[i] == -2
                later += got[i] >= 0
        if policy == GCAPS:
            # D_h in EVERY jitter (Sec. 5.4 with GPU priority = CPU priority) can only be larger
            gm, ge, eta = seg_arrays(tasks)
            allD, _, _ = oracle.gprio_rta_taskset([t["C"] for t in tasks], [t["T"] for t in tasks],
                                                  [t["D"] for t in tasks], [t["prio"] for t in tasks],
                                                  [t["core"] for t in tasks], eta, gm, ge,
                                                  [t["prio"] for t in tasks], eps_us=eps, wait_mode=wait)
            for i in range(n):
                assert allD[i] == -1 or (0 <= got[i] <= allD[i])
    assert later > 30


def test_every_task_missing_equals_deadline_jitters(oracle):
    """If every task above tau_i missed, every jitter tau_i sees is the one of Sec. 5.4."""
    tasks = four_tasks()
    tasks[0]["D"] = 5   # tau1: own demand 10 > 5
    tasks[1]["D"] = 15  # tau2: 16 > 15
    got, _, _ = oracle_bound(oracle, tasks, GCAPS, SUSPEND, 0, 0, 1, options=oracle.OPT_CONTINUE_AFTER_MISS)
    gm, ge, eta = seg_arrays(tasks)
    allD, _, _ = oracle.gprio_rta_taskset([t["C"] for t in tasks], [t["T"] for t in tasks], [t["D"] for t in tasks],
                                          [t["prio"] for t in tasks], [t["core"] for t in tasks], eta, gm, ge,
                                          [t["prio"] for t in tasks], eps_us=0, wait_mode=SUSPEND)
    assert list(got[:2]) == [-1, -1] and list(got) == list(allD) and got[2] > 0 and got[3] > 0
