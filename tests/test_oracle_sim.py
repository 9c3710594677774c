"""Pins of the batch form of the simulation oracle (oracle/sim_oracle.cpp: oracle_simulate_batch).

The per-task form is pinned by test_oracle_des.py (bounds of Sec. 5 from above, directed schedules).  Here:
schedules worked out by hand on paper (the numbers in the tests were not produced by the simulator), the
closed form of single-core fixed-priority scheduling, invariance under the order the caller lists tasks in,
the way C_i is dealt to the CPU segments, and the analysis bounds from above on generated tasksets."""
import numpy as np
import pytest

import oracle
from paper_2406_05221_amd import taskgen

GCAPS, RR, BOTH, BUSY, SUSPEND = 1, 2, 3, 0, 1


def one_taskset(tasks, theta, eps, L, S=None):
    """tasks: dicts with C, T, prio, core, gm (list), ge (list), off."""
    n = len(tasks)
    S = max([len(t["ge"]) for t in tasks] + [1]) if S is None else S
    b = dict(theta_us=np.array([theta], np.uint32), eps_us=np.array([eps], np.uint32),
             slice_us=np.array([L], np.uint32), cpu_us=np.zeros((1, n), np.uint32),
             period_us=np.zeros((1, n), np.uint32), deadline_us=np.zeros((1, n), np.uint32),
             prio=np.zeros((1, n), np.int32), core=np.zeros((1, n), np.uint8), n_gseg=np.zeros((1, n), np.uint8),
             gm_us=np.zeros((1, n, S), np.uint32), ge_us=np.zeros((1, n, S), np.uint32))
    off = np.zeros((1, n), np.uint32)
    for i, t in enumerate(tasks):
        b["cpu_us"][0, i], b["period_us"][0, i], b["deadline_us"][0, i] = t["C"], t["T"], t["T"]
        b["prio"][0, i], b["core"][0, i], b["n_gseg"][0, i] = t["prio"], t["core"], len(t["ge"])
        b["gm_us"][0, i, :len(t["ge"])], b["ge_us"][0, i, :len(t["ge"])] = t["gm"], t["ge"]
        off[0, i] = t.get("off", 0)
    return b, off


PREEMPTION = [dict(C=2, T=100, prio=3, core=0, gm=[1], ge=[2], off=3),
              dict(C=2, T=100, prio=1, core=1, gm=[0], ge=[10], off=0)]


def test_gcaps_preemption_by_hand():
    """The structure of the motivational example of Sec. 4: the high-priority task asks for the GPU while a
    lower-priority segment runs there, takes it over after one runlist update and hands it back with another.
    eps = 1.  Low task: CPU [0,1), update [1,2), GPU from 2.  High task (released at 3): CPU [3,4), launch [4,5),
    update [5,6), GPU [6,8), update [8,9), CPU [9,10): response 7 = its own 5 ticks + 2 eps.  The low task had 4 of
    its 10 GPU ticks before the takeover, waits during [6,9), runs [9,15), update [15,16), CPU [16,17)."""
    b, off = one_taskset(PREEMPTION, theta=1, eps=1, L=4)
    for wait in (BUSY, SUSPEND):
        mort, jobs, flag = oracle.simulate_batch(b, GCAPS, wait, 50, offset=off)
        assert mort[0, 0].tolist() == [7, 17] and jobs[0, 0].tolist() == [1, 1] and flag[0, 0] == 0


def test_gcaps_with_reversed_gpu_priorities_by_hand():
    """The same two tasks with the GPU-segment priorities the other way round (Sec. 4.3): the request of the task
    with the high CPU priority no longer preempts; it joins the pending list at 5 for free.  Low task: GPU [2,12),
    closing update [12,13), CPU [13,14): response 14.  High task: GPU [13,15), closing update [15,16), CPU [16,17):
    response 17 - 3 = 14.  Round-robin does not look at priorities."""
    b, off = one_taskset(PREEMPTION, theta=1, eps=1, L=4)
    gprio = np.array([[1, 2]], np.int32)
    for wait in (BUSY, SUSPEND):
        mort, jobs, flag = oracle.simulate_batch(b, BOTH, wait, 50, offset=off, gprio=gprio)
        assert mort[:, 0].tolist() == [[14, 14], [10, 16]] and (jobs == 1).all() and (flag == 0).all()


def test_a_task_waiting_for_the_driver_lock_sleeps_in_either_mode():
    """Worked by hand, eps = 2.  Core 1: tau_l (lowest, C = 0, one GPU segment of 5) takes the lock for its opening
    update [0,2).  Core 0: tau_m (C = 3, CPU-only) runs from 0; tau_h (highest, C = 0, one GPU segment of 3) is
    released at 1 and asks for its opening update while the lock is taken: it sleeps on the lock (an rt-mutex,
    Sec. 5.3) and tau_m runs on, [1,2).  At 2 tau_h gets the lock: update [2,4) (tau_l's segment runs [2,4) until the
    update takes effect), GPU [4,7), closing update [7,9): response 8.  Busy-waiting: tau_h keeps core 0 during
    [4,7), tau_m's last tick is [9,10): response 10 (11 if tau_h had spun on the lock during [1,2)).
    Self-suspension: tau_m's last tick is [4,5): response 5.  tau_l: GPU [9,12), closing update [12,14): 14."""
    tasks = [dict(C=0, T=100, prio=3, core=0, gm=[0], ge=[3], off=1),
             dict(C=3, T=100, prio=2, core=0, gm=[], ge=[], off=0),
             dict(C=0, T=100, prio=1, core=1, gm=[0], ge=[5], off=0)]
    b, off = one_taskset(tasks, theta=0, eps=2, L=4)
    mort, _, flag = oracle.simulate_batch(b, GCAPS, BUSY, 60, offset=off)
    assert mort[0, 0].tolist() == [8, 10, 14] and flag[0, 0] == 0
    mort, _, flag = oracle.simulate_batch(b, GCAPS, SUSPEND, 60, offset=off)
    assert mort[0, 0].tolist() == [8, 5, 14] and flag[0, 0] == 0


def test_round_robin_slices_by_hand():
    """The same two tasks under time-sliced round-robin, L = 4, theta = 1.  Low task on the GPU from 1; the
    high task joins the ring at 5.  The low task's slice that began at 5 ends at 9 (it has had 8 ticks), switch
    [9,10), high task [10,12), switch [12,13), low task [13,15).  High: CPU [12,13), response 13 - 3 = 10.
    Low: CPU [15,16), response 16."""
    b, off = one_taskset(PREEMPTION, theta=1, eps=1, L=4)
    for wait in (BUSY, SUSPEND):
        mort, jobs, flag = oracle.simulate_batch(b, RR, wait, 50, offset=off)
        assert mort[0, 0].tolist() == [10, 16] and jobs[0, 0].tolist() == [1, 1] and flag[0, 0] == 0
    both = oracle.simulate_batch(b, BOTH, SUSPEND, 50, offset=off)[0]
    assert both[:, 0].tolist() == [[7, 17], [10, 16]]  # planes: GCAPS, then round-robin


def test_cpu_time_is_dealt_to_the_segments_first_segments_longer():
    """C = 5 around one GPU segment is 3 + 2.  Self-suspension, one core: the high task runs [0,3), is on the GPU
    [3,7) while the low task (C = 3) runs [3,6): response 6 (it would be 5 under a 2 + 3 split); the high task
    ends at 9."""
    tasks = [dict(C=5, T=50, prio=2, core=0, gm=[0], ge=[4]), dict(C=3, T=50, prio=1, core=0, gm=[], ge=[])]
    b, off = one_taskset(tasks, theta=0, eps=0, L=100)
    mort, _, _ = oracle.simulate_batch(b, RR, SUSPEND, 50, offset=off)
    assert mort[0, 0].tolist() == [9, 6]
    mort, _, _ = oracle.simulate_batch(b, RR, BUSY, 50, offset=off)
    assert mort[0, 0].tolist() == [9, 12]  # busy waiting keeps the core: the low task starts at 9


def test_simultaneous_arrivals_take_the_gpu_in_priority_order():
    """Two tasks on two cores reach their GPU segments at the same instant (CPU [0,1) each, G^e = 3, one slice, no
    switch cost): the higher-priority one enters the ring first whatever the order the caller lists them in.
    It runs [1,4) and ends at 5; the other runs [4,7) and ends at 8."""
    low = dict(C=2, T=50, prio=1, core=1, gm=[0], ge=[3])
    high = dict(C=2, T=50, prio=2, core=0, gm=[0], ge=[3])
    for tasks, want in (([low, high], [8, 5]), ([high, low], [5, 8])):
        b, off = one_taskset(tasks, theta=0, eps=0, L=10)
        for wait in (BUSY, SUSPEND):
            mort, _, _ = oracle.simulate_batch(b, RR, wait, 50, offset=off)
            assert mort[0, 0].tolist() == want


def classic_response_time(C, T, i):
    R = C[i]
    while True:
        nxt = C[i] + sum(-(-R // T[h]) * C[h] for h in range(i))
        if nxt == R:
            return R
        R = nxt


def test_single_core_cpu_only_equals_the_textbook_recurrence():
    """Synchronous release on one core is the critical instant: the first job of every task has exactly the response
    time of the classic recurrence R = C_i + sum ceil(R / T_h) C_h, and no later job has a longer one."""
    rng = np.random.default_rng(5)
    done = 0
    while done < 40:
        n = int(rng.integers(2, 6))
        T = sorted(int(x) for x in rng.integers(5, 40, n))
        C = [int(rng.integers(1, max(2, t // 3))) for t in T]
        if sum(c / t for c, t in zip(C, T)) > 0.95:
            continue
        want = [classic_response_time(C, T, i) for i in range(n)]
        if any(w > t for w, t in zip(want, T)):
            continue
        tasks = [dict(C=C[i], T=T[i], prio=n - i, core=0, gm=[], ge=[]) for i in range(n)]
        b, off = one_taskset(tasks, theta=3, eps=2, L=7)
        for policy in (GCAPS, RR):
            mort, jobs, flag = oracle.simulate_batch(b, policy, BUSY, 2000, offset=None)
            assert mort[0, 0].tolist() == want and flag[0, 0] == 0
            assert (jobs[0, 0] >= [2000 // t - 1 for t in T]).all()
        done += 1


def test_result_does_not_depend_on_the_order_of_the_tasks():
    batch = small_batch(12, seed=3)
    rng = np.random.default_rng(9)
    perm = rng.permutation(batch["cpu_us"].shape[1])
    shuffled = {k: (v[:, perm] if v.ndim >= 2 else v) for k, v in batch.items()}
    for wait in (BUSY, SUSPEND):
        a = oracle.simulate_batch(batch, BOTH, wait, 3000)
        s = oracle.simulate_batch(shuffled, BOTH, wait, 3000)
        assert (a[0][:, :, perm] == s[0]).all() and (a[1][:, :, perm] == s[1]).all() and (a[2] == s[2]).all()


def small_batch(N, seed, util=(0.2, 0.5)):
    """Generated tasksets with small numbers (periods of 40-400 ticks) so that the unit-tick oracle is quick."""
    return taskgen.generate(N, n_cores=2, tasks_per_core=3, max_gseg=2, util=util, eta=(0, 2), share=(0.1, 0.5),
                            period=(40, 400), overhead=(1, 3), slice_us=8, seed=seed, stream=77)


def gpu_tasks_lead_their_cores(b):
    """True for tasksets in which no GPU-using task has a higher-priority task on its own core."""
    prio, core, eta = b["prio"], b["core"], b["n_gseg"]
    above = (core[:, :, None] == core[:, None, :]) & (prio[:, None, :] > prio[:, :, None])  # [ts, i, h]
    return ~((eta[:, :, None] > 0) & above).any(axis=(1, 2))


def tasks_no_delayed_update_reaches(b):
    """[N, n] bool, the domain of the GCAPS comparison with eps > 0: tasks above which (in priority) every GPU-using
    task is the highest-priority task of its core.  Only a GPU-using task with a task above it on its core can be
    kept from its closing update, and only tasks below it wait for that."""
    prio, core, eta = b["prio"], b["core"], b["n_gseg"]
    N, n = prio.shape
    out = np.ones((N, n), bool)
    for ts in range(N):
        for i in range(n):
            for h in range(n):
                if prio[ts, h] > prio[ts, i] and eta[ts, h] > 0 and any(
                        core[ts, a] == core[ts, h] and prio[ts, a] > prio[ts, h] for a in range(n)):
                    out[ts, i] = False
    return out


@pytest.mark.parametrize("wait", [BUSY, SUSPEND])
def test_observed_response_times_stay_below_the_bounds(wait):
    """Sec. 5 bounds every job of a schedulable taskset; round-robin is compared at theta = 0 (see test_oracle_des.py
    for the reason).  GCAPS is compared on the tasks that no delayed closing update can reach: a task that is
    preempted on its core between the end of its GPU work and its closing runlist update keeps the GPU from
    lower-priority segments for that long, which the simulator shows and Lemmas 10 and 13 do not charge
    (test_gcaps_bound_misses_a_delayed_closing_update)."""
    batch = small_batch(600, seed=11)
    rr = dict(batch, theta_us=np.zeros_like(batch["theta_us"]))
    rng = np.random.default_rng(2)
    checked = 0
    for policy, b in ((GCAPS, batch), (RR, rr)):
        R, sched, _ = oracle.rta_batch(b, policy, wait)
        ok = sched[0].astype(bool)
        domain = np.broadcast_to(ok[:, None], R[0].shape).copy()
        if policy == GCAPS:
            domain &= tasks_no_delayed_update_reaches(b)
            assert (domain[gpu_tasks_lead_their_cores(b) & ok]).all()  # the taskset-wide condition is the narrower one
        for trial in range(3):
            off = None if trial == 0 else rng.integers(0, 200, b["cpu_us"].shape).astype(np.uint32)
            mort, jobs, flag = oracle.simulate_batch(b, policy, wait, 4000, offset=off)
            assert (flag[0][ok] == 0).all()
            assert (mort[0][domain] <= R[0][domain]).all()
            checked += int(domain.sum())
            assert (jobs[0][ok] >= 1).all()
    assert checked > 3000


def test_gcaps_bound_misses_a_delayed_closing_update():
    """Worked by hand, eps = 1.  Core 0: tau_a (highest, CPU-only, C = 10, released at 3) and tau_b (C = 0, one GPU
    segment of 3).  Core 1: tau_c (lowest, one GPU segment of 2, released at 1).  tau_b: update [0,1), GPU [1,4); at 3
    tau_a takes core 0 until 13, so tau_b can issue its closing update only then, [13,14): response 14.  tau_c joined
    the pending list at 1 for free; its segment runs [14,16), its closing update [16,17): response 16.  Lemma 13
    charges tau_c one job of tau_b: (2 + 2 eps) + 2 eps of blocking + (3 + 2 eps) = 11."""
    tasks = [dict(C=10, T=100, prio=3, core=0, gm=[], ge=[], off=3),
             dict(C=0, T=100, prio=2, core=0, gm=[0], ge=[3], off=0),
             dict(C=0, T=100, prio=1, core=1, gm=[0], ge=[2], off=1)]
    b, off = one_taskset(tasks, theta=0, eps=1, L=4)
    mort, _, _ = oracle.simulate_batch(b, GCAPS, SUSPEND, 60, offset=off)
    assert mort[0, 0].tolist() == [10, 14, 16]
    R, sched, _ = oracle.rta_batch(b, GCAPS, SUSPEND)
    assert sched[0, 0] == 1 and R[0, 0, 2] == 11


def test_overrun_stops_the_taskset_and_is_flagged():
    tasks = [dict(C=8, T=10, prio=2, core=0, gm=[], ge=[]), dict(C=5, T=12, prio=1, core=0, gm=[], ge=[])]
    b, off = one_taskset(tasks, theta=0, eps=0, L=4)
    mort, jobs, flag = oracle.simulate_batch(b, RR, BUSY, 1000, offset=off)
    # low task: 2 ticks in [8,10), none in [10,18), [18,20) -> 4 of 5 done at its next release at 12? no: released
    # again at 12 while the first job still runs -> stop at 12
    assert flag[0, 0] == 1 and jobs[0, 0].tolist() == [1, 0] and mort[0, 0].tolist() == [8, 0]


def test_rejects_a_broken_task_model():
    tasks = [dict(C=1, T=10, prio=1, core=0, gm=[], ge=[])]
    b, off = one_taskset(tasks, theta=0, eps=0, L=0)
    with pytest.raises(ValueError, match="first bad taskset 0"):
        oracle.simulate_batch(b, RR, BUSY, 10, offset=off)
