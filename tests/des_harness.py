"""Per-task wrapper of the unit-tick simulator (oracle/sim_oracle.cpp, host only)."""
import ctypes

import numpy as np

import oracle


def build(force=False):
    return oracle.build_sim(force)


def _load():
    return oracle.sim_library()


def run(tasks, *, policy, wait_mode, theta, eps, L, offsets, horizon, gprio=None, free_switch=None):
    """tasks: list of dicts with core, prio, T, D, c (eta+1 ints), gm, ge (eta ints each).
    gprio: priorities of the GPU segments (GCAPS runlist decisions), default = prio.
    free_switch: round-robin only, flags of the tasks whose own time slices are brought in by a switch
    that takes no time (the accounting of Eq. 3 from those tasks' side), default: none.
    Returns (rc, max_resp[n], jobs_done[n])."""
    n = len(tasks)
    max_eta = max(len(t["ge"]) for t in tasks)
    c = np.zeros((n, max_eta + 1), np.int32)
    gm = np.zeros((n, max(max_eta, 1)), np.int32)
    ge = np.zeros((n, max(max_eta, 1)), np.int32)
    eta = np.zeros(n, np.int32)
    for i, t in enumerate(tasks):
        e = len(t["ge"])
        assert len(t["gm"]) == e and len(t["c"]) == e + 1
        eta[i] = e
        c[i, : e + 1] = t["c"]
        gm[i, :e] = t["gm"]
        ge[i, :e] = t["ge"]
    if max_eta == 0:
        gm = np.zeros((n, 0), np.int32)
        ge = np.zeros((n, 0), np.int32)
    gm = np.ascontiguousarray(gm[:, :max_eta])
    ge = np.ascontiguousarray(ge[:, :max_eta])
    arr = lambda key: np.ascontiguousarray([t[key] for t in tasks], dtype=np.int32)
    core, prio, T, D = arr("core"), arr("prio"), arr("T"), arr("D")
    off = np.ascontiguousarray(offsets, dtype=np.int32)
    mr = np.zeros(n, np.int32)
    jd = np.zeros(n, np.int32)
    p = lambda a: a.ctypes.data_as(ctypes.c_void_p)
    gp = prio if gprio is None else np.ascontiguousarray(gprio, dtype=np.int32)
    assert gp.size == n
    fs = None if free_switch is None else np.ascontiguousarray(free_switch, dtype=np.int32)
    assert fs is None or fs.size == n
    lib = _load()
    lib.des_run_free.restype = ctypes.c_int
    rc = lib.des_run_free(n, max_eta, policy, wait_mode, theta, eps, L, p(core), p(prio), p(gp), p(T), p(D), p(off),
                          p(eta), p(c), p(gm), p(ge), None if fs is None else p(fs), horizon, p(mr), p(jd))
    return rc, mr, jd
