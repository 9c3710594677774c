"""ctypes access to the CPU oracle (test infrastructure only).

Only tests, the smoke check and the benchmark's CPU-baseline leg import this
package.  It marshals numpy arrays into ``liboracle_rta.so`` (the analysis, built from
``rta_oracle.cpp`` with g++) and ``liboracle_sim.so`` (the unit-tick simulator, built from
``sim_oracle.cpp``) and holds no arithmetic of its own.
"""
import ctypes
import os
import subprocess

import numpy as np

_DIR = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_DIR, "liboracle_rta.so")
_SIM_PATH = os.path.join(_DIR, "liboracle_sim.so")
_lib = None
_sim = None

POLICY_GCAPS = 1
POLICY_RR = 2
POLICY_BOTH = 3
WAIT_BUSY = 0
WAIT_SUSPEND = 1
OPT_LITERAL_LEMMA10 = 1
OPT_CONTINUE_AFTER_MISS = 2
RESP_MISS = -1
RESP_NOT_ANALYSED = -2
OK = 0
EINVAL = -1
ETASK = -2
EORDER = -3


def build(force=False):
    """Compile rta_oracle.cpp into liboracle_rta.so (g++, host only)."""
    src = os.path.join(_DIR, "rta_oracle.cpp")
    if not force and os.path.exists(_LIB_PATH) and os.path.getmtime(_LIB_PATH) >= max(
        os.path.getmtime(src), os.path.getmtime(os.path.join(_DIR, "rta_oracle.h"))
    ):
        return _LIB_PATH
    cmd = ["g++", "-std=c++17", "-O2", "-fPIC", "-shared", "-pthread", "-Wall", "-Wextra",
           "-o", _LIB_PATH, src]
    subprocess.run(cmd, check=True, cwd=_DIR)
    build_sim(force)
    return _LIB_PATH


def build_sim(force=False):
    """Compile sim_oracle.cpp into liboracle_sim.so (g++, host only)."""
    src = os.path.join(_DIR, "sim_oracle.cpp")
    if force or not os.path.exists(_SIM_PATH) or os.path.getmtime(_SIM_PATH) < os.path.getmtime(src):
        subprocess.run(["g++", "-std=c++17", "-O2", "-fPIC", "-shared", "-pthread", "-Wall", "-Wextra",
                        "-o", _SIM_PATH, src], check=True, cwd=_DIR)
    return _SIM_PATH


def open_sim_library(path):
    """Load a build of the simulator's source (the mutation tests load altered copies)."""
    lib = ctypes.CDLL(path)
    lib.des_run.restype = ctypes.c_int
    lib.des_run_gprio.restype = ctypes.c_int
    u32, i32, p = ctypes.c_uint32, ctypes.c_int, ctypes.c_void_p
    lib.oracle_simulate_batch.restype = ctypes.c_int
    lib.oracle_simulate_batch.argtypes = [u32, u32, u32, p, p, p, p, p, p, p, p, p, p, p, p, i32, i32, u32, i32,
                                          p, p, p, p]
    return lib


def sim_library():
    """The simulator's library (ctypes), built on first use."""
    global _sim
    if _sim is None:
        build_sim()
        _sim = open_sim_library(_SIM_PATH)
    return _sim


def _open(path):
    lib = ctypes.CDLL(path)
    u32, i32 = ctypes.c_uint32, ctypes.c_int
    p = ctypes.c_void_p
    lib.oracle_rta_taskset.restype = ctypes.c_int
    lib.oracle_rta_taskset.argtypes = [u32, u32, u32, u32, u32, p, p, p, p, p, p, p, p,
                                       i32, i32, u32, p, p, p]
    lib.oracle_rta_batch.restype = ctypes.c_int
    lib.oracle_rta_batch.argtypes = [u32, u32, u32, p, p, p, p, p, p, p, p, p, p, p,
                                     i32, i32, u32, i32, p, p, p, p]
    lib.oracle_gprio_rta_taskset.restype = ctypes.c_int
    lib.oracle_gprio_rta_taskset.argtypes = [u32, u32, u32, p, p, p, p, p, p, p, p, p, i32, u32, p, p, p]
    lib.oracle_gprio_rta_batch.restype = ctypes.c_int
    lib.oracle_gprio_rta_batch.argtypes = [u32, u32, u32, p, p, p, p, p, p, p, p, p, p, i32, u32, p, p, p]
    lib.oracle_gprio_assign_taskset.restype = ctypes.c_int
    lib.oracle_gprio_assign_taskset.argtypes = [u32, u32, u32, p, p, p, p, p, p, p, p, i32, u32, p, p, p, p]
    lib.oracle_gprio_assign_batch.restype = ctypes.c_int
    lib.oracle_gprio_assign_batch.argtypes = [u32, u32, u32, p, p, p, p, p, p, p, p, p, p, i32, u32, i32,
                                              p, p, p, p, p]
    return lib


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            build()
        _lib = _open(_LIB_PATH)
    return _lib


def open_library(path):
    """Load another build of the oracle's source (used by the mutation tests)."""
    return _open(path)


def _arr(x, dtype):
    return np.ascontiguousarray(np.asarray(x, dtype=dtype))


def _ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p) if a is not None and a.size else None


def npol(policy_mask):
    return bin(policy_mask).count("1")


class OracleError(RuntimeError):
    def __init__(self, code, first_bad=None):
        super().__init__(f"oracle error {code} (first bad taskset: {first_bad})")
        self.code = code
        self.first_bad = first_bad


def rta_taskset(cpu_us, period_us, deadline_us, prio, core, n_gseg, gm_us, ge_us, *, theta_us,
                eps_us, slice_us, policy, wait_mode, options=0, lib=None):
    """One taskset, one policy.  gm_us/ge_us are [n][S].  Returns (resp[n] int64, sched, terms)."""
    cpu = _arr(cpu_us, np.uint32)
    n = cpu.size
    per = _arr(period_us, np.uint32)
    dl = _arr(deadline_us, np.uint32)
    pr = _arr(prio, np.int32)
    co = _arr(core, np.uint8)
    ng = _arr(n_gseg, np.uint8)
    gm = _arr(gm_us, np.uint32).reshape(n, -1) if np.size(gm_us) else np.zeros((n, 0), np.uint32)
    ge = _arr(ge_us, np.uint32).reshape(n, -1) if np.size(ge_us) else np.zeros((n, 0), np.uint32)
    S = gm.shape[1]
    assert ge.shape == gm.shape
    for a in (per, dl, pr, co, ng):
        assert a.size == n
    gm = np.ascontiguousarray(gm)
    ge = np.ascontiguousarray(ge)
    resp = np.zeros(n, np.int64)
    sched = np.zeros(1, np.uint8)
    terms = np.zeros(1, np.uint64)
    rc = (lib or _load()).oracle_rta_taskset(n, S, int(theta_us), int(eps_us), int(slice_us), _ptr(cpu),
                                    _ptr(per), _ptr(dl), _ptr(pr), _ptr(co), _ptr(ng), _ptr(gm),
                                    _ptr(ge), policy, wait_mode, options, _ptr(resp), _ptr(sched),
                                    _ptr(terms))
    if rc != OK:
        raise OracleError(rc)
    return resp, int(sched[0]), int(terms[0])


def rta_batch(batch, policy_mask, wait_mode, *, options=0, threads=1, lib=None):
    """A batch given as a dict of numpy arrays (keys as in the task model:
    theta_us, eps_us, slice_us [N]; cpu_us, period_us, deadline_us, prio, core,
    n_gseg [N, n]; gm_us, ge_us [N, n, S]).  Returns (resp[npol, N, n], sched[npol, N], terms)."""
    cpu = _arr(batch["cpu_us"], np.uint32)
    N, n = cpu.shape
    gm = _arr(batch["gm_us"], np.uint32).reshape(N, n, -1)
    ge = _arr(batch["ge_us"], np.uint32).reshape(N, n, -1)
    S = gm.shape[2]
    th = _arr(batch["theta_us"], np.uint32)
    ep = _arr(batch["eps_us"], np.uint32)
    sl = _arr(batch["slice_us"], np.uint32)
    per = _arr(batch["period_us"], np.uint32)
    dl = _arr(batch["deadline_us"], np.uint32)
    pr = _arr(batch["prio"], np.int32)
    co = _arr(batch["core"], np.uint8)
    ng = _arr(batch["n_gseg"], np.uint8)
    for a in (th, ep, sl):
        assert a.shape == (N,)
    for a in (per, dl, pr, co, ng):
        assert a.shape == (N, n)
    assert ge.shape == gm.shape
    P = npol(policy_mask)
    resp = np.zeros((P, N, n), np.int64)
    sched = np.zeros((P, N), np.uint8)
    terms = np.zeros(1, np.uint64)
    bad = np.full(1, 0xFFFFFFFF, np.uint32)
    rc = (lib or _load()).oracle_rta_batch(N, n, S, _ptr(th), _ptr(ep), _ptr(sl), _ptr(cpu), _ptr(per),
                                  _ptr(dl), _ptr(pr), _ptr(co), _ptr(ng), _ptr(gm), _ptr(ge),
                                  policy_mask, wait_mode, options, threads, _ptr(resp), _ptr(sched),
                                  _ptr(terms), _ptr(bad))
    if rc != OK:
        raise OracleError(rc, int(bad[0]))
    return resp, sched, int(terms[0])


def _taskset_arrays(cpu_us, period_us, deadline_us, prio, core, n_gseg, gm_us, ge_us):
    cpu = _arr(cpu_us, np.uint32)
    n = cpu.size
    per, dl = _arr(period_us, np.uint32), _arr(deadline_us, np.uint32)
    pr, co, ng = _arr(prio, np.int32), _arr(core, np.uint8), _arr(n_gseg, np.uint8)
    gm = _arr(gm_us, np.uint32).reshape(n, -1) if np.size(gm_us) else np.zeros((n, 0), np.uint32)
    ge = _arr(ge_us, np.uint32).reshape(n, -1) if np.size(ge_us) else np.zeros((n, 0), np.uint32)
    assert ge.shape == gm.shape
    for a in (per, dl, pr, co, ng):
        assert a.size == n
    return n, gm.shape[1], cpu, per, dl, pr, co, ng, np.ascontiguousarray(gm), np.ascontiguousarray(ge)


def gprio_rta_taskset(cpu_us, period_us, deadline_us, prio, core, n_gseg, gm_us, ge_us, gprio, *, eps_us,
                      wait_mode, options=0, lib=None):
    """Sec. 5.4 for given GPU-segment priorities.  Returns (resp[n], sched, terms)."""
    n, S, cpu, per, dl, pr, co, ng, gm, ge = _taskset_arrays(cpu_us, period_us, deadline_us, prio, core,
                                                             n_gseg, gm_us, ge_us)
    gp = _arr(gprio, np.int32)
    assert gp.size == n
    resp = np.zeros(n, np.int64)
    sched = np.zeros(1, np.uint8)
    terms = np.zeros(1, np.uint64)
    rc = (lib or _load()).oracle_gprio_rta_taskset(n, S, int(eps_us), _ptr(cpu), _ptr(per), _ptr(dl), _ptr(pr),
                                                   _ptr(co), _ptr(ng), _ptr(gm), _ptr(ge), _ptr(gp), wait_mode,
                                                   options, _ptr(resp), _ptr(sched), _ptr(terms))
    if rc != OK:
        raise OracleError(rc)
    return resp, int(sched[0]), int(terms[0])


def gprio_assign_taskset(cpu_us, period_us, deadline_us, prio, core, n_gseg, gm_us, ge_us, *, eps_us,
                         wait_mode, options=0, lib=None):
    """Sec. 4.3 search.  Returns (gprio[n] int32, resp[n] int64, sched, terms)."""
    n, S, cpu, per, dl, pr, co, ng, gm, ge = _taskset_arrays(cpu_us, period_us, deadline_us, prio, core,
                                                             n_gseg, gm_us, ge_us)
    gp = np.zeros(n, np.int32)
    resp = np.zeros(n, np.int64)
    sched = np.zeros(1, np.uint8)
    terms = np.zeros(1, np.uint64)
    rc = (lib or _load()).oracle_gprio_assign_taskset(n, S, int(eps_us), _ptr(cpu), _ptr(per), _ptr(dl),
                                                      _ptr(pr), _ptr(co), _ptr(ng), _ptr(gm), _ptr(ge),
                                                      wait_mode, options, _ptr(gp), _ptr(resp), _ptr(sched),
                                                      _ptr(terms))
    if rc != OK:
        raise OracleError(rc)
    return gp, resp, int(sched[0]), int(terms[0])


def gprio_assign_batch(batch, wait_mode, *, skip=None, options=0, threads=1, lib=None):
    """Sec. 4.3 search over a batch (dict as for rta_batch).  skip: uint8 [N] or None.
    Returns (gprio[N, n] int32, resp[N, n] int64, sched[N] uint8, terms)."""
    cpu = _arr(batch["cpu_us"], np.uint32)
    N, n = cpu.shape
    gm = _arr(batch["gm_us"], np.uint32).reshape(N, n, -1)
    ge = _arr(batch["ge_us"], np.uint32).reshape(N, n, -1)
    S = gm.shape[2]
    ep = _arr(batch["eps_us"], np.uint32)
    per, dl = _arr(batch["period_us"], np.uint32), _arr(batch["deadline_us"], np.uint32)
    pr, co, ng = _arr(batch["prio"], np.int32), _arr(batch["core"], np.uint8), _arr(batch["n_gseg"], np.uint8)
    assert ep.shape == (N,) and ge.shape == gm.shape
    for a in (per, dl, pr, co, ng):
        assert a.shape == (N, n)
    sk = None if skip is None else _arr(skip, np.uint8)
    assert sk is None or sk.shape == (N,)
    gp = np.zeros((N, n), np.int32)
    resp = np.zeros((N, n), np.int64)
    sched = np.zeros(N, np.uint8)
    terms = np.zeros(1, np.uint64)
    bad = np.full(1, 0xFFFFFFFF, np.uint32)
    rc = (lib or _load()).oracle_gprio_assign_batch(N, n, S, _ptr(ep), _ptr(cpu), _ptr(per), _ptr(dl), _ptr(pr),
                                                    _ptr(co), _ptr(ng), _ptr(gm), _ptr(ge),
                                                    sk.ctypes.data_as(ctypes.c_void_p) if sk is not None else None,
                                                    wait_mode, options, threads, _ptr(gp), _ptr(resp),
                                                    _ptr(sched), _ptr(terms), _ptr(bad))
    if rc != OK:
        raise OracleError(rc, int(bad[0]))
    return gp, resp, sched, int(terms[0])


def gprio_rta_batch(batch, gprio, wait_mode, *, options=0, lib=None):
    """Sec. 5.4 for given GPU-segment priorities over a batch (dict as for rta_batch; gprio int32 [N, n]).
    Returns (resp[N, n] int64, sched[N] uint8)."""
    cpu = _arr(batch["cpu_us"], np.uint32)
    N, n = cpu.shape
    gm = _arr(batch["gm_us"], np.uint32).reshape(N, n, -1)
    ge = _arr(batch["ge_us"], np.uint32).reshape(N, n, -1)
    S = gm.shape[2]
    ep = _arr(batch["eps_us"], np.uint32)
    per, dl = _arr(batch["period_us"], np.uint32), _arr(batch["deadline_us"], np.uint32)
    pr, co, ng = _arr(batch["prio"], np.int32), _arr(batch["core"], np.uint8), _arr(batch["n_gseg"], np.uint8)
    gp = _arr(gprio, np.int32)
    assert gp.shape == (N, n) and ep.shape == (N,)
    resp = np.zeros((N, n), np.int64)
    sched = np.zeros(N, np.uint8)
    bad = np.full(1, 0xFFFFFFFF, np.uint32)
    rc = (lib or _load()).oracle_gprio_rta_batch(N, n, S, _ptr(ep), _ptr(cpu), _ptr(per), _ptr(dl), _ptr(pr), _ptr(co),
                                                 _ptr(ng), _ptr(gm), _ptr(ge), _ptr(gp), wait_mode, options,
                                                 _ptr(resp), _ptr(sched), _ptr(bad))
    if rc != OK:
        raise OracleError(rc, int(bad[0]))
    return resp, sched


def simulate_batch(batch, policy_mask, wait_mode, horizon, offset=None, threads=None, gprio=None):
    """Unit-tick simulation of every taskset of a batch (dict of numpy arrays, analysis layout).
    Returns (mort[P,N,n] int64, jobs[P,N,n] uint32, flag[P,N] uint8); raises ValueError with the index of
    the first taskset that breaks the task model."""
    C = np.ascontiguousarray(batch["cpu_us"], dtype=np.uint32)
    N, n = C.shape
    gm = np.ascontiguousarray(batch["gm_us"], dtype=np.uint32)
    ge = np.ascontiguousarray(batch["ge_us"], dtype=np.uint32)
    S = gm.shape[2]
    P = 2 if policy_mask == POLICY_BOTH else 1
    arrs = [np.ascontiguousarray(batch[k], dtype=t) for k, t in
            (("theta_us", np.uint32), ("eps_us", np.uint32), ("slice_us", np.uint32))]
    T = np.ascontiguousarray(batch["period_us"], dtype=np.uint32)
    prio = np.ascontiguousarray(batch["prio"], dtype=np.int32)
    core = np.ascontiguousarray(batch["core"], dtype=np.uint8)
    eta = np.ascontiguousarray(batch["n_gseg"], dtype=np.uint8)
    off = None if offset is None else np.ascontiguousarray(offset, dtype=np.uint32)
    assert off is None or off.shape == (N, n)
    gp = None if gprio is None else np.ascontiguousarray(gprio, dtype=np.int32)
    assert gp is None or gp.shape == (N, n)
    mort = np.empty((P, N, n), np.int64)
    jobs = np.empty((P, N, n), np.uint32)
    flag = np.empty((P, N), np.uint8)
    bad = ctypes.c_int64(-1)
    ptr = lambda a: None if a is None or a.size == 0 else a.ctypes.data_as(ctypes.c_void_p)
    if threads is None:
        threads = min(16, os.cpu_count() or 1)
    rc = sim_library().oracle_simulate_batch(N, n, S, ptr(arrs[0]), ptr(arrs[1]), ptr(arrs[2]), ptr(C), ptr(T),
                                             ptr(prio), ptr(core), ptr(eta), ptr(gm), ptr(ge), ptr(off),
                                             ptr(gp), policy_mask, wait_mode, int(horizon), threads, ptr(mort), ptr(jobs),
                                             ptr(flag), ctypes.byref(bad))
    if rc != 0:
        raise ValueError(f"simulate_batch: rc={rc}, first bad taskset {bad.value}")
    return mort, jobs, flag
