"""ctypes access to the CPU oracle (test infrastructure only).

Only tests, the smoke check and the benchmark's CPU-baseline leg import this
package.  It marshals numpy arrays into ``liboracle_rta.so`` (built from
``rta_oracle.cpp`` with g++) and holds no arithmetic of its own.
"""
import ctypes
import os
import subprocess

import numpy as np

_DIR = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_DIR, "liboracle_rta.so")
_lib = None

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
    return _LIB_PATH


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
