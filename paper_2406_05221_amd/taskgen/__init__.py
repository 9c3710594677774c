"""Seeded synthetic tasksets shaped like the schedulability experiments of Sec. 6.1.

Input generation only: this module (and ``taskgen.cpp`` behind it) holds none of
the response-time analysis.  ``config(k)`` returns the five named workloads;
``generate`` is the general entry.  A batch is a dict of numpy arrays:

    theta_us, eps_us, slice_us            uint32 [N]
    cpu_us, period_us, deadline_us        uint32 [N, n]
    prio int32 [N, n]; core, n_gseg       uint8  [N, n]
    gm_us, ge_us                          uint32 [N, n, S]
"""
import ctypes
import os
import subprocess

import numpy as np

_DIR = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_DIR, "taskgen.cpp")
_LIB_PATH = os.path.join(_DIR, "libtaskgen.so")
_lib = None


def build(force=False):
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < os.path.getmtime(_SRC):
        # -ffp-contract=off: no fused multiply-add, so that the device generator can match bit for bit
        subprocess.run(["g++", "-std=c++17", "-O2", "-ffp-contract=off", "-fPIC", "-shared", "-pthread", "-Wall",
                        "-Wextra", "-o", _LIB_PATH, _SRC], check=True)
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            build()
        _lib = ctypes.CDLL(_LIB_PATH)
        u64, u32, dbl, p, i32 = ctypes.c_uint64, ctypes.c_uint32, ctypes.c_double, ctypes.c_void_p, ctypes.c_int
        _lib.taskgen_generate.restype = ctypes.c_int
        _lib.taskgen_generate.argtypes = ([u64, u64, u64, u32, u32, u32, u32, dbl, dbl, p, u32, u32, dbl, dbl, p,
                                           u32, u32, u32, u32, p, u32, p, i32] + [p] * 11)
        _lib.taskgen_table3.restype = ctypes.c_int
        _lib.taskgen_table3.argtypes = ([u64, u64, u64, u32, u32, u32, u32, u32, dbl, dbl, dbl, dbl, u32, u32, u32, u32,
                                         dbl, dbl, dbl, dbl, u32, u32, u32, i32] + [p] * 12)
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def generate(n_tasksets, *, n_cores, tasks_per_core, max_gseg, util, eta, share, period, overhead, slice_us,
             seed=0, stream=0, first_index=0, threads=None):
    """util/share: (lo, hi) drawn uniformly (util per core, share per task) or a float64 array [N]
    fixing the value per taskset; eta, period: inclusive integer ranges; overhead (theta = eps):
    inclusive integer range or uint32 array [N]; slice_us: int or uint32 array [N]."""
    N, n, S = int(n_tasksets), n_cores * tasks_per_core, max_gseg

    def rng_or_fixed(x, dtype):
        if isinstance(x, np.ndarray):
            a = np.ascontiguousarray(x, dtype=dtype)
            assert a.shape == (N,)
            return (0, 0), a
        return x, None

    (u_lo, u_hi), u_fix = rng_or_fixed(util, np.float64)
    (s_lo, s_hi), s_fix = rng_or_fixed(share, np.float64)
    (o_lo, o_hi), o_fix = rng_or_fixed(overhead, np.uint32)
    if isinstance(slice_us, np.ndarray):
        l_fix, l_val = np.ascontiguousarray(slice_us, dtype=np.uint32), 0
        assert l_fix.shape == (N,)
    else:
        l_fix, l_val = None, int(slice_us)
    out = dict(theta_us=np.empty(N, np.uint32), eps_us=np.empty(N, np.uint32), slice_us=np.empty(N, np.uint32),
               cpu_us=np.empty((N, n), np.uint32), period_us=np.empty((N, n), np.uint32),
               deadline_us=np.empty((N, n), np.uint32), prio=np.empty((N, n), np.int32),
               core=np.empty((N, n), np.uint8), n_gseg=np.empty((N, n), np.uint8),
               gm_us=np.empty((N, n, S), np.uint32), ge_us=np.empty((N, n, S), np.uint32))
    if threads is None:
        threads = min(16, os.cpu_count() or 1)
    rc = _load().taskgen_generate(seed, stream, first_index, N, n_cores, tasks_per_core, S, float(u_lo), float(u_hi),
                                  _ptr(u_fix), eta[0], eta[1], float(s_lo), float(s_hi), _ptr(s_fix), period[0],
                                  period[1], int(o_lo), int(o_hi), _ptr(o_fix), l_val, _ptr(l_fix), threads,
                                  *[_ptr(out[k]) for k in ("theta_us", "eps_us", "slice_us", "cpu_us", "period_us",
                                                           "deadline_us", "prio", "core", "n_gseg", "gm_us", "ge_us")])
    if rc != 0:
        raise ValueError("taskgen: invalid generation parameters")
    return out


# ---- the five named workloads -------------------------------------------------------------------
CONFIG_SIZES = {1: 1000, 2: 9000, 3: 1_000_000, 4: 100_000, 5: 10_000_000}
CONFIG_SHAPES = {1: (2, 3, 1), 2: (4, 4, 3), 3: (4, 5, 3), 4: (8, 10, 5), 5: (4, 6, 4)}  # cores, tasks/core, S

_GRID5 = [(u, g, o, l) for u in (0.3, 0.5, 0.7, 0.9) for g in (0.1, 0.3, 0.5) for o in (50, 200, 500)
          for l in (512, 1024, 2048)]


def config_params(k, n_tasksets=None, *, first_index=0, seed=0):
    """The generation parameters of workload k (1..5) as keyword arguments of ``generate`` (and of the
    device-side generator of the GPU library, which takes the same ones), with n_tasksets first."""
    N = CONFIG_SIZES[k] if n_tasksets is None else int(n_tasksets)
    cores, per_core, S = CONFIG_SHAPES[k]
    idx = np.arange(first_index, first_index + N, dtype=np.int64)
    common = dict(n_cores=cores, tasks_per_core=per_core, max_gseg=S, seed=seed, stream=k, first_index=first_index)
    if k == 1:
        return N, dict(util=(0.4, 0.4), eta=(1, 1), share=(0.10, 0.30), period=(10_000, 100_000),
                       overhead=(200, 200), slice_us=1024, **common)
    if k == 2:
        util = (0.1 * (1 + (idx // 1000) % 9)).astype(np.float64)
        return N, dict(util=util, eta=(1, 3), share=(0.10, 0.50), period=(1_000, 500_000),
                       overhead=(200, 200), slice_us=1024, **common)
    if k == 3:
        return N, dict(util=(0.2, 0.8), eta=(1, 3), share=(0.10, 0.60), period=(1_000, 1_000_000),
                       overhead=(50, 500), slice_us=1024, **common)
    if k == 4:
        return N, dict(util=(0.5, 0.9), eta=(1, 5), share=(0.20, 0.70), period=(500, 2_000_000),
                       overhead=(300, 300), slice_us=2048, **common)
    if k == 5:
        cell = np.array(_GRID5, dtype=np.float64)[idx % len(_GRID5)]
        return N, dict(util=np.ascontiguousarray(cell[:, 0]), eta=(1, 4),
                       share=np.ascontiguousarray(cell[:, 1]), period=(1_000, 1_000_000),
                       overhead=cell[:, 2].astype(np.uint32), slice_us=cell[:, 3].astype(np.uint32), **common)
    raise ValueError(f"unknown workload {k}")


def config(k, n_tasksets=None, *, first_index=0, seed=0, threads=None):
    """Workload k (1..5).  n_tasksets defaults to the workload's full size; first_index selects
    where in the workload's taskset sequence the batch starts (workload 5 is streamed in
    batches; its grid cell and workload 2's sweep point are functions of the taskset index)."""
    N, params = config_params(k, n_tasksets, first_index=first_index, seed=seed)
    return generate(N, threads=threads, **params)


# ---- the recipe of the paper's schedulability experiments (Sec. 6.1, Table 3) ---------------------
TABLE3 = dict(n_cpus=4, tasks_per_cpu=(3, 6), gpu_ratio=(0.4, 0.6), util=(0.4, 0.6), period=(30_000, 500_000),
              eta=(1, 3), g_over_c=(0.2, 2.0), gm_over_g=(0.1, 0.3), theta_us=200, eps_us=1000, slice_us=1024,
              be_ratio=0.0)


def table3(n_tasksets, *, seed=0, stream=300, first_index=0, threads=None, **overrides):
    """Tasksets drawn by the recipe of Sec. 6.1 with the ranges of Table 3 (any of them can be
    overridden by keyword, e.g. ``util=(0.5, 0.5)`` for one point of a sweep): tasks per CPU drawn
    per CPU, UUniFast per CPU, uniform periods, a share of GPU-using tasks, G/C and G^m/G ratios,
    rate-monotonic priorities, worst-fit-decreasing re-allocation to the CPUs.

    Tasksets differ in their number of tasks, a batch of the library does not: the result is a dict
    {n: (indices, batch)} with one batch per task count n, `indices` saying which of the generated
    tasksets (in generation order) the rows of the batch are.

    be_ratio > 0 (the last experiment of Sec. 6.1): round(be_ratio * n) tasks of every taskset, chosen
    at random, are best-effort tasks.  They run below every real-time task (their priorities are
    moved below, keeping their order) and have no deadline to test; each batch then also holds
    ``best_effort`` (uint8 [N, n], not part of the library's task model: see ``sweep.py`` for how
    the analyses treat such tasks)."""
    q = dict(TABLE3)
    unknown = set(overrides) - set(q)
    if unknown:
        raise ValueError(f"unknown Table 3 parameters: {sorted(unknown)}")
    q.update(overrides)
    N = int(n_tasksets)
    n_max, S = q["n_cpus"] * q["tasks_per_cpu"][1], q["eta"][1]
    count = np.zeros(N, np.uint32)
    out = dict(theta_us=np.empty(N, np.uint32), eps_us=np.empty(N, np.uint32), slice_us=np.empty(N, np.uint32),
               cpu_us=np.empty((N, n_max), np.uint32), period_us=np.empty((N, n_max), np.uint32),
               deadline_us=np.empty((N, n_max), np.uint32), prio=np.empty((N, n_max), np.int32),
               core=np.empty((N, n_max), np.uint8), n_gseg=np.empty((N, n_max), np.uint8),
               gm_us=np.empty((N, n_max, S), np.uint32), ge_us=np.empty((N, n_max, S), np.uint32))
    if threads is None:
        threads = min(16, os.cpu_count() or 1)
    rc = _load().taskgen_table3(seed, stream, first_index, N, q["n_cpus"], q["tasks_per_cpu"][0], q["tasks_per_cpu"][1],
                                S, float(q["gpu_ratio"][0]), float(q["gpu_ratio"][1]), float(q["util"][0]),
                                float(q["util"][1]), q["period"][0], q["period"][1], q["eta"][0], q["eta"][1],
                                float(q["g_over_c"][0]), float(q["g_over_c"][1]), float(q["gm_over_g"][0]),
                                float(q["gm_over_g"][1]), q["theta_us"], q["eps_us"], q["slice_us"], threads,
                                _ptr(count), *[_ptr(out[k]) for k in ("theta_us", "eps_us", "slice_us", "cpu_us",
                                                                      "period_us", "deadline_us", "prio", "core",
                                                                      "n_gseg", "gm_us", "ge_us")])
    if rc != 0:
        raise ValueError("taskgen: invalid Table 3 parameters")
    be = float(q["be_ratio"])
    if not 0.0 <= be <= 1.0:
        raise ValueError("be_ratio must be within [0, 1]")
    groups = {}
    for n in np.unique(count):
        idx = np.flatnonzero(count == n)
        n = int(n)
        batch = {k: np.ascontiguousarray(v[idx] if v.ndim == 1 else v[idx, :n]) for k, v in out.items()}
        if be > 0.0:
            rng = np.random.default_rng([seed, stream, 7, n])
            order = np.argsort(rng.random((len(idx), n)), axis=1)
            chosen = np.zeros((len(idx), n), bool)
            np.put_along_axis(chosen, order[:, :int(np.floor(be * n + 0.5))], True, axis=1)
            batch["best_effort"] = chosen.astype(np.uint8)
            batch["prio"] = np.where(chosen, batch["prio"] - n, batch["prio"]).astype(np.int32)
        groups[n] = (idx, batch)
    return groups


def without_tasks(batch, drop):
    """The batch with the tasks marked in `drop` (bool [N, n], the same number per taskset) removed."""
    N, n = batch["cpu_us"].shape
    keep = ~np.asarray(drop, bool)
    m = int(keep[0].sum())
    assert (keep.sum(axis=1) == m).all()
    sel = np.argsort(~keep, axis=1, kind="stable")[:, :m]  # kept tasks in their order
    out = {}
    for k, v in batch.items():
        if v.ndim == 1:
            out[k] = v
        elif v.ndim == 2:
            out[k] = np.ascontiguousarray(np.take_along_axis(v, sel, axis=1))
        else:
            out[k] = np.ascontiguousarray(np.take_along_axis(v, sel[:, :, None], axis=1))
    return out
