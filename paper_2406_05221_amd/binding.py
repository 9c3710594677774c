"""Thin ctypes binding of the C ABI in include/gcaps_rta.h.

Argument marshalling only: every step of the analysis runs in the HIP kernels of
``libgcaps_rta.so``.  There is no CPU fallback; if the library has not been built
the import of this module fails.  Device memory and streams come from PyTorch.
"""
import ctypes
import os

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
# GCAPS_RTA_LIBRARY: another build of the same sources (e.g. with other tuning macros) instead of the in-tree one
LIB_PATH = os.environ.get("GCAPS_RTA_LIBRARY") or os.path.join(_PKG, "libgcaps_rta.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -c 'import __graft_entry__ as g; g.build()'` "
                      "(hipcc --offload-arch=gfx950); there is no fallback path")

_lib = ctypes.CDLL(LIB_PATH)

GCAPS_POLICY_GCAPS, GCAPS_POLICY_RR, GCAPS_POLICY_BOTH = 1, 2, 3
GCAPS_WAIT_BUSY, GCAPS_WAIT_SUSPEND = 0, 1
GCAPS_OK, GCAPS_EINVAL, GCAPS_ETASK, GCAPS_ENOMEM, GCAPS_EDEVICE, GCAPS_ESIZE = 0, -1, -2, -3, -4, -5
GCAPS_RESP_MISS, GCAPS_RESP_NOT_ANALYSED = -1, -2

EXPORTS = ["gcaps_create", "gcaps_destroy", "gcaps_rta_batch", "gcaps_rta_batch_device", "gcaps_status",
           "gcaps_last_wide_count", "gcaps_set_binning", "gcaps_strerror", "gcaps_gprio_assign_batch",
           "gcaps_gprio_assign_batch_device", "gcaps_set_continue_after_miss", "gcaps_gprio_rta_batch",
           "gcaps_gprio_rta_batch_device", "gcaps_simulate_batch", "gcaps_simulate_batch_device",
           "gcaps_last_sim_steps", "gcaps_taskgen_device", "gcaps_rta_batch_device_static", "gcaps_valu_probe", "gcaps_hbm_probe",
           "gcaps_table3_count_device", "gcaps_table3_generate_device"]

_p, _u32, _int = ctypes.c_void_p, ctypes.c_uint32, ctypes.c_int


class gcaps_batch(ctypes.Structure):
    _fields_ = [("n_tasksets", _u32), ("n_tasks", _u32), ("max_gseg", _u32),
                ("theta_us", _p), ("eps_us", _p), ("slice_us", _p),
                ("cpu_us", _p), ("n_cseg", _p), ("period_us", _p), ("deadline_us", _p), ("prio", _p),
                ("core", _p), ("n_gseg", _p), ("gm_us", _p), ("ge_us", _p)]


_lib.gcaps_create.restype = _int
_lib.gcaps_create.argtypes = [ctypes.POINTER(_p), _int, _p]
_lib.gcaps_destroy.restype = None
_lib.gcaps_destroy.argtypes = [_p]
_lib.gcaps_rta_batch.restype = _int
_lib.gcaps_rta_batch.argtypes = [_p, ctypes.POINTER(gcaps_batch), _int, _int, _p, _p, ctypes.POINTER(_u32)]
_lib.gcaps_rta_batch_device.restype = _int
_lib.gcaps_rta_batch_device.argtypes = [_p, ctypes.POINTER(gcaps_batch), _int, _int, _p, _p]
_lib.gcaps_rta_batch_device_static.restype = _int
_lib.gcaps_rta_batch_device_static.argtypes = [_p, ctypes.POINTER(gcaps_batch), _int, _int, _p, _p]
_lib.gcaps_status.restype = _int
_lib.gcaps_status.argtypes = [_p, ctypes.POINTER(_u32)]
_lib.gcaps_last_wide_count.restype = _int
_lib.gcaps_last_wide_count.argtypes = [_p, ctypes.POINTER(_u32)]
_lib.gcaps_set_binning.restype = _int
_lib.gcaps_set_binning.argtypes = [_p, _int]
_lib.gcaps_gprio_assign_batch.restype = _int
_lib.gcaps_gprio_assign_batch.argtypes = [_p, ctypes.POINTER(gcaps_batch), _int, _p, _p, _p, _p, ctypes.POINTER(_u32)]
_lib.gcaps_gprio_assign_batch_device.restype = _int
_lib.gcaps_gprio_assign_batch_device.argtypes = [_p, ctypes.POINTER(gcaps_batch), _int, _p, _p, _p, _p]
_lib.gcaps_gprio_rta_batch.restype = _int
_lib.gcaps_gprio_rta_batch.argtypes = [_p, ctypes.POINTER(gcaps_batch), _int, _p, _p, _p, ctypes.POINTER(_u32)]
_lib.gcaps_gprio_rta_batch_device.restype = _int
_lib.gcaps_gprio_rta_batch_device.argtypes = [_p, ctypes.POINTER(gcaps_batch), _int, _p, _p, _p]
_lib.gcaps_set_continue_after_miss.restype = _int
_lib.gcaps_set_continue_after_miss.argtypes = [_p, _int]
_lib.gcaps_strerror.restype = ctypes.c_char_p
_lib.gcaps_strerror.argtypes = [_int]

PROBE_KINDS = ["add_u32", "mad_u32_u24", "mul_hi_u32_u24", "mul_lo_u32", "mul_hi_u32", "lshrrev_b32", "min_u32",
               "term", "cndmask_sgpr", "cmp_cndmask"]


class gcaps_valu_rates(ctypes.Structure):
    _fields_ = [("cu_count", _int), ("clock_khz", _int), ("wavefront_size", _int), ("simd_per_cu", _int),
                ("spec_lane_ops_per_s", ctypes.c_double), ("lane_ops_per_s", ctypes.c_double * len(PROBE_KINDS))]


_lib.gcaps_valu_probe.restype = _int
_lib.gcaps_valu_probe.argtypes = [_p, ctypes.POINTER(gcaps_valu_rates)]

HBM_KINDS = ["copy", "copy_stream", "read", "read_stream", "write", "write_stream"]


class gcaps_hbm_rates(ctypes.Structure):
    _fields_ = [("bytes", ctypes.c_size_t), ("bytes_per_s", ctypes.c_double * len(HBM_KINDS))]


_lib.gcaps_hbm_probe.restype = _int
_lib.gcaps_hbm_probe.argtypes = [_p, ctypes.c_size_t, ctypes.POINTER(gcaps_hbm_rates)]

_FIELDS = [("theta_us", np.uint32, 1), ("eps_us", np.uint32, 1), ("slice_us", np.uint32, 1),
           ("cpu_us", np.uint32, 2), ("period_us", np.uint32, 2), ("deadline_us", np.uint32, 2),
           ("prio", np.int32, 2), ("core", np.uint8, 2), ("n_gseg", np.uint8, 2),
           ("gm_us", np.uint32, 3), ("ge_us", np.uint32, 3)]


class GcapsError(RuntimeError):
    def __init__(self, code, first_bad=None):
        msg = _lib.gcaps_strerror(code).decode()
        if first_bad is not None:
            msg += f" (first invalid taskset: {first_bad})"
        super().__init__(msg)
        self.code = code
        self.first_bad = first_bad


def gcaps_strerror(code):
    return _lib.gcaps_strerror(code).decode()


def npol(policy):
    return bin(policy & 3).count("1")


def gcaps_create(device_id=0, hip_stream=None):
    """Returns an opaque context handle.  hip_stream: integer hipStream_t (e.g.
    ``torch.cuda.Stream().cuda_stream``) or None for the default stream."""
    h = _p()
    rc = _lib.gcaps_create(ctypes.byref(h), device_id, _p(hip_stream) if hip_stream else None)
    if rc != GCAPS_OK:
        raise GcapsError(rc)
    return h


def gcaps_destroy(ctx):
    _lib.gcaps_destroy(ctx)


def gcaps_set_binning(ctx, enable):
    rc = _lib.gcaps_set_binning(ctx, int(enable))
    if rc != GCAPS_OK:
        raise GcapsError(rc)


def gcaps_set_continue_after_miss(ctx, enable):
    rc = _lib.gcaps_set_continue_after_miss(ctx, int(enable))
    if rc != GCAPS_OK:
        raise GcapsError(rc)


def _shape(batch):
    N, n = batch["cpu_us"].shape
    S = batch["gm_us"].shape[2] if batch["gm_us"].ndim == 3 else 0
    return int(N), int(n), int(S)


def gcaps_rta_batch(ctx, batch, policy, wait_mode):
    """Host entry point.  batch: dict of numpy arrays (see ``taskgen``).  Returns
    (resp int64 [npol, N, n], sched uint8 [npol, N])."""
    N, n, S = _shape(batch)
    keep = {}
    b = gcaps_batch(n_tasksets=N, n_tasks=n, max_gseg=S)
    for name, dtype, ndim in _FIELDS:
        a = np.ascontiguousarray(batch[name], dtype=dtype)
        assert a.ndim == ndim and a.shape[0] == N, name
        keep[name] = a
        setattr(b, name, a.ctypes.data if a.size else None)
    P = npol(policy)
    resp = np.empty((P, N, n), np.int64)
    sched = np.empty((P, N), np.uint8)
    bad = _u32(0xFFFFFFFF)
    rc = _lib.gcaps_rta_batch(ctx, ctypes.byref(b), policy, wait_mode, resp.ctypes.data, sched.ctypes.data,
                              ctypes.byref(bad))
    if rc != GCAPS_OK:
        raise GcapsError(rc, bad.value if rc == GCAPS_ETASK else None)
    return resp, sched


def to_device(batch, device="cuda:0"):
    """Copies a numpy batch into torch device tensors (memory plumbing only)."""
    import torch

    out = {}
    for name, dtype, _ in _FIELDS:
        a = np.ascontiguousarray(batch[name], dtype=dtype)
        t = torch.from_numpy(a.view(np.int32) if dtype == np.uint32 else a)
        out[name] = t.to(device)
    return out


def gcaps_rta_batch_device(ctx, dbatch, policy, wait_mode, d_resp, d_sched, static=False):
    """Device entry point.  dbatch: dict of torch device tensors with the batch layout;
    d_resp: int64 [npol, N, n], d_sched: uint8 [npol, N] device tensors.  Queues the work
    on the context's stream and returns; call ``gcaps_status`` to wait and check.
    static: call ``gcaps_rta_batch_device_static`` (no device allocation, bounded sizes)."""
    N, n = dbatch["cpu_us"].shape
    S = dbatch["gm_us"].shape[2] if dbatch["gm_us"].dim() == 3 else 0
    b = gcaps_batch(n_tasksets=int(N), n_tasks=int(n), max_gseg=int(S))
    for name, _, _ in _FIELDS:
        t = dbatch[name]
        assert t.is_cuda and t.is_contiguous(), name
        setattr(b, name, t.data_ptr() if t.numel() else None)
    P = npol(policy)
    assert d_resp.is_cuda and d_resp.is_contiguous() and d_resp.numel() == P * N * n and d_resp.element_size() == 8
    assert d_sched.is_cuda and d_sched.is_contiguous() and d_sched.numel() == P * N and d_sched.element_size() == 1
    fn = _lib.gcaps_rta_batch_device_static if static else _lib.gcaps_rta_batch_device
    rc = fn(ctx, ctypes.byref(b), policy, wait_mode, d_resp.data_ptr(), d_sched.data_ptr())
    if rc != GCAPS_OK:
        raise GcapsError(rc)


def gcaps_rta_batch_device_static(ctx, dbatch, policy, wait_mode, d_resp, d_sched):
    """``gcaps_rta_batch_device`` in the library's fixed scratch array: allocates nothing."""
    gcaps_rta_batch_device(ctx, dbatch, policy, wait_mode, d_resp, d_sched, static=True)


def gcaps_valu_probe(ctx):
    """Measured integer VALU rates of the device: dict with cu_count, clock_khz, wavefront_size,
    simd_per_cu, spec_lane_ops_per_s and lane_ops_per_s (by instruction kind)."""
    r = gcaps_valu_rates()
    rc = _lib.gcaps_valu_probe(ctx, ctypes.byref(r))
    if rc != GCAPS_OK:
        raise GcapsError(rc)
    return dict(cu_count=r.cu_count, clock_khz=r.clock_khz, wavefront_size=r.wavefront_size,
                simd_per_cu=r.simd_per_cu, spec_lane_ops_per_s=r.spec_lane_ops_per_s,
                lane_ops_per_s={k: r.lane_ops_per_s[i] for i, k in enumerate(PROBE_KINDS)})


def gcaps_hbm_probe(ctx, nbytes=1 << 30):
    """Measured HBM rates of the device: dict of bytes moved per second by kind (copy, read, write; plain or
    with the non-temporal hint) over buffers of ``nbytes``."""
    r = gcaps_hbm_rates()
    rc = _lib.gcaps_hbm_probe(ctx, nbytes, ctypes.byref(r))
    if rc != GCAPS_OK:
        raise GcapsError(rc)
    return {k: r.bytes_per_s[i] for i, k in enumerate(HBM_KINDS)}


def gcaps_status(ctx):
    bad = _u32(0xFFFFFFFF)
    rc = _lib.gcaps_status(ctx, ctypes.byref(bad))
    if rc != GCAPS_OK:
        raise GcapsError(rc, bad.value if rc == GCAPS_ETASK else None)


def gcaps_last_wide_count(ctx):
    c = _u32(0)
    rc = _lib.gcaps_last_wide_count(ctx, ctypes.byref(c))
    if rc != GCAPS_OK:
        raise GcapsError(rc)
    return c.value


def gcaps_gprio_assign_batch(ctx, batch, wait_mode, skip=None):
    """Host entry point of the GPU-segment priority assignment.  batch: dict of numpy arrays;
    skip: uint8 [N] or None.  Returns (gprio int32 [N, n], resp int64 [N, n], sched uint8 [N])."""
    N, n, S = _shape(batch)
    keep = {}
    b = gcaps_batch(n_tasksets=N, n_tasks=n, max_gseg=S)
    for name, dtype, ndim in _FIELDS:
        a = np.ascontiguousarray(batch[name], dtype=dtype)
        assert a.ndim == ndim and a.shape[0] == N, name
        keep[name] = a
        setattr(b, name, a.ctypes.data if a.size else None)
    sk = None if skip is None else np.ascontiguousarray(skip, dtype=np.uint8)
    assert sk is None or sk.shape == (N,)
    gprio = np.empty((N, n), np.int32)
    resp = np.empty((N, n), np.int64)
    sched = np.empty(N, np.uint8)
    bad = _u32(0xFFFFFFFF)
    rc = _lib.gcaps_gprio_assign_batch(ctx, ctypes.byref(b), wait_mode, sk.ctypes.data if sk is not None else None,
                                       gprio.ctypes.data, resp.ctypes.data, sched.ctypes.data, ctypes.byref(bad))
    if rc != GCAPS_OK:
        raise GcapsError(rc, bad.value if rc == GCAPS_ETASK else None)
    return gprio, resp, sched


def gcaps_gprio_assign_batch_device(ctx, dbatch, wait_mode, d_skip, d_gprio, d_resp, d_sched):
    """Device entry point of the GPU-segment priority assignment.  dbatch as for
    ``gcaps_rta_batch_device``; d_skip: uint8 [N] device tensor or None; d_gprio: int32 [N, n],
    d_resp: int64 [N, n], d_sched: uint8 [N] device tensors.  Queues the work and returns."""
    N, n = dbatch["cpu_us"].shape
    S = dbatch["gm_us"].shape[2] if dbatch["gm_us"].dim() == 3 else 0
    b = gcaps_batch(n_tasksets=int(N), n_tasks=int(n), max_gseg=int(S))
    for name, _, _ in _FIELDS:
        t = dbatch[name]
        assert t.is_cuda and t.is_contiguous(), name
        setattr(b, name, t.data_ptr() if t.numel() else None)
    for t, count, size in ((d_gprio, N * n, 4), (d_resp, N * n, 8), (d_sched, N, 1)):
        assert t.is_cuda and t.is_contiguous() and t.numel() == count and t.element_size() == size
    if d_skip is not None:
        assert d_skip.is_cuda and d_skip.is_contiguous() and d_skip.numel() == N and d_skip.element_size() == 1
    rc = _lib.gcaps_gprio_assign_batch_device(ctx, ctypes.byref(b), wait_mode,
                                              d_skip.data_ptr() if d_skip is not None else None,
                                              d_gprio.data_ptr(), d_resp.data_ptr(), d_sched.data_ptr())
    if rc != GCAPS_OK:
        raise GcapsError(rc)


def gcaps_gprio_rta_batch(ctx, batch, wait_mode, gprio):
    """Host entry point of the analysis for given GPU-segment priorities (int32 [N, n]).
    Returns (resp int64 [N, n], sched uint8 [N])."""
    N, n, S = _shape(batch)
    keep = {}
    b = gcaps_batch(n_tasksets=N, n_tasks=n, max_gseg=S)
    for name, dtype, ndim in _FIELDS:
        a = np.ascontiguousarray(batch[name], dtype=dtype)
        assert a.ndim == ndim and a.shape[0] == N, name
        keep[name] = a
        setattr(b, name, a.ctypes.data if a.size else None)
    gp = np.ascontiguousarray(gprio, dtype=np.int32)
    assert gp.shape == (N, n)
    resp = np.empty((N, n), np.int64)
    sched = np.empty(N, np.uint8)
    bad = _u32(0xFFFFFFFF)
    rc = _lib.gcaps_gprio_rta_batch(ctx, ctypes.byref(b), wait_mode, gp.ctypes.data, resp.ctypes.data,
                                    sched.ctypes.data, ctypes.byref(bad))
    if rc != GCAPS_OK:
        raise GcapsError(rc, bad.value if rc == GCAPS_ETASK else None)
    return resp, sched


def gcaps_gprio_rta_batch_device(ctx, dbatch, wait_mode, d_gprio, d_resp, d_sched):
    """Device entry point of the analysis for given GPU-segment priorities."""
    N, n = dbatch["cpu_us"].shape
    S = dbatch["gm_us"].shape[2] if dbatch["gm_us"].dim() == 3 else 0
    b = gcaps_batch(n_tasksets=int(N), n_tasks=int(n), max_gseg=int(S))
    for name, _, _ in _FIELDS:
        t = dbatch[name]
        assert t.is_cuda and t.is_contiguous(), name
        setattr(b, name, t.data_ptr() if t.numel() else None)
    for t, count, size in ((d_gprio, N * n, 4), (d_resp, N * n, 8), (d_sched, N, 1)):
        assert t.is_cuda and t.is_contiguous() and t.numel() == count and t.element_size() == size
    rc = _lib.gcaps_gprio_rta_batch_device(ctx, ctypes.byref(b), wait_mode, d_gprio.data_ptr(), d_resp.data_ptr(),
                                           d_sched.data_ptr())
    if rc != GCAPS_OK:
        raise GcapsError(rc)


_lib.gcaps_simulate_batch.restype = _int
_lib.gcaps_simulate_batch.argtypes = [_p, ctypes.POINTER(gcaps_batch), _p, _p, _int, _int, _u32, _p, _p, _p,
                                      ctypes.POINTER(_u32)]
_lib.gcaps_simulate_batch_device.restype = _int
_lib.gcaps_simulate_batch_device.argtypes = [_p, ctypes.POINTER(gcaps_batch), _p, _p, _int, _int, _u32, _p, _p, _p]


def gcaps_simulate_batch(ctx, batch, policy, wait_mode, horizon, offset=None, gprio=None):
    """Host entry point of the schedule simulation.  offset: uint32 [N, n] first releases or None; gprio: int32
    [N, n] GPU-segment priorities or None (the task priorities).
    Returns (mort int64 [P, N, n], jobs uint32 [P, N, n], flag uint8 [P, N])."""
    N, n, S = _shape(batch)
    keep = {}
    b = gcaps_batch(n_tasksets=N, n_tasks=n, max_gseg=S)
    for name, dtype, ndim in _FIELDS:
        a = np.ascontiguousarray(batch[name], dtype=dtype)
        assert a.ndim == ndim and a.shape[0] == N, name
        keep[name] = a
        setattr(b, name, a.ctypes.data if a.size else None)
    off = None if offset is None else np.ascontiguousarray(offset, dtype=np.uint32)
    assert off is None or off.shape == (N, n)
    gp = None if gprio is None else np.ascontiguousarray(gprio, dtype=np.int32)
    assert gp is None or gp.shape == (N, n)
    P = 2 if policy == GCAPS_POLICY_BOTH else 1
    mort = np.empty((P, N, n), np.int64)
    jobs = np.empty((P, N, n), np.uint32)
    flag = np.empty((P, N), np.uint8)
    bad = _u32(0xFFFFFFFF)
    rc = _lib.gcaps_simulate_batch(ctx, ctypes.byref(b), None if off is None else off.ctypes.data,
                                   None if gp is None else gp.ctypes.data, policy, wait_mode,
                                   int(horizon), mort.ctypes.data, jobs.ctypes.data, flag.ctypes.data,
                                   ctypes.byref(bad))
    if rc != GCAPS_OK:
        raise GcapsError(rc, bad.value if rc == GCAPS_ETASK else None)
    return mort, jobs, flag


def gcaps_simulate_batch_device(ctx, dbatch, policy, wait_mode, horizon, d_mort, d_jobs, d_flag, d_offset=None,
                                d_gprio=None):
    """Device entry point of the schedule simulation (queued on the context's stream)."""
    N, n = dbatch["cpu_us"].shape
    S = dbatch["gm_us"].shape[2] if dbatch["gm_us"].dim() == 3 else 0
    b = gcaps_batch(n_tasksets=int(N), n_tasks=int(n), max_gseg=int(S))
    for name, _, _ in _FIELDS:
        t = dbatch[name]
        assert t.is_cuda and t.is_contiguous(), name
        setattr(b, name, t.data_ptr() if t.numel() else None)
    P = 2 if policy == GCAPS_POLICY_BOTH else 1
    for t, count, size in ((d_mort, P * N * n, 8), (d_jobs, P * N * n, 4), (d_flag, P * N, 1)):
        assert t.is_cuda and t.is_contiguous() and t.numel() == count and t.element_size() == size
    if d_offset is not None:
        assert d_offset.is_cuda and d_offset.is_contiguous() and d_offset.numel() == N * n
        assert d_offset.element_size() == 4
    if d_gprio is not None:
        assert d_gprio.is_cuda and d_gprio.is_contiguous() and d_gprio.numel() == N * n
        assert d_gprio.element_size() == 4
    rc = _lib.gcaps_simulate_batch_device(ctx, ctypes.byref(b), None if d_offset is None else d_offset.data_ptr(),
                                          None if d_gprio is None else d_gprio.data_ptr(), policy, wait_mode, int(horizon), d_mort.data_ptr(), d_jobs.data_ptr(),
                                          d_flag.data_ptr())
    if rc != GCAPS_OK:
        raise GcapsError(rc)


_lib.gcaps_last_sim_steps.restype = _int
_lib.gcaps_last_sim_steps.argtypes = [_p, ctypes.POINTER(ctypes.c_uint64)]


def gcaps_last_sim_steps(ctx):
    """Steps (jumps to the next event) taken by all lanes of the most recent simulation call."""
    c = ctypes.c_uint64(0)
    rc = _lib.gcaps_last_sim_steps(ctx, ctypes.byref(c))
    if rc != GCAPS_OK:
        raise GcapsError(rc)
    return c.value


class gcaps_taskgen_spec(ctypes.Structure):
    _fields_ = [("seed", ctypes.c_uint64), ("stream", ctypes.c_uint64), ("first_index", ctypes.c_uint64),
                ("n_cores", _u32), ("tasks_per_core", _u32), ("util_lo", ctypes.c_double), ("util_hi", ctypes.c_double),
                ("util_fixed", _p), ("eta_lo", _u32), ("eta_hi", _u32), ("share_lo", ctypes.c_double),
                ("share_hi", ctypes.c_double), ("share_fixed", _p), ("period_lo", _u32), ("period_hi", _u32),
                ("overhead_lo", _u32), ("overhead_hi", _u32), ("overhead_fixed", _p), ("slice_us", _u32),
                ("slice_fixed", _p)]


_lib.gcaps_taskgen_device.restype = _int
_lib.gcaps_taskgen_device.argtypes = [_p, ctypes.POINTER(gcaps_taskgen_spec), ctypes.POINTER(gcaps_batch)]


def gcaps_taskgen_device(ctx, n_tasksets, *, n_cores, tasks_per_core, max_gseg, util, eta, share, period, overhead,
                         slice_us, seed=0, stream=0, first_index=0, out=None, device="cuda:0", fixed=None):
    """Generates a batch on the device with the parameters of ``taskgen.generate`` (a numpy array [N] in place of
    a range fixes the value per taskset; it is copied to the device).  Returns the dict of torch device tensors
    that ``gcaps_rta_batch_device`` and the other device entry points take; `out` reuses the tensors of an
    earlier call of the same shape.  `fixed`: per-taskset values that are already on the device, as a dict of
    torch tensors [N] keyed util / share (float64), overhead / slice_us (uint32 bits in int32); the caller keeps them
    alive until the work has run.  The work is queued on the context's stream."""
    import torch
    N, n, S = int(n_tasksets), n_cores * tasks_per_core, int(max_gseg)
    if out is None:
        shapes = {1: (N,), 2: (N, n), 3: (N, n, S)}
        kinds = {np.uint32: torch.int32, np.int32: torch.int32, np.uint8: torch.uint8}  # uint32 bits in int32 tensors
        out = {name: torch.empty(shapes[ndim], dtype=kinds[dtype], device=device) for name, dtype, ndim in _FIELDS}
    b = gcaps_batch(n_tasksets=N, n_tasks=n, max_gseg=S)
    for name, _, _ in _FIELDS:
        t = out[name]
        assert t.is_cuda and t.is_contiguous(), name
        setattr(b, name, t.data_ptr() if t.numel() else None)
    keep = []

    fixed = fixed or {}

    def rng_or_fixed(x, dtype, key=None):
        if key in fixed:
            t = fixed[key]
            assert t.is_cuda and t.is_contiguous() and t.shape == (N,) and t.element_size() == np.dtype(dtype).itemsize
            return (0, 0), t.data_ptr()
        if isinstance(x, np.ndarray):
            a = np.ascontiguousarray(x, dtype=dtype)
            t = torch.from_numpy(a.view(np.int32) if dtype == np.uint32 else a).to(device)
            assert t.shape == (N,)
            keep.append(t)
            return (0, 0), t.data_ptr()
        return x, None

    (u_lo, u_hi), u_fix = rng_or_fixed(util, np.float64, "util")
    (s_lo, s_hi), s_fix = rng_or_fixed(share, np.float64, "share")
    (o_lo, o_hi), o_fix = rng_or_fixed(overhead, np.uint32, "overhead")
    if isinstance(slice_us, np.ndarray) or "slice_us" in fixed:
        (_, _), l_fix = rng_or_fixed(slice_us, np.uint32, "slice_us")
        l_val = 0
    else:
        l_fix, l_val = None, int(slice_us)
    spec = gcaps_taskgen_spec(seed=seed, stream=stream, first_index=first_index, n_cores=n_cores,
                              tasks_per_core=tasks_per_core, util_lo=float(u_lo), util_hi=float(u_hi), util_fixed=u_fix,
                              eta_lo=eta[0], eta_hi=eta[1], share_lo=float(s_lo), share_hi=float(s_hi),
                              share_fixed=s_fix, period_lo=period[0], period_hi=period[1], overhead_lo=int(o_lo),
                              overhead_hi=int(o_hi), overhead_fixed=o_fix, slice_us=l_val, slice_fixed=l_fix)
    rc = _lib.gcaps_taskgen_device(ctx, ctypes.byref(spec), ctypes.byref(b))
    if rc != GCAPS_OK:
        raise GcapsError(rc)
    if keep:
        torch.cuda.synchronize()  # the per-taskset arrays must outlive the kernel that reads them
    return out


class gcaps_table3_spec(ctypes.Structure):
    _fields_ = [("seed", ctypes.c_uint64), ("stream", ctypes.c_uint64), ("first_index", ctypes.c_uint64),
                ("n_cpus", _u32), ("per_cpu_lo", _u32), ("per_cpu_hi", _u32),
                ("gpu_ratio_lo", ctypes.c_double), ("gpu_ratio_hi", ctypes.c_double),
                ("util_lo", ctypes.c_double), ("util_hi", ctypes.c_double),
                ("period_lo", _u32), ("period_hi", _u32), ("eta_lo", _u32), ("eta_hi", _u32),
                ("gc_lo", ctypes.c_double), ("gc_hi", ctypes.c_double), ("gm_lo", ctypes.c_double),
                ("gm_hi", ctypes.c_double), ("theta_us", _u32), ("eps_us", _u32), ("slice_us", _u32)]


_lib.gcaps_table3_count_device.restype = _int
_lib.gcaps_table3_count_device.argtypes = [_p, ctypes.POINTER(gcaps_table3_spec), _u32, _p]
_lib.gcaps_table3_generate_device.restype = _int
_lib.gcaps_table3_generate_device.argtypes = [_p, ctypes.POINTER(gcaps_table3_spec), _p, ctypes.POINTER(gcaps_batch)]


def gcaps_table3_device(ctx, n_tasksets, *, seed=0, stream=300, first_index=0, device="cuda:0", **overrides):
    """The recipe of Sec. 6.1 / Table 3 generated on the device, with the parameters of ``taskgen.table3`` (any
    of ``taskgen.TABLE3`` can be overridden by keyword; best-effort tasks are not generated here).  Returns
    {n: (indices, batch)} like ``taskgen.table3``: one device batch per task count n, `indices` (int64 device
    tensor) saying which tasksets of the stream its rows are.  The tasksets are the host generator's, bit for bit.
    Tensor bookkeeping (grouping by count: one stable sort, one allocation per field shared by the groups) is done
    with torch on the device; one small copy of the group sizes comes back to the host."""
    import torch
    from . import taskgen
    q = dict(taskgen.TABLE3)
    unknown = set(overrides) - set(q)
    if unknown:
        raise ValueError(f"unknown Table 3 parameters: {sorted(unknown)}")
    q.update(overrides)
    if float(q["be_ratio"]) != 0.0:
        raise ValueError("best-effort tasks are added on the host (taskgen.table3)")
    N, S = int(n_tasksets), int(q["eta"][1])
    spec = gcaps_table3_spec(seed=seed, stream=stream, first_index=first_index, n_cpus=q["n_cpus"],
                             per_cpu_lo=q["tasks_per_cpu"][0], per_cpu_hi=q["tasks_per_cpu"][1],
                             gpu_ratio_lo=float(q["gpu_ratio"][0]), gpu_ratio_hi=float(q["gpu_ratio"][1]),
                             util_lo=float(q["util"][0]), util_hi=float(q["util"][1]), period_lo=q["period"][0],
                             period_hi=q["period"][1], eta_lo=q["eta"][0], eta_hi=q["eta"][1],
                             gc_lo=float(q["g_over_c"][0]), gc_hi=float(q["g_over_c"][1]),
                             gm_lo=float(q["gm_over_g"][0]), gm_hi=float(q["gm_over_g"][1]), theta_us=q["theta_us"],
                             eps_us=q["eps_us"], slice_us=q["slice_us"])
    count = torch.empty(N, dtype=torch.int32, device=device)
    rc = _lib.gcaps_table3_count_device(ctx, ctypes.byref(spec), N, count.data_ptr())
    if rc != GCAPS_OK:
        raise GcapsError(rc)
    gcaps_status(ctx)  # waits for the context's stream
    # one stable sort puts the tasksets of a count side by side, in stream order; one copy brings the sizes back
    order = torch.argsort(count, stable=True)
    order32 = order.to(torch.int32)
    sizes = torch.bincount(count).tolist()
    present = [(n, M) for n, M in enumerate(sizes) if M > 0]
    # every field of every group in one allocation per field, each group's part at a multiple of 256 bytes
    kinds = {np.uint32: torch.int32, np.int32: torch.int32, np.uint8: torch.uint8}  # uint32 bits in int32 tensors
    per_row = {1: lambda n: 1, 2: lambda n: n, 3: lambda n: n * S}

    def carve(dtype, ndim):
        step = 256 // torch.empty(0, dtype=dtype).element_size()
        starts, total = [], 0
        for n, M in present:
            starts.append(total)
            total += -(-(M * per_row[ndim](n)) // step) * step
        return torch.empty(total, dtype=dtype, device=device), starts

    flat = {name: carve(kinds[dtype], ndim) for name, dtype, ndim in _FIELDS}
    torch.cuda.current_stream().synchronize()  # the index lists were made on torch's stream
    groups, first = {}, 0
    for g, (n, M) in enumerate(present):
        shapes = {1: (M,), 2: (M, n), 3: (M, n, S)}
        batch = {}
        for name, _, ndim in _FIELDS:
            buf, starts = flat[name]
            batch[name] = buf[starts[g]:starts[g] + M * per_row[ndim](n)].view(shapes[ndim])
        b = gcaps_batch(n_tasksets=M, n_tasks=n, max_gseg=S)
        for name, _, _ in _FIELDS:
            setattr(b, name, batch[name].data_ptr() if batch[name].numel() else None)
        rc = _lib.gcaps_table3_generate_device(ctx, ctypes.byref(spec), order32[first:first + M].data_ptr(),
                                               ctypes.byref(b))
        if rc != GCAPS_OK:
            raise GcapsError(rc)
        groups[int(n)] = (order[first:first + M], batch)
        first += M
    gcaps_status(ctx)  # waits for the stream: the groups are written (their index lists come from the counts above)
    return groups


def to_host(dbatch):
    """The numpy form of a device batch (uint32 fields are kept in int32 tensors on the device)."""
    return {name: (dbatch[name].cpu().numpy().view(np.uint32) if dtype == np.uint32 else dbatch[name].cpu().numpy())
            for name, dtype, _ in _FIELDS}
