"""Tasksets generated on the device (gcaps_taskgen_device): the host generator's batches, bit for bit (same
random streams, same sequence of IEEE double operations, the same logarithm and power routines on both
sides).  Results of the library on a device-generated batch equal the oracle's on the host-generated one."""
import numpy as np
import pytest

from test_gpu_parity import gpu  # noqa: F401 (fixture)

pytestmark = pytest.mark.gpu

BOTH, BUSY, SUSPEND = 3, 0, 1


@pytest.mark.parametrize("k,N,first", [(1, 1000, 0), (2, 9000, 0), (3, 200_000, 300_000), (4, 20_000, 7),
                                       (5, 216_000, 1_000_000)])
def test_same_batches_as_the_host_generator(gpu, k, N, first):
    import torch
    from paper_2406_05221_amd import taskgen
    B, ctx, stream = gpu
    _, params = taskgen.config_params(k, N, first_index=first)
    with torch.cuda.stream(stream):
        d = B.gcaps_taskgen_device(ctx, N, **params)
    stream.synchronize()
    dev = B.to_host(d)
    host = taskgen.generate(N, **params)
    for name in dev:
        assert np.array_equal(dev[name], host[name]), name
    # the task model holds on the device batch
    eta = dev["n_gseg"]
    assert (dev["cpu_us"] >= 1).all() and (dev["period_us"] >= params["period"][0]).all()
    assert (dev["period_us"] <= params["period"][1]).all()
    assert (eta >= params["eta"][0]).all() and (eta <= params["eta"][1]).all()
    S = dev["gm_us"].shape[2]
    unused = np.arange(S)[None, None, :] >= eta[:, :, None]
    assert (dev["gm_us"][unused] == 0).all() and (dev["ge_us"][unused] == 0).all()
    used = ~unused
    assert (dev["ge_us"][used] >= 1).all()
    n = dev["prio"].shape[1]
    assert (np.sort(dev["prio"], axis=1) == np.arange(1, n + 1)).all()
    order = np.argsort(-dev["prio"], axis=1)
    assert (np.diff(np.take_along_axis(dev["period_us"].astype(np.int64), order, 1), axis=1) >= 0).all()


def test_regenerated_in_pieces_and_analysed_where_it_is(oracle, gpu):
    """A batch generated in two calls equals the batch generated in one (the random stream belongs to the taskset
    index); the analyses of the library on the device batch equal the oracle on its copy."""
    import torch
    from paper_2406_05221_amd import taskgen
    B, ctx, stream = gpu
    N = 6_000
    _, params = taskgen.config_params(3, N, first_index=500)
    with torch.cuda.stream(stream):
        whole = B.gcaps_taskgen_device(ctx, N, **params)
        _, p1 = taskgen.config_params(3, 2_500, first_index=500)
        _, p2 = taskgen.config_params(3, 3_500, first_index=3_000)
        a = B.gcaps_taskgen_device(ctx, 2_500, **p1)
        b = B.gcaps_taskgen_device(ctx, 3_500, **p2)
        n = whole["cpu_us"].shape[1]
        d_resp = torch.empty((2, N, n), dtype=torch.int64, device="cuda:0")
        d_sched = torch.empty((2, N), dtype=torch.uint8, device="cuda:0")
        B.gcaps_rta_batch_device(ctx, whole, BOTH, SUSPEND, d_resp, d_sched)
        B.gcaps_status(ctx)
    stream.synchronize()
    for name in whole:
        assert torch.equal(whole[name], torch.cat([a[name], b[name]])), name
    host = B.to_host(whole)
    want_r, want_s, _ = oracle.rta_batch(host, BOTH, SUSPEND, threads=16)
    assert (d_resp.cpu().numpy() == want_r).all() and (d_sched.cpu().numpy() == want_s).all()
    again = B.gcaps_taskgen_device(ctx, N, out=whole, **params)
    stream.synchronize()
    assert all((B.to_host(again)[k] == host[k]).all() for k in host)


def test_relaxed_recipes_and_cpu_only_tasks_match_too(oracle, gpu):
    """Ranges other than the named workloads', CPU-only tasks (eta = 0: the whole demand stays CPU time), 80 tasks,
    one core, a period range of two values (ties in the rate-monotonic order), periods on both sides of 2^24 (the
    generator ranks smaller ones by packed keys)."""
    import torch
    from paper_2406_05221_amd import taskgen
    B, ctx, stream = gpu
    for N, kw in ((30_011, dict(n_cores=4, tasks_per_core=5, max_gseg=3, util=(0.25, 0.85), eta=(0, 3), share=(0.05, 0.5),
                                period=(20_000, 1_000_000), overhead=(0, 40), slice_us=1024, seed=3, stream=1000)),
                  (2_003, dict(n_cores=8, tasks_per_core=10, max_gseg=5, util=(0.1, 0.6), eta=(0, 5), share=(0.2, 0.7),
                               period=(500, 2_000_000), overhead=(300, 300), slice_us=2048, seed=4, stream=5)),
                  (1_501, dict(n_cores=2, tasks_per_core=6, max_gseg=2, util=(0.2, 0.7), eta=(0, 2), share=(0.1, 0.6),
                               period=(16_000_000, 40_000_000), overhead=(10, 20), slice_us=512, seed=6, stream=7)),
                  (777, dict(n_cores=1, tasks_per_core=9, max_gseg=1, util=(0.5, 0.99), eta=(1, 1), share=(0.1, 0.2),
                             period=(1_000, 1_001), overhead=(0, 0), slice_us=64, seed=5, stream=6))):
        with torch.cuda.stream(stream):
            d = B.gcaps_taskgen_device(ctx, N, first_index=123_456_789, **kw)
        stream.synchronize()
        dev, host = B.to_host(d), taskgen.generate(N, first_index=123_456_789, **kw)
        for name in dev:
            assert np.array_equal(dev[name], host[name]), (name, kw["n_cores"])
    # CPU-only tasks keep their whole demand: the utilisation per core is what was asked for
    cpu_only = host["n_gseg"] == 0
    assert (host["gm_us"].sum(2)[cpu_only] == 0).all()


def test_one_lane_per_taskset_kernels_give_the_same_batches(monkeypatch):
    """GCAPS_GEN_KERNEL=taskset: the generator kernels with one lane per taskset (stores gathered through LDS, or
    word by word where a taskset's values do not fit), which serve shapes the one-lane-per-task kernel has no LDS for."""
    import torch
    from paper_2406_05221_amd import binding as B, taskgen
    monkeypatch.setenv("GCAPS_GEN_KERNEL", "taskset")
    stream = torch.cuda.Stream()
    ctx = B.gcaps_create(0, stream.cuda_stream)
    try:
        cases = [taskgen.config_params(k, N, first_index=first)[1] | dict(N=N)
                 for k, N, first in ((2, 9000, 0), (3, 50_000, 300_000), (4, 5_000, 7), (5, 21_600, 1_000_000))]
        cases.append(dict(N=3_001, n_cores=4, tasks_per_core=5, max_gseg=3, util=(0.25, 0.85), eta=(0, 3), share=(0.05, 0.5),
                          period=(20_000, 1_000_000), overhead=(0, 40), slice_us=1024, seed=3, stream=1000))
        for kw in cases:
            N = kw.pop("N")
            with torch.cuda.stream(stream):
                d = B.gcaps_taskgen_device(ctx, N, **kw)
            stream.synchronize()
            dev, host = B.to_host(d), taskgen.generate(N, **kw)
            for name in dev:
                assert np.array_equal(dev[name], host[name]), (name, kw["n_cores"])
    finally:
        B.gcaps_destroy(ctx)


def test_invalid_arguments(gpu):
    from paper_2406_05221_amd import taskgen
    B, ctx, _ = gpu
    _, params = taskgen.config_params(1, 64)
    for change in (dict(eta=(1, 2)), dict(period=(0, 10)), dict(period=(10, 5)), dict(overhead=(5, 1)),
                   dict(util=(0.5, 0.4)), dict(slice_us=0)):
        with pytest.raises(B.GcapsError) as e:
            B.gcaps_taskgen_device(ctx, 64, **{**params, **change})
        assert e.value.code == B.GCAPS_EINVAL
