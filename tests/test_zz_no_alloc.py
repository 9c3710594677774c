"""gcaps_rta_batch_device_static (the entry point that allocates nothing: its launches work in a
fixed device array of the library) against gcaps_rta_batch_device, through the C ABI, bit for bit;
two calls in a row, the second with a smaller input, in a fresh context that has made no other call."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

BOTH, BUSY, SUSPEND = 3, 0, 1


def mixed_batch(N, seed):
    """Mostly schedulable tasksets (both fast launches take part) with one in seven scaled beyond the
    24-bit range (the 64-bit kernel and its scratch columns take part)."""
    from paper_2406_05221_amd import taskgen
    rng = np.random.default_rng(seed)
    b = taskgen.generate(N, n_cores=4, tasks_per_core=5, max_gseg=3, util=(0.25, 0.85), eta=(0, 3),
                         share=(0.05, 0.5), period=(20_000, 1_000_000), overhead=(0, 40), slice_us=1024,
                         seed=seed, stream=79)
    scale = rng.choice([1, 1, 1, 1, 1, 1, 3000], size=(N, 1)).astype(np.uint64)
    for key in ("cpu_us", "period_us", "deadline_us"):
        b[key] = np.minimum(b[key].astype(np.uint64) * scale, 2**32 - 1).astype(np.uint32)
    for key in ("gm_us", "ge_us"):
        b[key] = np.minimum(b[key].astype(np.uint64) * scale[:, :, None], 2**32 - 1).astype(np.uint32)
    return b


def run(B, ctx, torch, batch, wait, static):
    N, n = batch["cpu_us"].shape
    d = B.to_device(batch)
    resp = torch.full((2, N, n), -77, dtype=torch.int64, device="cuda:0")
    sched = torch.full((2, N), 77, dtype=torch.uint8, device="cuda:0")
    torch.cuda.synchronize()
    B.gcaps_rta_batch_device(ctx, d, BOTH, wait, resp, sched, static=static)
    B.gcaps_status(ctx)
    return resp.cpu().numpy(), sched.cpu().numpy(), B.gcaps_last_wide_count(ctx)


def test_static_scratch_calls_match_the_allocating_entry_point():
    import torch
    assert torch.cuda.is_available(), "this test needs the MI355X"
    from paper_2406_05221_amd import binding as B
    stream = torch.cuda.Stream()
    ref_ctx = B.gcaps_create(0, stream.cuda_stream)
    ctx = B.gcaps_create(0, stream.cuda_stream)  # makes static calls only
    try:
        # first a large call, then a smaller one: the second runs over what the first left in the array
        for N, seed in ((40_003, 1), (1_037, 2)):
            batch = mixed_batch(N, seed)
            for wait in (BUSY, SUSPEND):
                print(f"static call N={N} wait={wait}", flush=True)
                want = run(B, ref_ctx, torch, batch, wait, static=False)
                got = run(B, ctx, torch, batch, wait, static=True)
                assert want[2] > N // 20 and got[2] == want[2]  # the 64-bit kernel took its share in both
                assert np.array_equal(got[0], want[0]) and np.array_equal(got[1], want[1])
                assert want[1][0].sum() > N // 10  # schedulable under GCAPS: the second launch took part
        # the same context may mix both entry points; a direct call afterwards is not disturbed
        batch = mixed_batch(5_000, 3)
        a = run(B, ctx, torch, batch, SUSPEND, static=False)
        b = run(B, ctx, torch, batch, SUSPEND, static=True)
        c = run(B, ctx, torch, batch, SUSPEND, static=False)
        assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
        assert np.array_equal(a[0], c[0]) and np.array_equal(a[1], c[1])
        # an invalid taskset is reported by gcaps_status as after the allocating call
        bad = {k: v.copy() for k, v in batch.items()}
        bad["period_us"][4_321, 7] = 0
        d = B.to_device(bad)
        resp = torch.empty((2, 5_000, 20), dtype=torch.int64, device="cuda:0")
        sched = torch.empty((2, 5_000), dtype=torch.uint8, device="cuda:0")
        B.gcaps_rta_batch_device(ctx, d, BOTH, BUSY, resp, sched, static=True)
        with pytest.raises(B.GcapsError) as e:
            B.gcaps_status(ctx)
        assert e.value.code == B.GCAPS_ETASK and e.value.first_bad == 4_321
        # beyond the limits: refused with the size error, nothing queued
        for N, cores in ((65_537, 1), (8, 33)):
            from paper_2406_05221_amd import taskgen
            big = taskgen.generate(N, n_cores=cores, tasks_per_core=1, max_gseg=1, util=(0.1, 0.2), eta=(0, 1),
                                   share=(0.1, 0.2), period=(20_000, 100_000), overhead=(0, 40), slice_us=1024,
                                   seed=1, stream=80)
            d = B.to_device(big)
            resp = torch.empty((2, N, cores), dtype=torch.int64, device="cuda:0")
            sched = torch.empty((2, N), dtype=torch.uint8, device="cuda:0")
            with pytest.raises(B.GcapsError) as e:
                B.gcaps_rta_batch_device(ctx, d, BOTH, BUSY, resp, sched, static=True)
            assert e.value.code == B.GCAPS_ESIZE
        # at the limits: accepted
        edge = mixed_batch(65_536, 5)
        got = run(B, ctx, torch, edge, BUSY, static=True)
        want = run(B, ref_ctx, torch, edge, BUSY, static=False)
        assert np.array_equal(got[0], want[0]) and np.array_equal(got[1], want[1])
    finally:
        B.gcaps_destroy(ctx)
        B.gcaps_destroy(ref_ctx)
