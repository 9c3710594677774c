#!/usr/bin/env python3
"""Benchmark of the batched response-time analysis on one MI355X.

One step = one pass of the whole hot path (task-model checks, priority ranking, per-task
aggregates, both response-time analyses, write-back) over one device-resident batch of
synthetic tasksets.  The default workload is the 1,000,000-taskset one (4 cores x 5 tasks,
1-3 GPU segments per task); both waiting modes are timed and the slower one is the headline.

Prints ONE JSON line (see the keys below).  `--gpus N` with N > 1 is refused: the path is
built and measured on one GPU.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0                      # MI355X HBM3E, published
# 32-bit integer lane-operations/s by the unit counts: CUs x SIMDs x lanes x clock = 39.3e12.  What the
# device sustains per instruction kind is measured by `--row peak` (profiles/int32_peak.md: add 1.36 x this
# figure, shifts 1.71 x, the 24-bit multiply-add 0.89 x, the 24-bit multiply-high 0.97 x, 32-bit multiplies
# 0.91-0.96 x: 24-bit and 32-bit multiplies run at the same rate; the four instructions of one interference
# term 1.13 x).  The rta rows run the probe themselves and report fractions against both.
VALU_PEAK_LANE_OPS = 256 * 4 * 16 * 2.4e9
OPS_PER_TERM = 6                           # add jitter, reciprocal ceil-div (~3), multiply-add, compare

# VALU work of one step as the hardware counted it, summed over the launches of a step: wavefront
# instructions (SQ_INSTS_VALU) and lane-operations (SQ_THREAD_CYCLES_VALU: one per active lane and
# instruction), per workload and waiting mode, 1,000,000 tasksets; valid for the kernel sources they were
# taken with (profiles/rta_step_workload3_counters.md, profiles/rta_step_workload0_counters.md).
MEASURED_VALU = dict(
    csrc_sha256="14f51d6b715949ec02784f7f42a74b41aaae5b685fc8af4c819906c05c366888", tasksets=1_000_000,
    per_workload={"3": dict(busy=dict(valu_wave_insts=59_609_954, valu_lane_ops=2_782_050_819),
                            suspend=dict(valu_wave_insts=65_539_242, valu_lane_ops=2_941_143_253)),
                  "0": dict(busy=dict(valu_wave_insts=386_276_643, valu_lane_ops=22_597_531_024),
                            suspend=dict(valu_wave_insts=590_321_854, valu_lane_ops=34_526_990_874))})

# HBM bytes of one default step (workload 3, both policies; mean of the two waiting modes), from
# rocprofv3 FETCH_SIZE / WRITE_SIZE summed over the launches of a step and scaled by what the same
# counters read for a device-to-device copy of 1 GiB (profiles/rta_step_workload3_hbm_traffic.md).
# Valid only for the kernel sources the counters were taken with (RTA_SOURCES / GPRIO_SOURCES below).
MEASURED_TRAFFIC = dict(csrc_sha256="14f51d6b715949ec02784f7f42a74b41aaae5b685fc8af4c819906c05c366888",
                        workload=3, tasksets=1_000_000, fetch_bytes=915827395, write_bytes=328834939)


# The same for `--row gprio` (workload 3; the skip flags of the run; mean of the two waiting modes;
# profiles/gprio_step_workload3_hbm_traffic.md).
MEASURED_TRAFFIC_GPRIO = dict(csrc_sha256="3d1f3d9819d9c94e3659b628b46be6cdc18f7517be3626a559ab12340c9b75d5",
                              workload=3, tasksets=1_000_000, fetch_bytes=877660561, write_bytes=242013028)


# the sources a row's kernels are built from: its counters stay valid while these are unchanged
RTA_SOURCES = ("gcaps_rta.hip", "rta_fast.hip.inc", "rta_quad.hip.inc", "rta_deep.hip.inc", "rta_wide.hip.inc",
               "rta_bin.hip.inc")
GPRIO_SOURCES = ("gcaps_rta.hip", "rta_fast.hip.inc", "rta_wide.hip.inc", "gprio_tile.hip.inc", "gprio_fast.hip.inc",
                 "gprio_wide.hip.inc")


def csrc_sha256(names=RTA_SOURCES):
    import hashlib
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_2406_05221_amd", "csrc")
    for name in sorted(names):
        h.update(name.encode())
        h.update(open(os.path.join(d, name), "rb").read())
    return h.hexdigest()


def copy_calibration():
    """Device-to-device copies of 1 GiB: a kernel of known traffic for scaling the HBM byte counters."""
    import torch
    src = torch.zeros(2**28, dtype=torch.int32, device="cuda:0")
    dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)
    torch.cuda.synchronize()
    del src, dst


def host_threads():
    """Host threads for the oracle leg: every core this process may run on, or the CPU share that the
    environment states for the job when that is smaller."""
    allowed = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
    share = os.environ.get("OMP_NUM_THREADS", "")
    return max(1, min(allowed, int(share)) if share.isdigit() and int(share) > 0 else allowed)


WORKLOAD0 = dict(n_cores=4, tasks_per_core=5, max_gseg=3, util=(0.25, 0.85), eta=(0, 3), share=(0.05, 0.5),
                 period=(20_000, 1_000_000), overhead=(0, 40), slice_us=1024, seed=0, stream=1000)


def timed_steps(B, ctx, stream, step, steps, warmup, spread=True):
    """`warmup` untimed and `steps` timed calls of step() on the context's stream: (seconds of wall time over
    the timed calls, device milliseconds per call from ONE pair of events around the timed calls on that stream,
    device milliseconds of each call of a further, untimed round with an event pair per call).  Events between
    the calls of the timed round would cost every step about 7 us of GPU idle time."""
    import torch
    for _ in range(warmup):
        step()
    B.gcaps_status(ctx)
    first, last = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    first.record(stream)
    for k in range(steps):
        step()
    last.record(stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    B.gcaps_status(ctx)
    each = []
    if spread:
        starts = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
        stops = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
        for k in range(steps):
            starts[k].record(stream)
            step()
            stops[k].record(stream)
        torch.cuda.synchronize()
        B.gcaps_status(ctx)
        each = [a.elapsed_time(b) for a, b in zip(starts, stops)]
    return t1 - t0, first.elapsed_time(last) / steps, each


def other_workloads(B, taskgen, ctx, stream, steps, warmup, skip):
    """Device milliseconds per step (both analyses) for the workloads the headline is not quoted on, each
    generated on the device by the host generator's recipe (the same tasksets bit for bit) at its own shape and
    at most 1,000,000 tasksets per batch."""
    import numpy as np
    import torch
    res = {}
    for k in (0, 1, 2, 3, 4, 5):
        if k == skip:
            continue
        if k == 0:
            N, params = 1_000_000, WORKLOAD0
        else:
            N, params = taskgen.config_params(k, min(taskgen.CONFIG_SIZES[k], 1_000_000))
        d = B.gcaps_taskgen_device(ctx, N, **params)
        n = params["n_cores"] * params["tasks_per_core"]
        resp = torch.empty((2, N, n), dtype=torch.int64, device="cuda:0")
        sched = torch.empty((2, N), dtype=torch.uint8, device="cuda:0")
        torch.cuda.synchronize()
        row = dict(tasksets=N, n_tasks=n, max_gseg=params["max_gseg"])
        for wait, name in ((B.GCAPS_WAIT_BUSY, "busy"), (B.GCAPS_WAIT_SUSPEND, "suspend")):
            _, dev, _ = timed_steps(B, ctx, stream, lambda: B.gcaps_rta_batch_device(ctx, d, B.GCAPS_POLICY_BOTH, wait,
                                                                                    resp, sched), steps, warmup, spread=False)
            row[f"device_ms_{name}"] = float(dev)
            row[f"sched_ratio_gcaps_{name}"] = float(sched[0].float().mean().item())
            row[f"tasksets_via_64bit_kernel_{name}"] = B.gcaps_last_wide_count(ctx)
        slow = max(row["device_ms_busy"], row["device_ms_suspend"])
        row["hbm_frac"] = algorithmic_bytes_per_taskset(n, params["max_gseg"], 2) * N / (slow * 1e-3) / 1e9 / HBM_PEAK_GBS
        res[str(k)] = row
        del d, resp, sched
    return res


def algorithmic_bytes_per_taskset(n, S, npol):
    """Bytes the path must move per taskset: every input once, every output once."""
    inputs = 3 * 4 + n * (4 * 4 + 2 * 1) + n * S * 2 * 4   # theta, eps, L; C, T, D, prio, core, eta; Gm, Ge
    outputs = npol * (n * 8 + 1)                           # int64 response times, uint8 flag
    return inputs + outputs


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", type=int, default=3, choices=[0, 1, 2, 3, 4, 5],
                    help="named workload; 5 is timed on one 1M-taskset batch of its stream; 0 = an extra, "
                         "iteration-heavy variant of workload 3 (long periods, small overheads: most tasksets "
                         "schedulable under GCAPS), not a headline")
    ap.add_argument("--tasksets", type=int, default=None, help="override the batch size")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-probe", action="store_true", help="skip the VALU rate probe (keeps a kernel trace short)")
    ap.add_argument("--no-end-to-end", action="store_true", help="skip the timing of the host entry point")
    ap.add_argument("--no-per-workload", action="store_true", help="skip the device timings of the other workloads")
    ap.add_argument("--binning", type=int, default=0, choices=[0, 1])
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run device-to-device copies of 1 GiB (a kernel of known traffic, for scaling "
                         "HBM byte counters collected over this command)")
    ap.add_argument("--print-csrc-hash", action="store_true", help="print the hash of the kernel sources and exit")
    ap.add_argument("--row", choices=["rta", "gprio", "sim", "stream", "peak"], default="rta",
                    help="rta (default, the headline): both response-time analyses; gprio: the GPU-segment "
                         "priority assignment (Sec. 4.3 / 5.4) for the tasksets that fail the GCAPS test with "
                         "GPU priority = CPU priority, as in the procedure of Sec. 6.1; sim: schedule simulation "
                         "(observed response times, Sec. 6.2) of lightly loaded tasksets of workload 3's shape; stream: "
                         "every step generates a fresh 1M-taskset batch of the workload on the device and analyses it "
                         "(workload 5's stream of batches without host-to-device copies); peak: the measured 32-bit integer "
                         "VALU rates of the device (independent chains of one instruction kind at full occupancy), "
                         "the denominators of the int32_valu figures")
    ap.add_argument("--recipe", choices=["workload", "table3"], default="workload",
                    help="--row stream: generate the named workload (default) or the paper's own recipe (Sec. 6.1, "
                         "Table 3: 12-24 tasks per taskset, grouped by task count on the device)")
    ap.add_argument("--horizon", type=int, default=1_000_000, help="--row sim: simulated interval (microseconds)")
    ap.add_argument("--search-all", action="store_true", help="--row gprio: search every taskset, skip none")
    ap.add_argument("--continue-after-miss", action="store_true",
                    help="--row rta: analyse every task, with D_h for the unknown R_h below a miss (not the headline)")
    args = ap.parse_args()
    if args.print_csrc_hash:
        print("rta", csrc_sha256(RTA_SOURCES))
        print("gprio", csrc_sha256(GPRIO_SOURCES))
        return
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this path is built and measured on ONE GPU; run it with --gpus 1 "
              "(tasksets are independent, more GPUs would each take a contiguous share)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2406_05221_amd import binding as B, taskgen

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    if args.row == "peak":
        ctx = B.gcaps_create(0, torch.cuda.Stream().cuda_stream)
        rates = B.gcaps_valu_probe(ctx)
        hbm = B.gcaps_hbm_probe(ctx, 1 << 30)
        B.gcaps_destroy(ctx)
        rates["relative_to_spec"] = {k: v / rates["spec_lane_ops_per_s"] for k, v in rates["lane_ops_per_s"].items()}
        print(json.dumps(dict(metric="32-bit integer VALU lane-operations/sec by instruction kind, 1 MI355X",
                              unit="lane-ops/s", n_gpus=1, **rates,
                              hbm_GBs={k: v / 1e9 for k, v in hbm.items()}, hbm_peak_GBs=HBM_PEAK_GBS,
                              hbm_note="bytes read + written per second of plain streaming kernels over 1 GiB "
                                       "buffers; _stream: with the non-temporal hint")))
        return
    if args.row == "sim":
        return bench_sim(args)
    if args.row == "stream":
        return bench_stream(args)
    if args.workload == 0:
        N = args.tasksets or 1_000_000
        cores, per_core, S = 4, 5, 3
        batch = taskgen.generate(N, **WORKLOAD0)
    else:
        N = args.tasksets or min(taskgen.CONFIG_SIZES[args.workload], 1_000_000)
        cores, per_core, S = taskgen.CONFIG_SHAPES[args.workload]
        batch = taskgen.config(args.workload, N)
    n = cores * per_core
    if args.row == "gprio":
        return bench_gprio(args, batch, N, cores, per_core, S)
    policy = B.GCAPS_POLICY_BOTH
    P = 2

    stream = torch.cuda.Stream()
    ctx = B.gcaps_create(0, stream.cuda_stream)
    B.gcaps_set_binning(ctx, args.binning)
    B.gcaps_set_continue_after_miss(ctx, int(args.continue_after_miss))
    d = B.to_device(batch)
    d_resp = torch.empty((P, N, n), dtype=torch.int64, device="cuda:0")
    d_sched = torch.empty((P, N), dtype=torch.uint8, device="cuda:0")
    torch.cuda.synchronize()

    modes = {}
    for wait, name in ((B.GCAPS_WAIT_BUSY, "busy"), (B.GCAPS_WAIT_SUSPEND, "suspend")):
        wall, dev, dev_each = timed_steps(B, ctx, stream,
                                          lambda: B.gcaps_rta_batch_device(ctx, d, policy, wait, d_resp, d_sched),
                                          args.steps, args.warmup)
        modes[name] = dict(wall_ms_per_step=wall * 1e3 / args.steps,
                           device_ms_per_step=float(dev),  # one event pair around the timed calls
                           device_ms_median=float(np.median(dev_each)),  # of a further round, one pair per call
                           tasksets_per_s=N * args.steps / wall,
                           sched_ratio_gcaps=float(d_sched[0].float().mean().item()),
                           sched_ratio_rr=float(d_sched[1].float().mean().item()),
                           tasksets_via_64bit_kernel=B.gcaps_last_wide_count(ctx))
    if args.copy_calibration:
        copy_calibration()
    head = min(modes, key=lambda m: modes[m]["tasksets_per_s"])
    head_wait = B.GCAPS_WAIT_BUSY if head == "busy" else B.GCAPS_WAIT_SUSPEND

    # ---- CPU oracle beside it (reported baseline, never the product path) ----
    cpu = None
    terms_per_taskset = None
    if not args.no_cpu_baseline:
        import oracle
        threads = host_threads()
        sample = min(N, 1_000_000)
        sub = {k: v[:sample] for k, v in batch.items()}
        t0 = time.perf_counter()
        opts = oracle.OPT_CONTINUE_AFTER_MISS if args.continue_after_miss else 0
        want_r, want_s, terms = oracle.rta_batch(sub, oracle.POLICY_BOTH, head_wait, threads=threads, options=opts)
        t_all = time.perf_counter() - t0
        one = min(sample, 100_000)
        sub1 = {k: v[:one] for k, v in batch.items()}
        t0 = time.perf_counter()
        oracle.rta_batch(sub1, oracle.POLICY_BOTH, head_wait, threads=1, options=opts)
        t_one = time.perf_counter() - t0
        terms_per_taskset = terms / sample
        # the benchmark's own outputs are checked against the oracle while we are here
        B.gcaps_rta_batch_device(ctx, d, policy, head_wait, d_resp, d_sched)
        B.gcaps_status(ctx)
        same = bool((d_resp[:, :sample].cpu().numpy() == want_r).all() and
                    (d_sched[:, :sample].cpu().numpy() == want_s).all())
        cpu = dict(value=sample / t_all, unit="tasksets/s", cores=threads, kind="oracle",
                   host_cores_visible=os.cpu_count(),
                   sample=f"first {sample} tasksets of the workload, both analyses, {head} mode, "
                          f"{threads} std::thread workers over tasksets (every core the job may use)",
                   one_core_value=one / t_one, one_core_sample=f"first {one} tasksets, 1 thread",
                   gpu_matches_oracle_on_sample=same)

    m = modes[head]
    bytes_per_launch = algorithmic_bytes_per_taskset(n, S, P) * N
    achieved = bytes_per_launch / (m["device_ms_per_step"] * 1e-3) / 1e9
    traffic = None
    mt = MEASURED_TRAFFIC
    if (mt["csrc_sha256"] and args.workload == mt["workload"] and N == mt["tasksets"] and not args.binning
            and not args.continue_after_miss
            and mt["csrc_sha256"] == csrc_sha256()):
        traffic = mt["fetch_bytes"] + mt["write_bytes"]
    roofline = dict(bound="hbm", achieved=achieved, peak=HBM_PEAK_GBS, unit="GB/s", frac=achieved / HBM_PEAK_GBS,
                    traffic=traffic, kernel="gcaps_rta_batch_device (all launches of one step)",
                    algorithmic_bytes_per_taskset=algorithmic_bytes_per_taskset(n, S, P))
    # the arithmetic side: the probe's rates are measured now, on this device
    alu = dict(peak=VALU_PEAK_LANE_OPS, peak_by="256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz",
               note="6 integer ops per interference term evaluated by plain iteration (oracle count); "
                    "peak_measured_term_mix = the add, 24-bit multiply-high, shift, 24-bit multiply-add of one term "
                    "in independent chains, measured in this run")
    term_mix = None
    if not args.no_probe:
        rates = B.gcaps_valu_probe(ctx)
        term_mix = rates["lane_ops_per_s"]["term"]
        alu.update(probe_lane_ops_per_s=rates["lane_ops_per_s"], probe_clock_khz=rates["clock_khz"],
                   probe_cu_count=rates["cu_count"], peak_measured_term_mix=term_mix)
    if terms_per_taskset is not None:
        ops = OPS_PER_TERM * terms_per_taskset * N / (m["device_ms_per_step"] * 1e-3)
        alu.update(terms_per_taskset=terms_per_taskset, terms_per_s=ops / OPS_PER_TERM, int32_lane_ops_per_s=ops,
                   frac=ops / VALU_PEAK_LANE_OPS,
                   frac_of_measured_term_mix=None if term_mix is None else ops / term_mix)
    hbm_measured = None
    if not args.no_probe:
        hbm_measured = {k: v / 1e9 for k, v in B.gcaps_hbm_probe(ctx, 1 << 30).items()}
    mv = MEASURED_VALU
    counted = mv["per_workload"].get(str(args.workload), {}).get(head)
    alu["measured_valu_lane_ops_per_s"] = None
    if (counted and N == mv["tasksets"] and not args.binning and not args.continue_after_miss
            and mv["csrc_sha256"] == csrc_sha256()):
        rate = counted["valu_lane_ops"] / (m["device_ms_per_step"] * 1e-3)
        alu.update(measured_valu_lane_ops_per_s=rate, measured_frac=rate / VALU_PEAK_LANE_OPS,
                   measured_valu_wave_insts_per_step=counted["valu_wave_insts"],
                   measured_active_lanes_per_valu_inst=counted["valu_lane_ops"] / counted["valu_wave_insts"],
                   measured_valu_issue_frac=counted["valu_wave_insts"] * 4 / (256 * 4 * 2.4e9 * m["device_ms_per_step"] * 1e-3),
                   measured_note="hardware counters of an earlier run of these kernel sources over the time of "
                                 "this run; issue fraction = VALU wavefront-instructions x 4 cycles over the "
                                 "SIMD-cycles of the step")

    # the host entry point: pack, copy in, analyse, copy out (the PCIe-inclusive rate; never `value`)
    end_to_end = None
    if not args.no_end_to_end:
        B.gcaps_rta_batch(ctx, batch, policy, head_wait)
        reps = 2
        t0 = time.perf_counter()
        for _ in range(reps):
            B.gcaps_rta_batch(ctx, batch, policy, head_wait)
        end_to_end = (time.perf_counter() - t0) * 1e3 / reps
    per_workload = None
    if not args.no_per_workload:
        per_workload = other_workloads(B, taskgen, ctx, stream, max(3, args.steps // 2), 2, args.workload)

    out = dict(metric="tasksets analysed/sec (both RTAs), 1 MI355X", value=m["tasksets_per_s"], unit="tasksets/s",
               n_gpus=1, steps=args.steps, warmup=args.warmup, ms_per_step=m["wall_ms_per_step"],
               higher_is_better=True, scaling="weak", vs_baseline=None, dtype="u32", data="synthetic",
               config=dict(workload=f"workload {args.workload}: {N} tasksets, {cores} cores x {per_core} tasks/core, "
                                    f"up to {S} GPU segments/task, GCAPS + round-robin analyses, headline = slower "
                                    f"waiting mode ({head})",
                           tasksets=N, n_tasks=n, max_gseg=S, policy="gcaps+rr", wait_mode=head,
                           binning=args.binning, continue_after_miss=bool(args.continue_after_miss)),
               modes=modes, roofline=roofline, int32_valu=alu, cpu_baseline=cpu,
               hbm_measured_GBs=hbm_measured,  # plain streaming kernels over 1 GiB, this run; beside roofline.peak
               end_to_end_ms=end_to_end,
               end_to_end_tasksets_per_s=None if end_to_end is None else N / (end_to_end * 1e-3),
               per_workload=per_workload)
    B.gcaps_destroy(ctx)
    print(json.dumps(out))


def bench_gprio(args, batch, N, cores, per_core, S):
    """One step = the GPU-segment priority search over one device-resident batch; tasksets that pass
    the GCAPS test with equal priorities are skipped (their flags are computed before the timed
    region by the response-time analysis, which is what the procedure of Sec. 6.1 has at that point)."""
    import numpy as np
    import torch
    from paper_2406_05221_amd import binding as B

    n = cores * per_core
    stream = torch.cuda.Stream()
    ctx = B.gcaps_create(0, stream.cuda_stream)
    d = B.to_device(batch)
    d_flags = torch.empty((1, N), dtype=torch.uint8, device="cuda:0")
    d_r1 = torch.empty((1, N, n), dtype=torch.int64, device="cuda:0")
    d_gprio = torch.empty((N, n), dtype=torch.int32, device="cuda:0")
    d_resp = torch.empty((N, n), dtype=torch.int64, device="cuda:0")
    d_sched = torch.empty((N,), dtype=torch.uint8, device="cuda:0")
    torch.cuda.synchronize()
    modes = {}
    for wait, name in ((B.GCAPS_WAIT_BUSY, "busy"), (B.GCAPS_WAIT_SUSPEND, "suspend")):
        B.gcaps_rta_batch_device(ctx, d, B.GCAPS_POLICY_GCAPS, wait, d_r1, d_flags)
        B.gcaps_status(ctx)
        d_skip = None if args.search_all else d_flags[0].clone()
        wall, dev, dev_each = timed_steps(B, ctx, stream,
                                          lambda: B.gcaps_gprio_assign_batch_device(ctx, d, wait, d_skip, d_gprio,
                                                                                    d_resp, d_sched),
                                          args.steps, args.warmup)
        searched = N if d_skip is None else int(N - d_skip.sum().item())
        found = int(d_sched.sum().item()) - (N - searched)
        modes[name] = dict(wall_ms_per_step=wall * 1e3 / args.steps, device_ms_per_step=float(dev),
                           device_ms_median=float(np.median(dev_each)), tasksets_per_s=N * args.steps / wall,
                           searched=searched, searched_per_s=searched * args.steps / wall,
                           assignments_found=found, tasksets_via_64bit_kernel=B.gcaps_last_wide_count(ctx),
                           skip=None if d_skip is None else d_skip.cpu().numpy())
    head = min(modes, key=lambda m: modes[m]["tasksets_per_s"])
    head_wait = B.GCAPS_WAIT_BUSY if head == "busy" else B.GCAPS_WAIT_SUSPEND
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        threads = host_threads()
        sample = min(N, 200_000)
        sub = {k: v[:sample] for k, v in batch.items()}
        skip = modes[head]["skip"]
        skip = None if skip is None else skip[:sample]
        t0 = time.perf_counter()
        want_g, want_r, want_s, _ = oracle.gprio_assign_batch(sub, head_wait, skip=skip, threads=threads)
        t_all = time.perf_counter() - t0
        B.gcaps_gprio_assign_batch_device(ctx, d, head_wait,
                                          None if args.search_all else torch.from_numpy(modes[head]["skip"]).cuda(),
                                          d_gprio, d_resp, d_sched)
        B.gcaps_status(ctx)
        same = bool((d_gprio[:sample].cpu().numpy() == want_g).all() and (d_resp[:sample].cpu().numpy() == want_r).all()
                    and (d_sched[:sample].cpu().numpy() == want_s).all())
        cpu = dict(value=sample / t_all, unit="tasksets/s", cores=threads, kind="oracle",
                   sample=f"first {sample} tasksets of the workload (same skip flags), {head} mode, "
                          f"{threads} std::thread workers over tasksets",
                   gpu_matches_oracle_on_sample=same)
    if args.copy_calibration:
        copy_calibration()
    for mm in modes.values():
        mm.pop("skip")
    m = modes[head]
    per_searched = 4 + 1 + n * (4 * 4 + 2) + n * S * 8   # eps, skip flag; C, T, D, prio, core, eta; Gm, Ge
    per_output = n * (4 + 8) + 1                         # level, bound; verdict
    alg_bytes = m["searched"] * per_searched + (N - m["searched"]) * 1 + N * per_output
    achieved = alg_bytes / (m["device_ms_per_step"] * 1e-3) / 1e9
    traffic = None
    mt = MEASURED_TRAFFIC_GPRIO
    if (mt["csrc_sha256"] and args.workload == mt["workload"] and N == mt["tasksets"] and not args.search_all
            and mt["csrc_sha256"] == csrc_sha256(GPRIO_SOURCES)):
        traffic = mt["fetch_bytes"] + mt["write_bytes"]
    roofline = dict(bound="hbm", achieved=achieved, peak=HBM_PEAK_GBS, unit="GB/s", frac=achieved / HBM_PEAK_GBS,
                    traffic=traffic, kernel="gcaps_gprio_assign_batch_device (all launches of one step)",
                    algorithmic_bytes_per_step=alg_bytes)
    out = dict(metric="tasksets through the GPU-segment priority search/sec, 1 MI355X", value=m["tasksets_per_s"],
               unit="tasksets/s", n_gpus=1, steps=args.steps, warmup=args.warmup, ms_per_step=m["wall_ms_per_step"],
               higher_is_better=True, scaling="weak", vs_baseline=None, dtype="u32", data="synthetic",
               config=dict(workload=f"workload {args.workload}: {N} tasksets, {cores} cores x {per_core} tasks/core, "
                                    f"up to {S} GPU segments/task; priority search for the tasksets that fail the "
                                    f"GCAPS test with equal priorities ({m['searched']} of {N}); headline = slower "
                                    f"waiting mode ({head})" if not args.search_all else
                                    f"workload {args.workload}: {N} tasksets, priority search for every taskset; "
                                    f"headline = slower waiting mode ({head})",
                           tasksets=N, n_tasks=n, max_gseg=S, wait_mode=head, row="gprio"),
               modes=modes, roofline=roofline, cpu_baseline=cpu)
    B.gcaps_destroy(ctx)
    print(json.dumps(out))


def bench_stream_table3(args):
    """One step = N fresh tasksets of the recipe of Sec. 6.1 / Table 3 generated on the device (counted, grouped
    by task count, written as one batch per count) and analysed under both policies, self-suspension.  The groups
    of the last step are copied back and analysed by the oracle."""
    import numpy as np
    import torch
    from paper_2406_05221_amd import binding as B

    N = args.tasksets or 200_000
    stream = torch.cuda.Stream()
    ctx = B.gcaps_create(0, stream.cuda_stream)
    wait = B.GCAPS_WAIT_SUSPEND

    def step(k):
        groups = B.gcaps_table3_device(ctx, N, seed=0, stream=300, first_index=k * N)
        outs = {}
        for n, (idx, d) in groups.items():
            M = int(idx.numel())
            outs[n] = (torch.empty((2, M, n), dtype=torch.int64, device="cuda:0"),
                       torch.empty((2, M), dtype=torch.uint8, device="cuda:0"))
        for n, (idx, d) in groups.items():
            B.gcaps_rta_batch_device(ctx, d, B.GCAPS_POLICY_BOTH, wait, *outs[n])
        B.gcaps_status(ctx)
        return groups, outs

    for k in range(args.warmup):
        step(k)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        groups, outs = step(args.warmup + k)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    cpu = None
    alg_bytes = 0
    for n, (idx, d) in groups.items():
        S = d["gm_us"].shape[2]
        inputs = 3 * 4 + n * (4 * 4 + 2 * 1) + n * S * 2 * 4
        alg_bytes += int(idx.numel()) * (inputs + algorithmic_bytes_per_taskset(n, S, 2))
    if not args.no_cpu_baseline:
        import oracle
        threads = os.cpu_count() or 1
        host = {n: B.to_host(d) for n, (idx, d) in groups.items()}
        t0c = time.perf_counter()
        want = {n: oracle.rta_batch(h, oracle.POLICY_BOTH, wait, threads=threads) for n, h in host.items()}
        t_all = time.perf_counter() - t0c
        same = all(bool((outs[n][0].cpu().numpy() == want[n][0]).all() and (outs[n][1].cpu().numpy() == want[n][1]).all())
                   for n in host)
        cpu = dict(value=N / t_all, unit="tasksets/s", cores=threads, kind="oracle",
                   sample=f"the tasksets of the last step ({N}, copied back), analysis only, {threads} std::thread "
                          f"workers over tasksets", gpu_matches_oracle_on_sample=same)
    ms = (t1 - t0) * 1e3 / args.steps
    achieved = alg_bytes / (ms * 1e-3) / 1e9
    out = dict(metric="tasksets generated on the device and analysed/sec (GCAPS + round-robin), 1 MI355X",
               value=N * args.steps / (t1 - t0), unit="tasksets/s", n_gpus=1, steps=args.steps, warmup=args.warmup,
               ms_per_step=ms, higher_is_better=True, scaling="weak", vs_baseline=None, dtype="u32", data="synthetic",
               config=dict(workload=f"the recipe of Sec. 6.1 / Table 3: {N} tasksets per step, 4 CPUs x 3-6 tasks, 40-60 % "
                                    f"GPU-using tasks with 1-3 segments, periods 30-500 ms, eps 1 ms, theta 200 us; counted, "
                                    f"grouped by task count ({len(groups)} batches) and analysed under both policies, "
                                    f"self-suspension; wall clock with the host's grouping in it",
                           tasksets=N, wait_mode="suspend", row="stream", recipe="table3"),
               roofline=dict(bound="hbm", achieved=achieved, peak=HBM_PEAK_GBS, unit="GB/s", frac=achieved / HBM_PEAK_GBS,
                             traffic=None, kernel="gen::table3_* + gcaps_rta_batch_device (all launches of one step)",
                             algorithmic_bytes_per_step=alg_bytes),
               cpu_baseline=cpu)
    B.gcaps_destroy(ctx)
    print(json.dumps(out))


def bench_stream(args):
    """One step = one fresh batch of the workload generated on the device (taskset indices continue from
    batch to batch) and analysed under both policies: the stream of batches of workload 5 with no host-to-device
    copy.  The batch of the last timed step is copied back and analysed by the oracle."""
    import numpy as np
    import torch
    from paper_2406_05221_amd import binding as B, taskgen

    if args.recipe == "table3":
        return bench_stream_table3(args)

    k = args.workload if args.workload in (1, 2, 3, 4, 5) else 5
    N = args.tasksets or min(taskgen.CONFIG_SIZES[k], 1_000_000)
    cores, per_core, S = taskgen.CONFIG_SHAPES[k]
    n = cores * per_core
    stream = torch.cuda.Stream()
    ctx = B.gcaps_create(0, stream.cuda_stream)
    d_resp = torch.empty((2, N, n), dtype=torch.int64, device="cuda:0")
    d_sched = torch.empty((2, N), dtype=torch.uint8, device="cuda:0")
    total = args.warmup + args.steps
    # per-taskset parameters of the workload (its sweep point or grid cell) for every batch: resident before timing
    specs = []
    for bidx in range(total):
        _, params = taskgen.config_params(k, N, first_index=bidx * N)
        specs.append({key: (torch.from_numpy(v.view(np.int32) if v.dtype == np.uint32 else v).cuda()
                            if isinstance(v, np.ndarray) else v) for key, v in params.items()})
    torch.cuda.synchronize()

    def generate(params, out):
        # device tensors stand in for the per-taskset arrays: marshal them as the binding does for numpy arrays
        fixed = {key: v for key, v in params.items() if isinstance(v, torch.Tensor)}
        plain = {key: ((0, 0) if key != "slice_us" else 1) if key in fixed else v for key, v in params.items()}
        return B.gcaps_taskgen_device(ctx, N, out=out, fixed=fixed, **plain)

    wait = B.GCAPS_WAIT_SUSPEND
    d = None
    with torch.cuda.stream(stream):
        for bidx in range(args.warmup):
            d = generate(specs[bidx], d)
            B.gcaps_rta_batch_device(ctx, d, B.GCAPS_POLICY_BOTH, wait, d_resp, d_sched)
        B.gcaps_status(ctx)
        first, last = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        first.record(stream)  # one event pair around the timed steps: events between them would idle the GPU
        for s in range(args.steps):
            d = generate(specs[args.warmup + s], d)
            B.gcaps_rta_batch_device(ctx, d, B.GCAPS_POLICY_BOTH, wait, d_resp, d_sched)
        last.record(stream)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        B.gcaps_status(ctx)
    dev_ms = first.elapsed_time(last) / args.steps
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        threads = host_threads()
        host = B.to_host(d)
        t0c = time.perf_counter()
        want_r, want_s, _ = oracle.rta_batch(host, oracle.POLICY_BOTH, wait, threads=threads)
        t_all = time.perf_counter() - t0c
        same = bool((d_resp.cpu().numpy() == want_r).all() and (d_sched.cpu().numpy() == want_s).all())
        cpu = dict(value=N / t_all, unit="tasksets/s", cores=threads, kind="oracle",
                   sample=f"the last batch of the stream ({N} tasksets, copied back), analysis only, "
                          f"{threads} std::thread workers over tasksets", gpu_matches_oracle_on_sample=same)
    inputs = 3 * 4 + n * (4 * 4 + 2 * 1) + n * S * 2 * 4
    alg_bytes = N * (inputs + algorithmic_bytes_per_taskset(n, S, 2))  # written by the generator; read and answered
    achieved = alg_bytes / (dev_ms * 1e-3) / 1e9
    out = dict(metric="tasksets generated on the device and analysed/sec (GCAPS + round-robin), 1 MI355X",
               value=N * args.steps / (t1 - t0), unit="tasksets/s", n_gpus=1, steps=args.steps, warmup=args.warmup,
               ms_per_step=(t1 - t0) * 1e3 / args.steps, higher_is_better=True, scaling="weak", vs_baseline=None,
               dtype="u32", data="synthetic",
               config=dict(workload=f"workload {k}: a stream of {args.steps} batches of {N} tasksets, {cores} cores x "
                                    f"{per_core} tasks/core, up to {S} GPU segments/task; each generated on the device "
                                    f"and analysed under both policies, self-suspension",
                           tasksets=N, n_tasks=n, max_gseg=S, wait_mode="suspend", row="stream"),
               device_ms_per_step=dev_ms,
               roofline=dict(bound="hbm", achieved=achieved, peak=HBM_PEAK_GBS, unit="GB/s",
                             frac=achieved / HBM_PEAK_GBS, traffic=None,
                             kernel="gen::generate_kernel + gcaps_rta_batch_device (all launches of one step)",
                             algorithmic_bytes_per_step=alg_bytes),
               cpu_baseline=cpu)
    B.gcaps_destroy(ctx)
    print(json.dumps(out))


INT_ALU_PEAK_TOPS = 256 * 64 * 2.4e9 / 1e12  # 256 compute units x 64 lanes per clock (4 SIMDs of 16) x 2.4 GHz


def bench_sim(args):
    """One step = the schedule simulation of one device-resident batch under both GPU policies over
    --horizon microseconds of task time."""
    import numpy as np
    import torch
    from paper_2406_05221_amd import binding as B, taskgen

    N = args.tasksets or 262_144
    cores, per_core, S = 4, 5, 3
    n = cores * per_core
    batch = taskgen.generate(N, n_cores=cores, tasks_per_core=per_core, max_gseg=S, util=(0.2, 0.4), eta=(1, 3),
                             share=(0.10, 0.60), period=(10_000, 100_000), overhead=(50, 500), slice_us=1024,
                             seed=0, stream=79)
    stream = torch.cuda.Stream()
    ctx = B.gcaps_create(0, stream.cuda_stream)
    d = B.to_device(batch)
    d_mort = torch.empty((2, N, n), dtype=torch.int64, device="cuda:0")
    d_jobs = torch.empty((2, N, n), dtype=torch.int32, device="cuda:0")
    d_flag = torch.empty((2, N), dtype=torch.uint8, device="cuda:0")
    torch.cuda.synchronize()
    steps = max(1, min(args.steps, 5))
    warmup = max(1, min(args.warmup, 1))
    modes = {}
    for wait, name in ((B.GCAPS_WAIT_BUSY, "busy"), (B.GCAPS_WAIT_SUSPEND, "suspend")):
        for _ in range(warmup):
            B.gcaps_simulate_batch_device(ctx, d, B.GCAPS_POLICY_BOTH, wait, args.horizon, d_mort, d_jobs, d_flag)
        B.gcaps_status(ctx)
        starts = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
        stops = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(steps):
            starts[k].record(stream)
            B.gcaps_simulate_batch_device(ctx, d, B.GCAPS_POLICY_BOTH, wait, args.horizon, d_mort, d_jobs, d_flag)
            stops[k].record(stream)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        B.gcaps_status(ctx)
        events = B.gcaps_last_sim_steps(ctx)
        dev_ms = [a.elapsed_time(b) for a, b in zip(starts, stops)]
        modes[name] = dict(wall_ms_per_step=(t1 - t0) * 1e3 / steps, device_ms_per_step=float(np.mean(dev_ms)),
                           tasksets_per_s=N * steps / (t1 - t0), events_per_step=events,
                           events_per_s=events / (float(np.mean(dev_ms)) * 1e-3),
                           jobs_completed=int(d_jobs.sum().item()),
                           stopped_at_an_overrun=int(d_flag.sum().item()))
    head = min(modes, key=lambda m: modes[m]["tasksets_per_s"])
    head_wait = B.GCAPS_WAIT_BUSY if head == "busy" else B.GCAPS_WAIT_SUSPEND
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        threads = host_threads()
        sample = min(N, 96)
        sub = {k: v[:sample] for k, v in batch.items()}
        t0 = time.perf_counter()
        want = oracle.simulate_batch(sub, oracle.POLICY_BOTH, head_wait, args.horizon, threads=threads)
        t_all = time.perf_counter() - t0
        B.gcaps_simulate_batch_device(ctx, d, B.GCAPS_POLICY_BOTH, head_wait, args.horizon, d_mort, d_jobs, d_flag)
        B.gcaps_status(ctx)
        same = bool((d_mort[:, :sample].cpu().numpy() == want[0]).all()
                    and (d_jobs[:, :sample].cpu().numpy().view(np.uint32) == want[1]).all()
                    and (d_flag[:, :sample].cpu().numpy() == want[2]).all())
        cpu = dict(value=sample / t_all, unit="tasksets/s", cores=threads, kind="oracle",
                   sample=f"first {sample} tasksets of the batch, both policies, {head} mode, one tick per "
                          f"microsecond, {threads} std::thread workers over tasksets",
                   gpu_matches_oracle_on_sample=same)
    m = modes[head]
    ops_per_event = 6 * n + 40  # per task: release / zero-time test, core arbitration, next-event minimum and charge
    achieved = m["events_per_step"] * ops_per_event / (m["device_ms_per_step"] * 1e-3) / 1e12
    roofline = dict(bound="alu", achieved=achieved, peak=INT_ALU_PEAK_TOPS, unit="TOP/s",
                    frac=achieved / INT_ALU_PEAK_TOPS, traffic=None, kernel="sim::simulate_kernel",
                    algorithmic_ops_per_event=ops_per_event, events_per_step=m["events_per_step"])
    out = dict(metric="tasksets simulated/sec (both GPU policies), 1 MI355X", value=m["tasksets_per_s"],
               unit="tasksets/s", n_gpus=1, steps=steps, warmup=warmup, ms_per_step=m["wall_ms_per_step"],
               higher_is_better=True, scaling="weak", vs_baseline=None, dtype="u32", data="synthetic",
               config=dict(workload=f"{N} tasksets of the shape and magnitudes of workload 3 ({cores} cores x {per_core} "
                                    f"tasks/core, up to {S} GPU segments/task, microseconds) at a per-core utilisation "
                                    f"of 0.2-0.4 and periods of 10-100 ms, simulated for {args.horizon} us under GCAPS "
                                    f"and round-robin; headline = slower waiting mode ({head})",
                           tasksets=N, n_tasks=n, max_gseg=S, horizon_us=args.horizon, wait_mode=head, row="sim"),
               modes=modes, roofline=roofline, cpu_baseline=cpu)
    B.gcaps_destroy(ctx)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
