"""Schedulability sweeps in the manner of Sec. 6.1: the share of randomly generated tasksets that
pass the response-time test, per analysis, while one generation parameter of Table 3 is varied.

    python -m paper_2406_05221_amd.sweep --param util --values 0.2,0.3,0.4,0.5,0.6 --tasksets 1000

Columns: the default round-robin TSG scheduling (Sec. 5.2) and GCAPS (Sec. 5.3), each with
busy-waiting and self-suspension, and GCAPS with the GPU-segment priority assignment tried for the
tasksets that fail with equal priorities (Sec. 4.3 / 5.4, the procedure of Sec. 6.1).  Everything
is computed by the GPU library; this module only draws inputs, groups them by task count (a batch
of the library has one task count) and averages verdicts.  Without best-effort tasks the inputs are
generated on the device as well (``--host-inputs`` to draw them on the host and copy them: the same
tasksets bit for bit), so that no taskset crosses the bus; only the verdicts come back.

Best-effort tasks (``--param be_ratio``, the last experiment of Sec. 6.1) run below every real-time
task and have no deadline.  Under round-robin TSG scheduling their GPU segments take part in the time
slicing: they stay in the taskset (Eq. 3 and Lemma 4 count every GPU-using task) and only the
real-time tasks' bounds decide the verdict.  Under GCAPS a lower-priority task can delay a real-time
task by the runlist-update blocking of Lemma 8 only, which is charged to every task anyway: the
best-effort tasks are left out of the taskset."""
import argparse

import numpy as np

from . import binding as B
from . import taskgen

COLUMNS = ["tsg_rr_busy", "tsg_rr_suspend", "gcaps_busy", "gcaps_suspend", "gcaps_busy+prio", "gcaps_suspend+prio"]


def verdicts(ctx, groups):
    """groups: {n: (indices, batch)} as returned by ``taskgen.table3``.  Returns a dict of uint8
    arrays over the generated tasksets (generation order), one per column."""
    total = sum(len(idx) for idx, _ in groups.values())
    out = {c: np.zeros(total, np.uint8) for c in COLUMNS}
    for idx, batch in groups.values():
        be = batch.get("best_effort")
        fields = {k: v for k, v in batch.items() if k != "best_effort"}
        real_time = fields if be is None else taskgen.without_tasks(fields, be != 0)
        for wait, name in ((B.GCAPS_WAIT_BUSY, "busy"), (B.GCAPS_WAIT_SUSPEND, "suspend")):
            if be is None:
                _, sched = B.gcaps_rta_batch(ctx, fields, B.GCAPS_POLICY_BOTH, wait)
                gcaps, rr = sched[0], sched[1]
            else:
                # round-robin: best-effort tasks stay (lowest priorities: they are analysed last and a miss
                # among them ends nothing above them); the verdict is that of the real-time tasks
                resp, _ = B.gcaps_rta_batch(ctx, fields, B.GCAPS_POLICY_RR, wait)
                rr = ((resp[0] >= 0) | (be != 0)).all(axis=1).astype(np.uint8)
                _, sched = B.gcaps_rta_batch(ctx, real_time, B.GCAPS_POLICY_GCAPS, wait)
                gcaps = sched[0]
            out[f"gcaps_{name}"][idx] = gcaps
            out[f"tsg_rr_{name}"][idx] = rr
            # separate GPU-segment priorities only where the test with equal priorities failed
            _, _, found = B.gcaps_gprio_assign_batch(ctx, real_time, wait, skip=gcaps)
            out[f"gcaps_{name}+prio"][idx] = found
    return out


def verdicts_device(ctx, groups, total):
    """The same for groups generated on the device ({n: (index tensor, device batch)} from
    ``binding.gcaps_table3_device``): device entry points only, the verdicts are copied back."""
    import torch
    out = {c: np.zeros(total, np.uint8) for c in COLUMNS}
    for idx, d in groups.values():
        N, n = d["cpu_us"].shape
        rows = idx.cpu().numpy()
        resp = torch.empty((2, N, n), dtype=torch.int64, device=idx.device)
        sched = torch.empty((2, N), dtype=torch.uint8, device=idx.device)
        gprio = torch.empty((N, n), dtype=torch.int32, device=idx.device)
        found = torch.empty((N,), dtype=torch.uint8, device=idx.device)
        torch.cuda.synchronize()  # the tensors were made on torch's stream, the library works on the context's
        for wait, name in ((B.GCAPS_WAIT_BUSY, "busy"), (B.GCAPS_WAIT_SUSPEND, "suspend")):
            B.gcaps_rta_batch_device(ctx, d, B.GCAPS_POLICY_BOTH, wait, resp, sched)
            # separate GPU-segment priorities only where the test with equal priorities failed
            B.gcaps_gprio_assign_batch_device(ctx, d, wait, sched[0], gprio, resp[0], found)
            B.gcaps_status(ctx)
            out[f"gcaps_{name}"][rows] = sched[0].cpu().numpy()
            out[f"tsg_rr_{name}"][rows] = sched[1].cpu().numpy()
            out[f"gcaps_{name}+prio"][rows] = found.cpu().numpy()
    return out


def sweep(ctx, param, values, n_tasksets, seed=0, host_inputs=False, **fixed):
    """One row per value of `param` (a key of ``taskgen.TABLE3``; range parameters are set to the
    single value): the share of schedulable tasksets per column.  `fixed`: other Table 3 parameters
    to hold at values of the caller's choice.  The tasksets are generated on the device unless
    best-effort tasks are asked for or `host_inputs` is set."""
    rows = []
    for k, v in enumerate(values):
        value = (v, v) if isinstance(taskgen.TABLE3[param], tuple) else v
        params = {**fixed, param: value}
        if host_inputs or float(params.get("be_ratio", 0.0)) != 0.0:
            res = verdicts(ctx, taskgen.table3(n_tasksets, seed=seed, stream=300 + k, **params))
        else:
            groups = B.gcaps_table3_device(ctx, n_tasksets, seed=seed, stream=300 + k, **params)
            res = verdicts_device(ctx, groups, n_tasksets)
        rows.append((v, {c: float(res[c].mean()) for c in COLUMNS}))
    return rows


def main():
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("--param", default="util", choices=sorted(taskgen.TABLE3))
    ap.add_argument("--values", default="0.2,0.3,0.4,0.5,0.6,0.7")
    ap.add_argument("--tasksets", type=int, default=1000, help="tasksets per point (the paper uses 1,000)")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--util", type=float, default=None, help="hold the utilisation per CPU at this value")
    ap.add_argument("--eps-us", type=int, default=None, help="hold the runlist-update delay at this value")
    ap.add_argument("--host-inputs", action="store_true", help="draw the tasksets on the host and copy them")
    args = ap.parse_args()
    cast = int if isinstance(taskgen.TABLE3[args.param], int) or args.param in ("tasks_per_cpu", "period", "eta") \
        else float
    values = [cast(x) for x in args.values.split(",")]
    ctx = B.gcaps_create(0)
    try:
        fixed = {}
        if args.util is not None and args.param != "util":
            fixed["util"] = (args.util, args.util)
        if args.eps_us is not None and args.param != "eps_us":
            fixed["eps_us"] = args.eps_us
        rows = sweep(ctx, args.param, values, args.tasksets, args.seed, host_inputs=args.host_inputs, **fixed)
    finally:
        B.gcaps_destroy(ctx)
    print(f"| {args.param} | " + " | ".join(COLUMNS) + " |")
    print("|---|" + "---|" * len(COLUMNS))
    for v, r in rows:
        print(f"| {v} | " + " | ".join(f"{100 * r[c]:.1f} %" for c in COLUMNS) + " |")


if __name__ == "__main__":
    main()
