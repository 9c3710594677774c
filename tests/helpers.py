"""Small host-side helpers shared by the tests (no analysis arithmetic)."""
import json
import os

import numpy as np

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")

VARIANTS = [(1, 0), (1, 1), (2, 0), (2, 1)]  # (policy, wait_mode): GCAPS=1, RR=2; busy=0, suspend=1


def seg_arrays(tasks):
    """tasks: list of dicts with gm, ge lists -> ([n,S] gm, [n,S] ge, eta[n])."""
    n = len(tasks)
    S = max(1, max(len(t["ge"]) for t in tasks))
    gm = np.zeros((n, S), np.uint32)
    ge = np.zeros((n, S), np.uint32)
    for i, t in enumerate(tasks):
        gm[i, : len(t["gm"])] = t["gm"]
        ge[i, : len(t["ge"])] = t["ge"]
    return gm, ge, np.array([len(t["ge"]) for t in tasks], np.uint8)


def oracle_bound(o, tasks, policy, wait, theta, eps, L, options=0):
    """tasks: dicts with C (or c list), T, D, prio, core, gm, ge."""
    gm, ge, eta = seg_arrays(tasks)
    C = [t["C"] if "C" in t else sum(t["c"]) for t in tasks]
    return o.rta_taskset(C, [t["T"] for t in tasks], [t["D"] for t in tasks], [t["prio"] for t in tasks],
                         [t["core"] for t in tasks], eta, gm, ge, theta_us=theta, eps_us=eps,
                         slice_us=L, policy=policy, wait_mode=wait, options=options)


def load_table2():
    with open(os.path.join(GOLDEN, "table2_taskset.json")) as f:
        g = json.load(f)
    tasks = []
    n = len(g["tasks"])
    for i, t in enumerate(g["tasks"]):
        tasks.append(dict(C=sum(t["cpu_segments"]), c=t["cpu_segments"], T=t["T"], D=t["D"], core=t["cpu"],
                          prio=n - i, gm=[s["gm"] for s in t["gpu_segments"]],
                          ge=[s["ge"] for s in t["gpu_segments"]]))
    return g, tasks


def classic_rta(C, T, D):
    """Textbook uniprocessor fixed-priority response-time analysis (Joseph & Pandya /
    Audsley et al.): tasks in decreasing priority, R = C_i + sum_h ceil(R/T_h) C_h.
    Returns list of R_i or None from the first deadline miss on."""
    out = []
    for i in range(len(C)):
        R = C[i]
        while True:
            nxt = C[i] + sum(-(-R // T[h]) * C[h] for h in range(i))
            if nxt > D[i]:
                R = None
                break
            if nxt == R:
                break
            R = nxt
        if R is None:
            out.extend([None] * (len(C) - i))
            break
        out.append(R)
    return out
