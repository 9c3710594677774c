"""Host-side contract of bench.py that needs no GPU: more than one GPU is refused with a message, the hash of the
kernel sources is printed on request."""
import os
import re
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run(*args, env=None):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True,
                          env={**os.environ, **(env or {})}, timeout=120)


def test_more_than_one_gpu_is_refused():
    r = run("--gpus", "2")
    assert r.returncode == 2 and "ONE GPU" in r.stderr and r.stdout == ""
    r = run(env={"WORLD_SIZE": "4"})
    assert r.returncode == 2 and "ONE GPU" in r.stderr


def test_source_hash():
    r = run("--print-csrc-hash")
    assert r.returncode == 0 and re.fullmatch(r"rta [0-9a-f]{64}\ngprio [0-9a-f]{64}\n", r.stdout)


def test_recorded_counters_belong_to_the_current_kernel_sources():
    """The HBM traffic and VALU counts that bench.py reports were taken with the kernel sources of the tree: a change
    to one of them without new counter runs would turn `roofline.traffic` into null, which this test notices first."""
    sys.path.insert(0, ROOT)
    import bench
    assert bench.MEASURED_TRAFFIC["csrc_sha256"] == bench.csrc_sha256(bench.RTA_SOURCES)
    assert bench.MEASURED_VALU["csrc_sha256"] == bench.csrc_sha256(bench.RTA_SOURCES)
    assert bench.MEASURED_TRAFFIC_GPRIO["csrc_sha256"] == bench.csrc_sha256(bench.GPRIO_SOURCES)
