"""Builds the HIP library (gfx950) and the host-only taskset generator in-tree."""
import os
import subprocess

_PKG = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_PKG)
LIB_PATH = os.path.join(_PKG, "libgcaps_rta.so")

HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
               # packed FP32 VALU forms are kept out of the generated code
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               "-Wall", "-Wextra", "-Wno-unused-parameter"]


def build_hip(extra_flags=(), output=LIB_PATH):
    src = os.path.join(_PKG, "csrc", "gcaps_rta.hip")
    cmd = ["hipcc", *HIPCC_FLAGS, *extra_flags, "-I", os.path.join(_ROOT, "include"), "-o", output, src]
    r = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in r.stderr.splitlines() if noise not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    return output


def build_all():
    from . import taskgen
    build_hip()
    taskgen.build(force=True)
    return LIB_PATH
