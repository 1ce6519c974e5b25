"""Builds libsla.so (the C-ABI library of HIP kernels) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libsla.so")
# The same library with the timing probes of k_attend.hip and k_linear.hip compiled in (-DSLA_PROBE_TIME: one wave writes
# the shader-clock and 100 MHz counters at the phase boundaries of its work; results are unchanged).  Only probe.py loads it.
PROBE_LIB = os.path.join(HERE, "libsla_probe.so")
PROBED = ["k_attend.hip", "k_linear.hip", "k_classify.hip"]
SOURCES = ["sla_api.hip", "k_classify.hip", "k_states.hip", "k_aggregate.hip", "k_attend.hip", "k_backward.hip", "k_quant.hip", "k_linear.hip"]
FLAGS = ["-O3", "--offload-arch=gfx950", "-fPIC", "-std=c++17", "-ffp-contract=off", "-Wall", "-Wextra",
         "-Wno-unused-parameter", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-mllvm", "-amdgpu-mfma-vgpr-form=1"]   # MFMA accumulators stay in VGPRs: no AGPR copy traffic


def _hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.isabs(c) and os.path.exists(c) or not os.path.isabs(c)):
            return c
    return "hipcc"


def _compile(job) -> str:
    src, probe = job if isinstance(job, tuple) else (job, False)
    obj = os.path.join(OBJ, ("probe_" if probe else "") + src.replace(".hip", ".o"))
    cmd = [_hipcc(), *FLAGS, *(["-DSLA_PROBE_TIME"] if probe else []), "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose: bool = True) -> str:
    os.makedirs(OBJ, exist_ok=True)
    jobs = [(s_, False) for s_ in SOURCES] + [(s_, True) for s_ in PROBED]
    with ThreadPoolExecutor(max_workers=8) as ex:
        objs = list(ex.map(_compile, jobs))
    plain, probed = objs[:len(SOURCES)], dict(zip(PROBED, objs[len(SOURCES):]))
    subprocess.check_call([_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", *plain, "-o", LIB])
    subprocess.check_call([_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC",
                           *[probed.get(s_, o) for s_, o in zip(SOURCES, plain)], "-o", PROBE_LIB])
    if verbose:
        print(f"built {LIB}")
    return LIB


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(os.path.join(CSRC, f)) > t for f in os.listdir(CSRC))


if __name__ == "__main__":
    build()
