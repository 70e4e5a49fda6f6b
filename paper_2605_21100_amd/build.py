"""Compile the HIP sources into libnanocp.so (gfx950), in-tree next to this file.

Every source is compiled to an object of its own (in parallel, objects under _build/), then linked.
Defining NANOCP_TUNING=1 in the environment builds the planner's and kernels' experiment knobs in
(-DNANOCP_TUNING); the product build has none.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SOURCES = ["plan.cpp", "sched.cpp", "generic.hip", "gqa_mfma.hip", "mla_mfma.hip", "kv_append.hip", "api.hip"]
LIB = os.path.join(HERE, "libnanocp.so")
OBJ_DIR = os.path.join(HERE, "_build")


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    out = "\n".join(l for l in (res.stdout + res.stderr).splitlines()
                    if "packed-fp32-ops" not in l)          # the host pass does not know the device feature
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)


def build(verbose=False, extra_flags=()):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ_DIR, exist_ok=True)
    flags = ["-x", "hip", "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             "-I", os.path.join(ROOT, "include"), "-I", os.path.join(HERE, "csrc")] + list(extra_flags)
    if os.environ.get("NANOCP_TUNING", "") == "1":
        flags.append("-DNANOCP_TUNING")
    objs = [os.path.join(OBJ_DIR, s + ".o") for s in SOURCES]
    jobs = [[hipcc] + flags + ["-c", os.path.join(HERE, "csrc", s), "-o", o] for s, o in zip(SOURCES, objs)]
    with ThreadPoolExecutor(max_workers=min(8, len(jobs))) as pool:
        list(pool.map(lambda c: _run(c, verbose), jobs))
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs, verbose)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
    sys.exit(0)
