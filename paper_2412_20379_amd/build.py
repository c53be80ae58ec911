"""Build libntp.so (HIP kernels + C boundary) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libntp.so")
PROBE_SRC = os.path.join(CSRC, "line_rate_probe.hip")
PROBE = os.path.join(PKG, "line_rate_probe")        # prints the chip's 128-byte line rates (L2 / Infinity Cache / HBM)

SOURCES = ["graph_build.cpp", "plan.cpp", "ntp_api.hip", "agg_kernels.hip", "scatter_kernels.hip", "chunk_kernels.hip", "attention_kernels.hip", "attention_scores_kernels.hip", "loss_kernels.hip", "nn_kernels.hip"]
HEADERS = [os.path.join(CSRC, "ntp_internal.h"), os.path.join(CSRC, "lane_util.h"), os.path.join(ROOT, "include", "ntp.h")]

COMMON = ["-O3", "-std=c++17", "-fPIC", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
          "-ffp-contract=off", "-Wall", "-Wno-unused-function"]
# packed fp32 instructions (v_pk_*_f32) are switched off for device code: the compiler must
# not form them from ordinary float arithmetic
DEVICE = ["--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.isabs(c) and os.path.exists(c) or not os.path.isabs(c)):
            return c
    raise RuntimeError("hipcc not found")


def _stale(out: str, deps) -> bool:
    if not os.path.exists(out):
        return True
    t = os.path.getmtime(out)
    return any(os.path.getmtime(d) > t for d in deps)


def build(force: bool = False, verbose: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    hipcc = _hipcc()
    jobs = []
    for s in SOURCES:
        src = os.path.join(CSRC, s)
        obj = os.path.join(OBJ, s + ".o")
        if force or _stale(obj, [src] + HEADERS):
            cmd = [hipcc, "-c", "-x", "hip", src, "-o", obj] + COMMON + DEVICE
            jobs.append(cmd)

    def run(cmd):
        if verbose:
            print(" ".join(cmd), flush=True)
        r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        if r.returncode != 0:
            raise RuntimeError("compile failed:\n%s\n%s" % (" ".join(cmd), r.stdout))
        return r.stdout

    with ThreadPoolExecutor(max_workers=min(8, max(1, len(jobs)))) as ex:
        for out in ex.map(run, jobs):
            if verbose and out.strip():
                print(out)
    objs = [os.path.join(OBJ, s + ".o") for s in SOURCES]
    if force or jobs or _stale(LIB, objs):
        tmp = LIB + ".tmp%d" % os.getpid()
        run([hipcc, "-shared", "-fPIC", "-o", tmp] + objs + ["--offload-arch=gfx950", "-lpthread"])
        os.replace(tmp, LIB)
    # the stand-alone measurement aid (its own executable: it links nothing of the library)
    if force or _stale(PROBE, [PROBE_SRC]):
        tmp = PROBE + ".tmp%d" % os.getpid()
        run([hipcc, "-O3", "-std=c++17", "-ffp-contract=off", "-o", tmp, PROBE_SRC] + DEVICE)
        os.replace(tmp, PROBE)
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv, verbose=True))
