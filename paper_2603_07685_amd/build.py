"""Builds libmoe_hip.so (the C-ABI library) in-tree with hipcc for gfx950."""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libmoe_hip.so")
SOURCES = ["ctx.hip", "route.hip", "permute.hip", "gemm.hip", "gemm_f32.hip", "fp8.hip"]  # missing files are skipped while the library grows

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
    # packed-fp32 VALU forms are kept off (known-unreliable on the test machines)
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
    # per-kernel register / scratch report on stderr, checked below
    "-Rpass-analysis=kernel-resource-usage",
]
# A kernel that needs more scratch than a handful of spilled registers has had a register array demoted to
# memory (e.g. a loop over the accumulators that silently failed to unroll): orders of magnitude slower and
# reported nowhere else, so the build refuses it.
MAX_SCRATCH_BYTES_PER_LANE = 256


def build_library(verbose: bool = False, jobs: int = 8, extra_flags=(), out: str | None = None) -> str:
    """Compile every csrc/*.hip to an object (in parallel) and link libmoe_hip.so.

    extra_flags / out build a variant library elsewhere (used for kernel tuning experiments)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    bdir = os.path.join(PKG, "_build" if out is None else "_build_" + os.path.basename(out))
    os.makedirs(bdir, exist_ok=True)
    procs = []
    objs = []
    for src in SOURCES:
        path = os.path.join(CSRC, src)
        if not os.path.exists(path):
            continue
        obj = os.path.join(bdir, src.replace(".hip", ".o"))
        objs.append(obj)
        cmd = [hipcc, *HIPCC_FLAGS, *extra_flags, "-c", path, "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        if len(procs) >= jobs:
            _drain(procs, verbose)
    _drain(procs, verbose)
    lib = out or LIB
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", lib]
    subprocess.check_call(cmd)
    if out is None:
        build_ceiling_probe(hipcc)
    return lib


CEILING_LIB = os.path.join(PKG, "libmfma_ceiling.so")


def build_ceiling_probe(hipcc: str) -> str:
    """The register-resident MFMA rate probe bench.py reports beside its numbers: a library of its own (one exported
    function, no part of the layer's C ABI)."""
    flags = [f for f in HIPCC_FLAGS if f != "-Rpass-analysis=kernel-resource-usage"]
    subprocess.check_call([hipcc, *flags, "-shared", os.path.join(CSRC, "mfma_ceiling.hip"), "-o", CEILING_LIB],
                          stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL)
    return CEILING_LIB


def _max_scratch(log: str):
    """(largest ScratchSize [bytes/lane], its kernel) from the compiler's resource-usage remarks."""
    worst, name, cur = 0, "", ""
    for line in log.splitlines():
        if "Function Name:" in line:
            cur = line.split("Function Name:")[1].split("[")[0].strip()
        elif "ScratchSize [bytes/lane]:" in line:
            v = int(line.split("ScratchSize [bytes/lane]:")[1].split("[")[0])
            if v > worst:
                worst, name = v, cur
    return worst, name


def _drain(procs, verbose):
    for src, p in procs:
        out, _ = p.communicate()
        worst = _max_scratch(out)
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l and "kernel-resource-usage" not in l and l.strip())
        if p.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{out}")
        if worst[0] > MAX_SCRATCH_BYTES_PER_LANE:
            raise RuntimeError(f"{src}: kernel {worst[1]} uses {worst[0]} bytes of scratch per lane "
                               f"(limit {MAX_SCRATCH_BYTES_PER_LANE}): a register array went to memory")
        if verbose and out:
            print(out, flush=True)
    procs.clear()


if __name__ == "__main__":
    print(build_library(verbose="-v" in sys.argv))
