"""Builds libptq.so (the C-ABI library of hand-written gfx950 kernels) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libptq.so")
PROBE_LIB = os.path.join(HERE, "libptq_probe.so")   # diagnostics for bench.py --mfma-control, not part of the product
SOURCES = ["ptq_api.hip", "hessian.hip", "cholesky.hip", "quantize.hip", "vq.hip", "layer_error.hip", "lopro.hip", "r1svd.hip", "r1svd_bf16.hip", "artifact.hip"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-result",
    # packed-FP32 instructions are kept out of every kernel
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]
# Accumulators of the float64 matrix instructions stay in ordinary VGPRs (those kernels fit
# 256 registers, and the AGPR form costs copies around each MFMA).  The bf16 Hessian kernel
# needs all 256 AGPRs for its accumulators and is compiled without the option.
VGPR_FORM = ["-mllvm", "-amdgpu-mfma-vgpr-form"]
NO_VGPR_FORM = {"hessian.hip"}


def _hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.isabs(c) and os.path.exists(c) or not os.path.isabs(c)):
            return c
    raise RuntimeError("hipcc not found")


def build(verbose: bool = True) -> str:
    """Compiles every source (always, also when a library is already there) and links."""
    hipcc = _hipcc()
    objs = []

    def compile_one(src):
        obj = os.path.join(CSRC, src.replace(".hip", ".o"))
        extra = [] if src in NO_VGPR_FORM else VGPR_FORM
        cmd = [hipcc, *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed for {src}:\n{r.stdout}\n{r.stderr}")
        errs = [l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l and l.strip()]
        if verbose and any("warning" in l for l in errs):
            print("\n".join(errs), file=sys.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    r = subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stdout}\n{r.stderr}")
    # the register-only MFMA probe, a library of its own
    r = subprocess.run([hipcc, *[f for f in FLAGS if f != "-Wall"], "-shared", os.path.join(CSRC, "probe_mfma.hip"), "-o",
                        PROBE_LIB], capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"probe library failed:\n{r.stdout}\n{r.stderr}")
    if verbose:
        print(f"built {LIB}")
    return LIB


if __name__ == "__main__":
    build()
