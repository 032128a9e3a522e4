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
SOURCES = ["ptq_api.hip", "hessian.hip", "hessian_f32.hip", "cholesky.hip", "quantize.hip", "vq.hip", "layer_error.hip", "lopro.hip", "r1svd.hip", "r1svd_bf16.hip", "artifact.hip"]
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


def check_dpp_wait_states(asm_text: str) -> int:
    """The leaf kernel of cholesky.hip issues DPP instructions from inline assembly, where the compiler
    does not count wait states: a DPP read needs two (two instructions, or s_nop) after a vector
    instruction wrote the register it reads.  The source keeps that distance by construction; this walks
    the generated assembly and raises if the compiler has put something closer (a copy into an
    accumulator, say).  Returns the number of DPP instructions seen."""
    import re

    def regs(tok):
        m = re.match(r"v\[(\d+):(\d+)\]", tok)
        if m:
            return set(range(int(m.group(1)), int(m.group(2)) + 1))
        m = re.match(r"v(\d+)$", tok)
        return {int(m.group(1))} if m else set()

    lines = [l.strip() for l in asm_text.splitlines()]
    lines = [l for l in lines if l and not l.startswith((";", ".")) and not l.endswith(":")]
    seen = 0
    for i, l in enumerate(lines):
        if "row_newbcast" not in l:
            continue
        seen += 1
        src0 = regs(l.split(None, 1)[1].split(",")[1].split()[0])
        waited, k = 0, i - 1
        while waited < 2 and k >= 0:
            p = lines[k]
            m = re.match(r"s_nop (\d+)", p)
            if m:
                waited += int(m.group(1)) + 1
            else:
                if p.startswith("v_") and regs(p.split(None, 1)[1].split(",")[0].split()[0]) & src0:
                    raise RuntimeError(f"DPP read too close to the write of its source:\n  {p}\n  {l}")
                waited += 1
            k -= 1
    return seen


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

    def check_leaf_assembly():
        cmd = [hipcc, *[f for f in FLAGS if f not in ("-fPIC", "-Wall")], *VGPR_FORM, "-S", "--cuda-device-only",
               os.path.join(CSRC, "cholesky.hip"), "-o", "-"]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc -S failed for cholesky.hip:\n{r.stderr}")
        if check_dpp_wait_states(r.stdout) == 0:
            raise RuntimeError("cholesky.hip: no DPP instruction found in the generated assembly (check out of date?)")

    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES) + 1)) as ex:
        checked = ex.submit(check_leaf_assembly)
        objs = list(ex.map(compile_one, SOURCES))
        checked.result()
    r = subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stdout}\n{r.stderr}")
    # the register-only MFMA probe, a library of its own: one source, compiled in both accumulator forms
    probe_objs = []
    for tag, extra in (("agpr", []), ("vgpr", ["-DPTQ_PROBE_VGPR_FORM", *VGPR_FORM])):
        obj = os.path.join(CSRC, f"probe_mfma_{tag}.o")
        r = subprocess.run([hipcc, *[f for f in FLAGS if f != "-Wall"], *extra, "-c", os.path.join(CSRC, "probe_mfma.hip"),
                            "-o", obj], capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"probe library failed:\n{r.stdout}\n{r.stderr}")
        probe_objs.append(obj)
    r = subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", PROBE_LIB, *probe_objs],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"probe library failed:\n{r.stdout}\n{r.stderr}")
    if verbose:
        print(f"built {LIB}")
    return LIB


if __name__ == "__main__":
    build()
