"""Builds libfsrgemm.so (the C-ABI library) in-tree with hipcc for gfx950."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB = os.path.join(_HERE, "libfsrgemm.so")
SOURCES = ("api.hip", "gemm_f32.hip", "gemm_bf16.hip", "gemm_bf16_main.hip", "transpose.hip", "gemv_f32.hip", "gemm_f32_skinny.hip", "gemv_bf16.hip", "gemm_f32_main.hip", "mfma_ceiling.hip")
HIPCC_FLAGS = (
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # packed-fp32 code generation is switched off for every device compile
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
)
# Sources whose kernels issue loads or MFMAs from inline assembly.  The compiler cannot place hazard wait
# states around those, which is safe only while it reloads no spilled register next to them: such kernels
# must compile without spills (checked below from the compiler's own resource-usage remarks).
NO_SPILL_SOURCES = ("gemm_bf16_main.hip", "gemm_f32_main.hip", "gemm_bf16.hip", "mfma_ceiling.hip")
# Every other kernel must at least stay out of scratch memory: a loop the compiler failed to unroll puts a
# kernel's register arrays there, which is correct but many times slower.
KERNEL_SOURCES = ("gemm_f32.hip", "gemm_bf16.hip", "gemm_bf16_main.hip", "transpose.hip", "gemv_f32.hip", "gemm_f32_skinny.hip", "gemv_bf16.hip", "gemm_f32_main.hip", "mfma_ceiling.hip")


def check_no_spills(src: str, remarks: str, scratch_only: bool = False) -> str:
    """Parse hipcc's kernel-resource-usage remarks; raise unless every kernel of `src` is free of spills
    (scratch_only: free of scratch memory; spills into spare registers are tolerated)."""
    import re

    fields = re.findall(r"remark:\s+(Function Name|SGPRs Spill|VGPRs Spill|ScratchSize \[bytes/lane\]):\s*(\S+)", remarks)
    names = [v for k, v in fields if k == "Function Name"]
    if not names:
        raise RuntimeError("no kernel-resource-usage remarks for %s: cannot verify that it compiled without spills" % src)
    bad = [(k, v) for k, v in fields if k != "Function Name" and v != "0" and (not scratch_only or k.startswith("Scratch"))]
    if bad:
        raise RuntimeError("%s must compile without %s, got %s" % (src, "scratch memory" if scratch_only else "register spills", bad))
    return "%d kernel(s), %s" % (len(names), "no scratch" if scratch_only else "no spills, no scratch")


def build_library(verbose: bool = False) -> str:
    """Compile every HIP source and link libfsrgemm.so beside this file."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    bdir = os.path.join(_HERE, "_build")
    os.makedirs(bdir, exist_ok=True)

    def compile_one(src: str) -> str:
        obj = os.path.join(bdir, src.replace(".hip", ".o"))
        cmd = [hipcc, *HIPCC_FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
        if src in KERNEL_SOURCES:
            cmd.insert(-4, "-Rpass-analysis=kernel-resource-usage")
        if verbose:
            print(" ".join(cmd), flush=True)
        r = subprocess.run(cmd, capture_output=True, text=True)
        err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
        if r.returncode != 0:
            raise RuntimeError("hipcc failed on %s:\n%s" % (src, err))
        if src in KERNEL_SOURCES:
            usage = check_no_spills(src, err, scratch_only=src not in NO_SPILL_SOURCES)
            err = "\n".join(l for l in err.splitlines() if "kernel-resource-usage" not in l and l.strip(" |^0123456789{"))
            if verbose:
                print("%s: %s" % (src, usage))
        if verbose and err.strip():
            print(err)
        return obj

    with ThreadPoolExecutor(max_workers=min(5, len(SOURCES))) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    tmp = LIB + ".tmp%d" % os.getpid()
    subprocess.check_call([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs])
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
