"""Builds libmlra.so (HIP, gfx950 only) in-tree with hipcc.

    python -m paper_2603_02188_amd.build

Objects go to paper_2603_02188_amd/_build/, the library to paper_2603_02188_amd/libmlra.so.
hipcc cross-compiles for gfx950 without a GPU.
"""
from __future__ import annotations

import glob
import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

try:
    from .check_isa import find_overlaps, find_reserved_acc_uses
except ImportError:  # run as a script
    from check_isa import find_overlaps, find_reserved_acc_uses

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
LIB = os.path.join(PKG, "libmlra.so")

HIP_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",   # keep packed-fp32 VALU forms out
    "-mllvm", "-amdgpu-mfma-vgpr-form",   # MFMA results in VGPRs: AGPRs are left to the pinned query operands
    "-Wno-unused-command-line-argument",
]


def _hipcc() -> str:
    cand = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(cand):
        raise RuntimeError("hipcc not found; libmlra needs ROCm's hipcc to build")
    return cand


def _run(cmd):
    p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(ln for ln in p.stdout.splitlines() if "packed-fp32-ops" not in ln)
    if p.returncode != 0:
        raise RuntimeError("command failed: " + " ".join(cmd) + "\n" + out)
    return out


def build(verbose: bool = False, jobs: int = 8) -> str:
    hipcc = _hipcc()
    bdir = os.path.join(PKG, "_build")
    os.makedirs(bdir, exist_ok=True)
    srcs = sorted(glob.glob(os.path.join(PKG, "csrc", "*.hip")))
    inc = ["-I", os.path.join(ROOT, "include"), "-I", os.path.join(PKG, "csrc")]
    objs = [os.path.join(bdir, os.path.basename(s)[:-4] + ".o") for s in srcs]

    def compile_one(so):
        src, obj = so
        out = _run([hipcc, *HIP_FLAGS, *inc, "-DMLRA_BUILDING", "-c", src, "-o", obj])
        if verbose and out.strip():
            print(out)
        # device assembly of the same translation unit, scanned for MFMA register overlaps
        asm = obj[:-2] + ".s"
        _run([hipcc, *HIP_FLAGS, *inc, "-DMLRA_BUILDING", "--cuda-device-only", "-S", src, "-o", asm])
        text = open(asm).read()
        bad = find_overlaps(text)
        if bad:
            raise RuntimeError(f"{src}: MFMA destination overlaps a source operand:\n" +
                               "\n".join(f"  {asm}:{ln}: {text}" for ln, text in bad))
        # the decode kernel's value accumulators (a0..a135) belong to its inline asm alone
        bad = find_reserved_acc_uses(text, r"decode_mfma_kernel", 136)
        if bad:
            raise RuntimeError(f"{src}: compiler-generated code touches the reserved accumulation registers:\n" +
                               "\n".join(f"  {asm}:{ln}: {text}" for ln, text in bad[:20]))
        return obj

    with ThreadPoolExecutor(max_workers=max(1, min(jobs, len(srcs)))) as ex:
        list(ex.map(compile_one, zip(srcs, objs)))
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs])
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
