"""Compile the HIP sources in csrc/ into paper_2504_19442_amd/libagg.so for gfx950 with hipcc."""
from __future__ import annotations

import glob
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libagg.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

# -packed-fp32-ops off: the compiler must not form packed fp32 instructions on the test machines.
# -amdgpu-spill-vgpr-to-agpr=0: the GEMM kernel keeps its accumulators in accumulator registers the compiler
# does not know about, so the compiler must never park values of its own there (check_agprs verifies it).
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-inline-asm",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-mllvm", "-amdgpu-spill-vgpr-to-agpr=0"]


def check_agprs(asm_path: str) -> None:
    """Fail if, in the device assembly of a GEMM translation unit, the compiler itself touches an accumulator register
    (any a<N> outside the inline-asm blocks), or if a kernel spills to scratch."""
    import re
    in_asm = False
    pat = re.compile(r"(?<![A-Za-z0-9_.])a(\[\d+(:\d+)?\]|\d+\b)")
    with open(asm_path) as f:
        for n, line in enumerate(f, 1):
            t = line.strip()
            if t.startswith(";;#ASMSTART"):
                in_asm = True
            elif t.startswith(";;#ASMEND"):
                in_asm = False
            elif not in_asm and not t.startswith(";") and not t.startswith("."):
                code = t.split(";")[0]
                if pat.search(code):
                    raise RuntimeError(f"compiler-allocated accumulator register in {asm_path} (line {n}): {t}")
            if t.startswith("; ScratchSize:") and t.split(":")[1].strip() != "0":
                raise RuntimeError(f"a GEMM kernel spills to scratch ({asm_path}): {t}")


def _is_gemm_unit(src: str) -> bool:
    return os.path.basename(src).startswith("gemm_inst_")


def _compile(src: str) -> str:
    base = os.path.basename(src)
    obj = os.path.join(OBJ, base + ".o")
    asm = os.path.join(OBJ, base[:-4] + "-hip-amdgcn-amd-amdhsa-gfx950.s")
    deps = [src] + glob.glob(os.path.join(CSRC, "*.h")) + [os.path.join(HERE, "..", "include", "agg.h")]
    fresh = os.path.exists(obj) and all(os.path.getmtime(obj) >= os.path.getmtime(d) for d in deps) \
        and os.environ.get("AGG_FORCE_BUILD") != "1"
    if not fresh:
        # the GEMM units keep their device assembly (-save-temps) for the accumulator-register check below
        extra = ["-save-temps=obj"] if _is_gemm_unit(src) else []
        r = subprocess.run([HIPCC, *FLAGS, *extra, "-c", src, "-o", obj], capture_output=True, text=True, cwd=OBJ)
        err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{err}")
        if err.strip():
            sys.stderr.write(err + "\n")
    if _is_gemm_unit(src):
        check_agprs(asm)
    return obj


def build(force: bool = True) -> str:
    os.makedirs(OBJ, exist_ok=True)
    if force:
        os.environ["AGG_FORCE_BUILD"] = "1"
    try:
        srcs = sorted(glob.glob(os.path.join(CSRC, "*.hip")))
        with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 4)) as ex:
            objs = list(ex.map(_compile, srcs))
    finally:
        os.environ.pop("AGG_FORCE_BUILD", None)
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB + ".tmp"], check=True)
    os.replace(LIB + ".tmp", LIB)
    return LIB


if __name__ == "__main__":
    print(build(force="--if-stale" not in sys.argv))
