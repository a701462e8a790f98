"""Build the gfx950 shared library in-tree with hipcc.

``python -m paper_2502_07864_amd.build`` compiles every ``csrc/*.hip`` for
gfx950 and links ``libmla_gfx950.so`` next to this file.  hipcc
cross-compiles, so this works on a machine without a GPU.
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor
from pathlib import Path

PKG = Path(__file__).resolve().parent
CSRC = PKG / "csrc"
INCLUDE = PKG.parent / "include"
OBJDIR = PKG / "_build"
LIB = PKG / "libmla_gfx950.so"

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
    "-Wall", "-Wno-unused-function",
    # never let the compiler form packed-fp32 VALU ops
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    f"-I{INCLUDE}", f"-I{CSRC}",
]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not Path(exe).exists():
        raise RuntimeError("hipcc not found (need ROCm to build the gfx950 library)")
    return exe


def sources():
    return sorted(CSRC.glob("*.hip"))


def build_library(verbose: bool = False, extra_flags=()) -> Path:
    OBJDIR.mkdir(exist_ok=True)
    cc = hipcc()

    def compile_one(src: Path) -> Path:
        obj = OBJDIR / (src.stem + ".o")
        cmd = [cc, *HIPCC_FLAGS, *extra_flags, "-c", str(src), "-o", str(obj)]
        r = subprocess.run(cmd, capture_output=True, text=True)
        out = "\n".join(l for l in (r.stdout + r.stderr).splitlines()
                        if "packed-fp32-ops" not in l and "target feature" not in l)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src.name}:\n{r.stdout}{r.stderr}")
        if verbose and out.strip():
            print(out)
        return obj

    def check_pending_registers() -> None:
        # decode_mfma.hip's query rows: loads with register outputs awaited later by count (asm_checks.py)
        from .asm_checks import check_listing
        src = CSRC / "decode_mfma.hip"
        asm = OBJDIR / "decode_mfma.s"
        cmd = [cc, *HIPCC_FLAGS, *extra_flags, "-S", "--cuda-device-only", str(src), "-o", str(asm)]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc -S failed on {src.name}:\n{r.stdout}{r.stderr}")
        seen = check_listing(asm.read_text(), "decode_mfma_kernel")
        if not seen or not all(seen.values()):
            raise RuntimeError(f"asm check found no query-row loads to look at in {sorted(seen)}")

    with ThreadPoolExecutor(max_workers=min(4, os.cpu_count() or 1)) as ex:
        check = ex.submit(check_pending_registers)
        objs = list(ex.map(compile_one, sources()))
        check.result()
    tmp = LIB.with_suffix(".so.tmp")
    cmd = [cc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", str(tmp), *map(str, objs)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stdout}{r.stderr}")
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose="-v" in sys.argv))
