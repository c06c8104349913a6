"""Builds libdpstage.so (hipcc, gfx950) in-tree next to this file."""
from __future__ import annotations

import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libdpstage.so")
SOURCES = ["stage.cpp", "planner.cpp", "ops.cpp", "elementwise.hip", "gemm_simple.hip", "attn_simple.hip", "gemm_mfma.hip", "gemm_dma.hip", "attn_mfma.hip", "probe.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-x", "hip",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument"]


# Kernels that issue global loads through inline asm and count them by hand must not
# spill: a spill store placed by the compiler right behind such a load would save the
# register before the data has arrived.
NO_SCRATCH = {"gemm_mfma.hip", "gemm_dma.hip"}

# Per-file compiler options.  attn_mfma.hip: with head dimension 128 the backward kernels keep
# 128 accumulator registers per wave beside 64 operand registers; by default the compiler puts
# the matrix instructions' results into accumulation registers and then moves them to and fro
# (768 v_accvgpr moves for 128 matrix instructions in the dK/dV loop); letting it choose ordinary
# registers for them removes nearly all of those moves.
EXTRA_FLAGS = {"attn_mfma.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form", "-Wno-inline-asm"],
               # the LDS-direct load names M0 as clobbered; clang warns that M0 is a reserved register
               "gemm_dma.hip": ["-Wno-inline-asm"]}


# Files whose inline asm writes M0 (the LDS-direct loads).  The asm declares the clobber, but M0 is a reserved
# register the compiler also uses by itself (LDS-indexed operations, lane moves, spill code) without modelling
# inline asm's writes: such a use next to the loads would be a silent miscompile.  The device assembly of these
# files must therefore name M0 only inside the inline asm blocks.
M0_BY_HAND = {"gemm_dma.hip", "attn_mfma.hip"}


def _check_m0(src: str) -> None:
    asm = os.path.join(OBJ, os.path.splitext(src)[0] + ".s")
    cmd = [HIPCC, *FLAGS, *EXTRA_FLAGS.get(src, []), "-S", "--cuda-device-only", os.path.join(CSRC, src), "-o", asm]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc -S failed for {src}:\n{r.stderr}")
    inside = False
    with open(asm) as f:
        for n, line in enumerate(f, 1):
            if "#ASMSTART" in line:
                inside = True
            elif "#ASMEND" in line:
                inside = False
            elif not inside:
                code = line.split(";", 1)[0]
                if re.search(r"\bm0\b", code):
                    raise RuntimeError(f"{src}: the compiler uses M0 outside the inline asm ({asm}:{n}: {line.strip()})")
    os.remove(asm)


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    extra = ["-Rpass-analysis=kernel-resource-usage"] if src in NO_SCRATCH else []
    cmd = [HIPCC, *FLAGS, *extra, *EXTRA_FLAGS.get(src, []), "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    lines = r.stderr.splitlines()
    if src in NO_SCRATCH and r.returncode == 0:
        name = "?"
        for l in lines:
            if "Function Name:" in l:
                name = l.split("Function Name:")[1].split()[0]
            if "ScratchSize [bytes/lane]:" in l and int(l.split("ScratchSize [bytes/lane]:")[1].split()[0]) != 0:
                raise RuntimeError(f"{src}: kernel {name} uses scratch memory (register spills are not allowed here)")
        # the remarks echo source lines; keep only real diagnostics
        keep, show = [], False
        for l in lines:
            if "remark:" in l:
                show = False
            elif "warning:" in l or "error:" in l:
                show = True
            if show:
                keep.append(l)
        lines = keep
    err = "\n".join(l for l in lines if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    if src in M0_BY_HAND:
        _check_m0(src)
    return obj


def build(verbose: bool = True) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(_compile, SOURCES))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    if verbose:
        print("built", LIB)
    return LIB


HOST_SOURCES = ["stage.cpp", "planner.cpp", "ops.cpp", "host_check.cpp"]
SANITIZERS = {"asan": "address,undefined", "tsan": "thread"}


def build_host_check(kind: str = "asan") -> str:
    """The library's host code (step walk and validator, planners, operator wrappers) compiled with host-side
    sanitizers -- AddressSanitizer + UBSan ("asan") or ThreadSanitizer ("tsan", for the planner's worker threads)
    -- and linked with csrc/host_check.cpp into an executable that drives the pure host entry points.  The device
    code is the ordinary build's; nothing in the executable touches a GPU."""
    san = SANITIZERS[kind]
    os.makedirs(OBJ, exist_ok=True)
    dev_objs = [os.path.join(OBJ, os.path.splitext(src)[0] + ".o") for src in SOURCES if src.endswith(".hip")]
    if not all(os.path.exists(o) for o in dev_objs):
        build(verbose=False)
    objs = []
    for src in HOST_SOURCES:
        obj = os.path.join(OBJ, f"{os.path.splitext(src)[0]}.{kind}.o")
        cmd = [HIPCC, *FLAGS, "-g", "-fno-omit-frame-pointer", "-Xarch_host", f"-fsanitize={san}",
               "-c", os.path.join(CSRC, src), "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc ({kind}) failed for {src}:\n{r.stderr}")
        objs.append(obj)
    exe = os.path.join(OBJ, f"host_check_{kind}")
    cmd = [HIPCC, "--offload-arch=gfx950", f"-fsanitize={san}", "-fno-gpu-sanitize", "-o", exe, *objs, *dev_objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link ({kind}) failed:\n" + r.stderr)
    return exe


if __name__ == "__main__":
    if len(sys.argv) > 1 and sys.argv[1] in SANITIZERS:
        print(build_host_check(sys.argv[1]))
    else:
        build()
