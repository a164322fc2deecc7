"""Builds libsn.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB_DIR = os.path.join(HERE, "lib")
LIB = os.path.join(LIB_DIR, "libsn.so")
OBJ_DIR = os.path.join(HERE, "_build")

SOURCES = ["schedule.cpp", "layout.cpp", "record.cpp", "coord.cpp", "k_elementwise.hip", "k_gemm_skinny.hip", "k_gemm_tile.hip",
           "k_attn_decode.hip", "k_attn_prefill.hip", "runtime.hip", "kernel_abi.hip"]

FLAGS = ["-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


# Per-file additions.  Prefill attention: its accumulators are rescaled by vector code between matrix-core
# products; with the accumulators in the AGPR half of the register file the compiler moves all of them to
# VGPRs and back every step (a quarter of the kernel's instructions), so its MFMAs take the VGPR form.
EXTRA_FLAGS = {"k_attn_prefill.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"],
               # grouped-query decode attention: the same rescale between products, and with its two tiles of K / V
               # in registers it only fits two wavefronts per SIMD without the AGPR copies
               "k_attn_decode.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"]}


def _compile(src: str) -> str:
    obj = os.path.join(OBJ_DIR, os.path.splitext(src)[0] + ".o")
    cmd = ["hipcc", *FLAGS, *EXTRA_FLAGS.get(src, []), "-c", os.path.join(CSRC, src), "-o", obj]
    if src.endswith(".cpp"):
        cmd[1:1] = ["-x", "hip"]
    if src.endswith(".hip"):
        cmd.append("-Rpass-analysis=kernel-resource-usage")
    r = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    lines, spills, name = [], [], "?"
    for l in r.stderr.splitlines():
        if noise in l:
            continue
        if "[-Rpass-analysis=kernel-resource-usage]" in l:
            # keep only what matters: a kernel that spills registers to scratch memory is a
            # performance bug here (every kernel is written to fit its register budget)
            if "Function Name:" in l:
                name = l.split("Function Name:")[1].split()[0]
            elif "ScratchSize [bytes/lane]:" in l and int(l.split("ScratchSize [bytes/lane]:")[1].split()[0]) > 0:
                spills.append(f"{src}: kernel {name} uses "
                              f"{l.split('ScratchSize [bytes/lane]:')[1].split()[0]} bytes/lane of scratch (register spills)")
            continue
        if l.startswith("      |") or l.strip() == "^" or (lines == [] and l[:1].isspace()):
            continue
        lines.append(l)
    err = "\n".join(l for l in lines if not l.lstrip()[:4].strip().isdigit())
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n" + "\n".join(
            l for l in r.stderr.splitlines() if noise not in l and "kernel-resource-usage" not in l))
    if spills:
        sys.stderr.write("WARNING: register spills\n  " + "\n  ".join(spills) + "\n")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose: bool = True) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    os.makedirs(LIB_DIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=8) as ex:
        objs = list(ex.map(_compile, SOURCES))
    cmd = ["hipcc", "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB, *objs, "-lpthread"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    if verbose:
        print(f"built {LIB}")
    return LIB


if __name__ == "__main__":
    build()
