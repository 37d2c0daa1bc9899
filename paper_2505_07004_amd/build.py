"""Build libgq.so (HIP kernels + C ABI) for gfx950, in-tree, with hipcc."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
CSRC = os.path.join(PKG_DIR, "csrc")
INCLUDE = os.path.join(ROOT, "include")
BUILD_DIR = os.path.join(PKG_DIR, "_build")
LIB_PATH = os.path.join(PKG_DIR, "libgq.so")
CEILING_PATH = os.path.join(PKG_DIR, "mfma_ceiling")

SOURCES = [
    "gq_api.hip",
    "gq_noalloc.hip",
    "group_weights.hip",
    "fisher_gram_f32.hip",
    "fisher_gram_bf16.hip",
    "fisher_gram_bf16_wide.hip",
    "heavy_tokens.hip",
    "mirror.hip",
    "objective.hip",
    "cd_assign.hip", "lnq_codebook.hip", "cholesky.hip",
]

HIPCC_FLAGS = [
    "--offload-arch=gfx950",
    "-O3",
    "-std=c++17",
    "-fPIC",
    "-Wall",
    "-Wno-unused-command-line-argument",
    # packed fp32 VALU forms are kept out of generated code on this platform
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def _hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found; libgq can only be built with ROCm's hipcc")
    return exe


def _run(cmd):
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in proc.stdout.splitlines()
                    if "packed-fp32-ops" not in l and "is not a recognized feature" not in l)
    if proc.returncode != 0:
        raise RuntimeError("command failed: %s\n%s" % (" ".join(cmd), out))
    return out


def build(verbose: bool = False, save_temps: bool = False) -> str:
    """Compile every HIP source and link libgq.so.  Always recompiles."""
    os.makedirs(BUILD_DIR, exist_ok=True)
    hipcc = _hipcc()
    # the token loop of the wide bf16 Gram kernel is generated assembly text (an include file)
    _run([sys.executable, os.path.join(CSRC, "gen_gram_wide_loop.py")])
    objs = []
    cmds = []
    for src in SOURCES:
        obj = os.path.join(BUILD_DIR, src.replace(".hip", ".o"))
        objs.append(obj)
        cmd = [hipcc] + HIPCC_FLAGS + ["-I", INCLUDE, "-I", CSRC, "-c", os.path.join(CSRC, src), "-o", obj]
        if save_temps:
            cmd += ["--save-temps=obj"]
        cmds.append(cmd)
    with ThreadPoolExecutor(max_workers=min(8, len(cmds))) as pool:
        for out in pool.map(_run, cmds):
            if verbose and out.strip():
                print(out)
    out = _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB_PATH] + objs)
    if verbose and out.strip():
        print(out)
    # stand-alone measurement of the bf16 MFMA ceiling (run by bench.py as a child process)
    out = _run([hipcc] + HIPCC_FLAGS + [os.path.join(CSRC, "mfma_ceiling.hip"), "-o", CEILING_PATH])
    if verbose and out.strip():
        print(out)
    return LIB_PATH


if __name__ == "__main__":
    print(build(verbose=True, save_temps="--save-temps" in sys.argv))
