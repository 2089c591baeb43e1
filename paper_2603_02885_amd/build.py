"""Compiles the HIP library for gfx950 in-tree (hipcc cross-compiles without a GPU)."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB_PATH = os.path.join(HERE, "libmuxlora.so")
SOURCES = ["mux_segtab.cpp", "mux_api.hip", "mux_ref_kernels.hip", "mux_fast_kernels.hip", "mux_gemm_mfma.hip", "mux_profile.cpp", "mux_adapter_mfma.hip", "mux_gemm_dma.hip", "mux_diff_kernels.hip", "mux_planner.cpp", "mux_attn.hip", "mux_dispatch.hip", "mux_probe.hip", "mux_mask.cpp"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function", "-Wno-unknown-warning-option", "-Wno-inline-asm"]


def build_library(verbose: bool = False, jobs: int = 4) -> str:
    csrc = os.path.join(HERE, "csrc")
    inc = ["-I", os.path.join(ROOT, "include"), "-I", csrc]
    bdir = os.path.join(HERE, "_build")
    os.makedirs(bdir, exist_ok=True)
    procs = []
    objs = []
    for src in SOURCES:
        obj = os.path.join(bdir, src + ".o")
        objs.append(obj)
        cmd = [HIPCC, "-x", "hip", "-c", os.path.join(csrc, src), "-o", obj] + FLAGS + inc
        if verbose:
            print(" ".join(cmd))
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)))
        if len(procs) >= jobs:
            _drain(procs)
    _drain(procs)
    tmp = LIB_PATH + f".tmp{os.getpid()}"
    subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs)
    os.replace(tmp, LIB_PATH)
    return LIB_PATH


def _drain(procs):
    while procs:
        src, p = procs.pop(0)
        out = p.communicate()[0].decode()
        lines = [l for l in out.splitlines() if "packed-fp32-ops" not in l]
        if p.returncode != 0:
            sys.stderr.write(out)
            raise RuntimeError(f"hipcc failed on {src}")
        if any("warning" in l or "error" in l for l in lines):
            sys.stderr.write("\n".join(lines) + "\n")


if __name__ == "__main__":
    print(build_library(verbose="-v" in sys.argv))
