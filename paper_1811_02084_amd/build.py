"""Builds libmtf.so (host planner + HIP kernels, gfx950 only) in-tree with hipcc."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
LIB = os.path.join(HERE, "libmtf.so")

SOURCES = ["mtf_host.cpp", "elementwise.hip", "einsum_local.hip", "gemm_bf16.hip", "gemm_bf16_large.hip", "gemm_bf16_small.hip", "gemm_bf16_small_deep.hip",
           "gemm_bf16_split.hip",
           "attention.hip", "attention_unfused.hip", "layer.hip", "timing.hip", "broadcast_reduce.hip", "vocab.hip", "reshape.hip", "layer_norm.hip"]

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wno-inline-asm",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",   # no packed fp32 instructions (unreliable here)
         "-I", INCLUDE, "-I", CSRC]


def build(verbose=True, jobs=8):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    procs = []
    objs = []
    for src in SOURCES:
        path = os.path.join(CSRC, src)
        if not os.path.exists(path):
            continue
        obj = os.path.join(objdir, src + ".o")
        objs.append(obj)
        cmd = [hipcc] + FLAGS + (["-x", "hip"] if src.endswith(".cpp") else []) + ["-c", path, "-o", obj]
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        if len(procs) >= jobs:
            _drain(procs, verbose)
    _drain(procs, verbose)
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    out = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if out.returncode:
        raise RuntimeError("link failed:\n" + out.stdout)
    if verbose:
        print("built", LIB)
    return LIB


def _drain(procs, verbose):
    while procs:
        src, p = procs.pop(0)
        text, _ = p.communicate()
        text = "\n".join(l for l in text.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode:
            raise RuntimeError(f"compiling {src} failed:\n{text}")
        if verbose and text.strip():
            print(text)


if __name__ == "__main__":
    build()
    sys.exit(0)
