"""Builds libvispec_verify.so (gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libvispec_verify.so")
SOURCES = ["api.hip", "tree_mask.hip", "attention_generic.hip", "attention_mfma.hip", "attention_mfma_pipe.hip", "attention_mfma_resident.hip", "accept.hip", "accept_sample.hip", "draft_tree.hip",
           "kv_commit.hip", "peaks.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument",
         "-I" + os.path.join(ROOT, "include"), "-I" + CSRC]


# host code under AddressSanitizer and UndefinedBehaviorSanitizer (device code is untouched)
SAN_FLAGS = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
             "-fno-sanitize-recover=all", "-g"]
SAN_LIB = os.path.join(HERE, "libvispec_verify_san.so")


def build_library(verbose: bool = False, extra=(), sanitize_host: bool = False) -> str:
    """Compile every HIP source into one shared library. Always recompiles.
    sanitize_host: build libvispec_verify_san.so instead, its host code instrumented; run it with
    the compiler's own sanitizer runtime preloaded (Python is not instrumented):
        RT=$(/opt/rocm/lib/llvm/bin/clang -print-file-name=libclang_rt.asan-x86_64.so)
        VISPEC_VERIFY_LIB=$PWD/paper_2509_15235_amd/libvispec_verify_san.so ASAN_OPTIONS=detect_leaks=0 \
        LD_PRELOAD=$RT LD_LIBRARY_PATH=$(dirname $RT) python -m pytest tests/test_boundary.py"""
    objs = []
    procs = []
    bdir = os.path.join(HERE, "_build_san" if sanitize_host else "_build")
    if sanitize_host:
        extra = list(extra) + SAN_FLAGS
    os.makedirs(bdir, exist_ok=True)
    for src in SOURCES:
        obj = os.path.join(bdir, src.replace(".hip", ".o"))
        cmd = [HIPCC, "-c"] + [f for f in FLAGS if f != "-shared"] + list(extra) + \
              [os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    failed = False
    for src, pr in procs:
        out, _ = pr.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if pr.returncode != 0:
            failed = True
            print(f"[build] {src} FAILED\n{out}", file=sys.stderr)
        elif verbose and out.strip():
            print(out)
    if failed:
        raise RuntimeError("hipcc failed")
    out = SAN_LIB if sanitize_host else LIB
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", out] + objs
    if sanitize_host:
        cmd += ["-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize", "-shared-libsan"]
    subprocess.check_call(cmd)
    return out


if __name__ == "__main__":
    print(build_library(verbose=True, sanitize_host="--sanitize-host" in sys.argv))
