"""Builds libmemo.so (the C-ABI library) in-tree with hipcc for gfx950."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libmemo.so")
# measurement aids of bench.py (an MFMA-only probe, an atomic-add probe): a library of their own, not part of libmemo
BENCH_AIDS_SRC = [os.path.join(HERE, "bench_aids", "probe_mfma.hip"), os.path.join(HERE, "bench_aids", "atomic_add.hip")]
BENCH_AIDS_LIB = os.path.join(HERE, "bench_aids", "libmemo_bench_aids.so")
# source -> extra flags.  Every file keeps IEEE NaN semantics: a NaN or Inf in an input must reach
# the outputs that depend on it (a training loop detects divergence that way).
SOURCES = {
    "memo_api.cpp": [],
    "memo_sched.cpp": [],
    "memo_dsa.cpp": [],
    "attn_f32.hip": [],
    "attn_bf16.hip": [],
    "attn_bwd_bf16.hip": [],
    "attn_bwd_static.hip": [],
    "recompute_bf16.hip": [],
}
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-x", "hip",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-command-line-argument"]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass warns that it does not know the packed-fp32 feature: harmless, filtered
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err, file=sys.stderr)


def build(verbose=False, extra=()):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)
    objs = []
    for src, flags in SOURCES.items():
        obj = os.path.join(OBJ, src + ".o")
        _run([hipcc] + FLAGS + flags + list(extra) + ["-c", os.path.join(CSRC, src), "-o", obj], verbose)
        objs.append(obj)
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs, verbose)
    return LIB


def build_bench_aids(verbose=False):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    _run([hipcc] + FLAGS + ["-shared"] + BENCH_AIDS_SRC + ["-o", BENCH_AIDS_LIB], verbose)
    return BENCH_AIDS_LIB


if __name__ == "__main__":
    build(verbose=True, extra=sys.argv[1:])
    build_bench_aids(verbose=True)
    print("built", LIB, BENCH_AIDS_LIB)
