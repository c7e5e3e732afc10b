"""Compile csrc/*.hip into libsparse_attn_hip.so for gfx950 (in-tree, plain hipcc)."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRCS = [os.path.join(HERE, "csrc", n) for n in ("sparse_attn.hip", "sparse_gemm_q.hip", "sparse_gemm_o.hip", "sparse_symbols.hip", "sparse_op_reuse.hip")]
LIB = os.path.join(HERE, "libsparse_attn_hip.so")


def hipcc_path() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    return "hipcc"


def build(verbose: bool = False, extra=()) -> str:
    cmd = [hipcc_path(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-I", os.path.join(ROOT, "include"),
           # packed fp32 VALU forms are kept out of the generated code on purpose
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-o", LIB, *SRCS, *extra]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True, extra=sys.argv[1:]))
