"""Build libctcspec.so (the C-ABI library of HIP kernels) for gfx950, in-tree.

    python -m paper_2412_00061_amd.build

hipcc cross-compiles without a GPU.  The library lands next to this file so that it travels with
the source tree; nothing is installed anywhere else.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SOURCES = ["context.hip", "draft_topk.hip", "collapse_tree.hip", "tree_attn.hip", "accept.hip", "verify_head.hip", "draft_layer.hip", "sum_score.hip", "ctc_loss.hip", "verify_sample.hip"]
LIB = os.path.join(HERE, "libctcspec.so")

HIPCC_FLAGS = [
    "-O3", "-std=c++20", "--offload-arch=gfx950", "-fPIC", "-shared",
    # keep the compiler from emitting packed fp32 VALU ops
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-unused-command-line-argument",
]


def build(verbose: bool = True) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + HIPCC_FLAGS + ["-I", os.path.join(ROOT, "include"), "-I", os.path.join(HERE, "csrc")]
    cmd += [os.path.join(HERE, "csrc", s) for s in SOURCES] + ["-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    out = "\n".join(l for l in (res.stdout + res.stderr).splitlines()
                    if "packed-fp32-ops" not in l and l.strip())
    if verbose and out:
        print(out, flush=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    return LIB


if __name__ == "__main__":
    build()
    sys.exit(0)
