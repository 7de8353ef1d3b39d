"""Builds libtsd.so (the C-ABI library) for gfx950 with hipcc, in-tree.

    python -m paper_2511_18191_amd.build

Cross-compiles without a GPU.  Objects go to paper_2511_18191_amd/_build/, the library to
paper_2511_18191_amd/libtsd.so.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OUT = os.path.join(HERE, "libtsd.so")
SOURCES = ["tsd_api.hip", "gemm.hip", "gemm_skinny.hip", "attn.hip", "misc.hip", "moe.hip", "draft_fused.hip", "accept_static.hip", "gemm_wide.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-I", os.path.join(ROOT, "include"), "-I", CSRC,
         # packed-fp32 instruction selection is switched off on purpose for the test machines
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # no implicit FMA contraction: a*b + c is fused only where the source says fmaf(), so the
         # rounding of a row's arithmetic cannot depend on which unrolled copy of a loop body it met
         "-ffp-contract=off",
         "-Wno-unused-command-line-argument"]


def _run(cmd):
    r = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in r.stderr.splitlines() if noise not in l)
    if r.returncode != 0:
        raise RuntimeError("command failed: " + " ".join(cmd) + "\n" + r.stdout + err)
    return err


def build(verbose=True):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    bdir = os.path.join(HERE, "_build")
    os.makedirs(bdir, exist_ok=True)
    objs = [os.path.join(bdir, s.replace(".hip", ".o")) for s in SOURCES]

    def one(pair):
        src, obj = pair
        return _run([hipcc, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj])

    with ThreadPoolExecutor(max_workers=min(4, os.cpu_count() or 1)) as ex:
        for src, warn in zip(SOURCES, ex.map(one, zip(SOURCES, objs))):
            if verbose and warn.strip():
                print(f"[{src}]\n{warn}", file=sys.stderr)
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", OUT])
    if verbose:
        print("built", OUT)
    return OUT


if __name__ == "__main__":
    build()
