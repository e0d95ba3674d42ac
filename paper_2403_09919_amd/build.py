"""Builds the HIP library (librd.so) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "librd.so")
SOURCES = ["rd_api.hip", "rd_dedup.hip", "rd_tree_attn.hip", "rd_tree_attn_bf16.hip",
           "rd_tree_attn_f16.hip", "rd_tree_attn_paged.hip", "rd_tree_attn_rope_bf16.hip", "rd_tree_attn_rope_f16.hip", "rd_tree_attn_f32.hip", "rd_accept.hip", "rd_accept_sample.hip", "rd_commit.hip", "rd_rope.hip", "rd_draft.hip"]
# -packed-fp32-ops is switched off for device code on purpose (hipcc's host pass does not
# know the feature and says so; that message is filtered below).
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function", "-Wno-unknown-attributes"]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l and l.strip())
    if res.returncode != 0:
        raise RuntimeError("hipcc failed: %s\n%s" % (" ".join(cmd), out))
    if verbose and out:
        print(out, flush=True)


def build(verbose: bool = False, extra_flags=()) -> str:
    """Compile every kernel source and link paper_2403_09919_amd/librd.so (always recompiles)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)
    inc = ["-I", os.path.join(ROOT, "include"), "-I", CSRC]
    objs = [os.path.join(OBJ, s.replace(".hip", ".o")) for s in SOURCES]
    jobs = [[hipcc, *FLAGS, *extra_flags, *inc, "-c", os.path.join(CSRC, s), "-o", o]
            for s, o in zip(SOURCES, objs)]
    with ThreadPoolExecutor(max_workers=min(8, len(jobs))) as ex:
        list(ex.map(lambda c: _run(c, verbose), jobs))
    tmp = LIB + ".tmp%d" % os.getpid()
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", tmp], verbose)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True, extra_flags=sys.argv[1:]))
