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


def build_host_sanitized(out_dir: str, verbose: bool = False):
    """The library's HOST code -- argument checks, launch plans, workspace sizing -- compiled with
    clang's address and undefined-behaviour sanitizers, for tests that drive the argument-error paths of
    the C ABI under them.  Only the host pass is compiled (seconds); the device images that the host
    objects refer to are replaced by empty stand-ins, so NOTHING in this library can be launched: it
    is for calls that return before a launch, in a process without a GPU.
    Returns (library path, path of the sanitizer runtime that the loading process must preload)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(out_dir, exist_ok=True)
    inc = ["-I", os.path.join(ROOT, "include"), "-I", CSRC]
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer"]
    objs = [os.path.join(out_dir, s.replace(".hip", ".host.o")) for s in SOURCES]
    jobs = [[hipcc, "--offload-arch=gfx950", "--cuda-host-only", "-O1", "-g", "-std=c++17", "-fPIC", *san, *inc,
             "-Wno-unused-function", "-Wno-unknown-attributes", "-c", os.path.join(CSRC, s), "-o", o]
            for s, o in zip(SOURCES, objs)]
    with ThreadPoolExecutor(max_workers=min(8, len(jobs))) as ex:
        list(ex.map(lambda c: _run(c, verbose), jobs))
    # stand-ins for the device images (one symbol per translation unit, named by the compiler)
    nm = subprocess.run(["nm", *objs], stdout=subprocess.PIPE, text=True, check=True).stdout
    syms = sorted({l.split()[-1] for l in nm.splitlines() if " U __hip_fatbin_" in l})
    stub = os.path.join(out_dir, "fatbin_stub.c")
    with open(stub, "w") as f:
        for sym in syms:
            f.write("const unsigned char %s[64] __attribute__((aligned(4096))) = {0};\n" % sym)
    stub_o = os.path.join(out_dir, "fatbin_stub.o")
    _run(["gcc", "-c", "-fPIC", stub, "-o", stub_o], verbose)
    lib = os.path.join(out_dir, "librd_hostsan.so")
    _run([hipcc, "--offload-arch=gfx950", "--cuda-host-only", "-shared", "-fPIC", "-fsanitize=address", "-fsanitize=undefined",
          "-shared-libsan", *objs, stub_o, "-o", lib], verbose)
    rt = subprocess.run([hipcc, "--offload-arch=gfx950", "-print-file-name=libclang_rt.asan-x86_64.so"],
                        stdout=subprocess.PIPE, text=True).stdout.strip()
    return lib, rt


if __name__ == "__main__":
    print(build(verbose=True, extra_flags=sys.argv[1:]))
