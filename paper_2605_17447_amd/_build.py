"""Builds libfastocr.so (hand-written HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
LIB = os.path.join(HERE, "libfastocr.so")
SOURCES = ["api.hip", "attn.hip", "score.hip", "score_resident.hip", "focal_fused.hip", "topk.hip", "probe.hip"]

# Packed-FP32 VALU forms are switched off for all device code (they have given silently wrong
# results on these machines); hipcc's host pass does not know the feature and says so.
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument", "-I", INCLUDE, "-I", CSRC]


# Host code only under AddressSanitizer and UndefinedBehaviorSanitizer (the device code is built as
# always): a checking build for the CPU-only tests of the argument validation, never the product.
HOST_SANITIZE = ["-g", "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                 "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer"]
LIB_HOSTSAN = os.path.join(HERE, "libfastocr_hostsan.so")


def build(verbose: bool = False, host_sanitize: bool = False) -> str:
    """Compile every source and link the shared library; returns its path."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = []
    procs = []
    flags = FLAGS + (HOST_SANITIZE if host_sanitize else [])
    lib = LIB_HOSTSAN if host_sanitize else LIB
    for src in SOURCES:
        obj = os.path.join(CSRC, src.replace(".hip", ".san.o" if host_sanitize else ".o"))
        cmd = [hipcc, *flags, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    failed = False
    for src, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "is not a recognized feature for this target" not in l)
        if p.returncode != 0:
            failed = True
            sys.stderr.write(f"--- {src} failed ---\n{out}\n")
        elif verbose and out.strip():
            print(out)
    if failed:
        raise RuntimeError("hipcc failed")
    tmp = lib + f".tmp{os.getpid()}"
    link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs]
    if host_sanitize:
        link += ["-fsanitize=address", "-fsanitize=undefined", "-shared-libsan"]
    subprocess.check_call(link)
    os.replace(tmp, lib)
    return lib


if __name__ == "__main__":
    print(build(verbose=True))
