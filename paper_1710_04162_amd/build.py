"""Builds libsynk.so (the C-ABI library of HIP kernels for gfx950) in-tree.

    python -m paper_1710_04162_amd.build

hipcc cross-compiles for gfx950 without a GPU.  Objects go to _build/ (not
tracked); the shared library lands next to this file so that it travels with
the source tree.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libsynk.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

# Packed-FP32 instructions are switched off on purpose (device flag only).
FLAGS = ["--offload-arch=gfx950", "-O3", "-fPIC", "-std=c++17", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def sources():
    return sorted(f for f in os.listdir(CSRC) if f.endswith(".hip"))


def _compile(src, obj):
    cmd = [HIPCC] + FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed on %s:\n%s" % (src, err))
    return err


def build_library(verbose=False):
    bdir = os.path.join(ROOT, "_build")
    os.makedirs(bdir, exist_ok=True)
    srcs = sources()
    objs = [os.path.join(bdir, s[:-4] + ".o") for s in srcs]
    with ThreadPoolExecutor(max_workers=min(8, len(srcs))) as ex:
        for s, msg in zip(srcs, ex.map(_compile, srcs, objs)):
            if verbose and msg.strip():
                print(msg, file=sys.stderr)
    tmp = LIB + ".tmp"
    r = subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs,
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    os.replace(tmp, LIB)
    return LIB


def build_oracle_c():
    """Compiles whatever C the oracle holds (none today: it is pure NumPy)."""
    odir = os.path.join(ROOT, "oracle")
    built = []
    for f in sorted(os.listdir(odir)):
        if f.endswith(".c"):
            out = os.path.join(odir, "lib" + f[:-2] + ".so")
            subprocess.run(["gcc", "-O2", "-shared", "-fPIC", "-o", out, os.path.join(odir, f), "-lm"],
                           check=True)
            built.append(out)
    return built


if __name__ == "__main__":
    print(build_library(verbose=True))
