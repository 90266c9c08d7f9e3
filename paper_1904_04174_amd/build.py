"""Builds the HIP library (csrc/ -> libconv2d_mi355x.so) for gfx950 with hipcc.

hipcc cross-compiles without a GPU.  Objects go to _build/ (git-ignored); the
shared library stays in-tree next to this file so that it travels with a
snapshot of the repository.
"""
import concurrent.futures
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libconv2d_mi355x.so")
# the ceilings helper (register-only MFMA loop, LDS read loop, copy kernels): a library of its
# own, outside the convolution library's C ABI, loaded only by bench.py --ceilings
CEILINGS_SRC = os.path.join(HERE, "ceilings", "ceilings.hip")
CEILINGS_LIB = os.path.join(HERE, "libconv2d_ceilings.so")
BUILD_DIR = os.path.join(HERE, "_build")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden", "--offload-arch=gfx950",
    # keep the compiler from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-inline-asm", "-Wno-unknown-warning-option",
]


def sources():
    return sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC)
                  if f.endswith(".hip") or f.endswith(".cpp"))


def _deps():
    hdrs = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h") or f.endswith(".inc")]
    hdrs.append(os.path.join(os.path.dirname(HERE), "include", "conv2d.h"))
    hdrs.append(os.path.abspath(__file__))
    return max(os.path.getmtime(h) for h in hdrs)


def _compile(src, force):
    obj = os.path.join(BUILD_DIR, os.path.basename(src) + ".o")
    if (not force and os.path.exists(obj)
            and os.path.getmtime(obj) >= max(os.path.getmtime(src), _deps())):
        return obj
    cmd = [HIPCC] + FLAGS + (["-x", "hip"] if src.endswith(".cpp") else []) + ["-c", src, "-o", obj]
    subprocess.check_call(cmd)
    return obj


def build(force=False, jobs=None):
    """Compile every source and link the shared library.  Returns its path."""
    os.makedirs(BUILD_DIR, exist_ok=True)
    srcs = sources()
    jobs = jobs or min(len(srcs), int(os.environ.get("MAX_JOBS", "8")))
    with concurrent.futures.ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(lambda s: _compile(s, force), srcs))
    tmp = LIB + ".tmp%d" % os.getpid()
    subprocess.check_call([HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", tmp] + objs)
    os.replace(tmp, LIB)
    if (force or not os.path.exists(CEILINGS_LIB)
            or os.path.getmtime(CEILINGS_LIB) < os.path.getmtime(CEILINGS_SRC)):
        tmp = CEILINGS_LIB + ".tmp%d" % os.getpid()
        subprocess.check_call([HIPCC] + FLAGS + ["-shared", CEILINGS_SRC, "-o", tmp])
        os.replace(tmp, CEILINGS_LIB)
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))
