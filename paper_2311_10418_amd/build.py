"""Build the HIP library (libdynastage.so) for gfx950, in-tree.

    python -m paper_2311_10418_amd.build        # compile what changed
    python -m paper_2311_10418_amd.build --force
"""
import concurrent.futures
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libdynastage.so")

HIP_SOURCES = ["elementwise.hip", "gemm.hip", "attention_generic.hip", "attention_mfma.hip", "attention_api.hip", "stage.hip", "probe.hip"]
CPP_SOURCES = ["planner.cpp", "schedule.cpp", "recompute.cpp"]

HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function", "-Wno-inline-asm",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
CXX_FLAGS = ["-O2", "-std=c++17", "-fPIC", "-Wall", "-Wextra", "-ffp-contract=off"]


def _deps_newer(obj):
    if not os.path.exists(obj):
        return True
    t = os.path.getmtime(obj)
    for root in (CSRC, os.path.join(HERE, "..", "include")):
        for f in os.listdir(root):
            if os.path.getmtime(os.path.join(root, f)) > t:
                return True
    return False


def _compile(args):
    src, force = args
    obj = os.path.join(OBJ, src + ".o")
    if not force and not _deps_newer(obj):
        return src, 0, ""
    if src.endswith(".hip"):
        cmd = ["hipcc"] + HIPCC_FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj]
    else:
        cmd = ["g++"] + CXX_FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj]
    p = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in p.stderr.splitlines() if "packed-fp32-ops" not in l)
    return src, p.returncode, err


def build(force=False, jobs=8):
    os.makedirs(OBJ, exist_ok=True)
    srcs = HIP_SOURCES + CPP_SOURCES
    with concurrent.futures.ThreadPoolExecutor(max_workers=jobs) as ex:
        results = list(ex.map(_compile, [(s, force) for s in srcs]))
    for src, rc, err in results:
        if err.strip():
            sys.stderr.write("[%s]\n%s\n" % (src, err))
        if rc != 0:
            raise RuntimeError("compilation of %s failed" % src)
    objs = [os.path.join(OBJ, s + ".o") for s in srcs]
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    p = subprocess.run(cmd, capture_output=True, text=True)
    if p.returncode != 0:
        sys.stderr.write(p.stderr)
        raise RuntimeError("link failed")
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))
