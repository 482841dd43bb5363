"""Builds libw2v_shard.so (HIP kernels + C ABI) for gfx950, in tree, with hipcc.

Usage: ``python -m paper_1606_08495_amd.build`` or ``build()`` from Python.  Objects go to
``_build/`` (not tracked); the shared library lands next to this file so that it travels with the
source tree.  hipcc cross-compiles without a GPU.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libw2v_shard.so")

HIP_SOURCES = ["api.hip", "k_gather.hip", "k_sort.hip", "k_adjust.hip", "k_pairs.hip", "k_cbow.hip", "k_topk.hip"]
CPP_SOURCES = ["tables.cpp"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
HIP_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
CPP_FLAGS = ["-O2", "-std=c++17", "-fPIC", "-Wall", "-ffp-contract=off"]


def _run(cmd):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("command failed: %s\n%s" % (" ".join(cmd), r.stdout))
    return r.stdout


def build(verbose=False, jobs=None, extra_flags=(), lib=None, obj_dir=None):
    """extra_flags / lib / obj_dir: for building experimental variants beside the default one."""
    global OBJ, LIB
    OBJ_SAVE, LIB_SAVE = OBJ, LIB
    if obj_dir:
        OBJ = obj_dir
    if lib:
        LIB = lib
    try:
        return _build(verbose, jobs, list(extra_flags))
    finally:
        OBJ, LIB = OBJ_SAVE, LIB_SAVE


def _build(verbose, jobs, extra_flags):
    os.makedirs(OBJ, exist_ok=True)
    jobs = jobs or min(8, len(HIP_SOURCES) + len(CPP_SOURCES))
    tasks = []
    for s in HIP_SOURCES:
        o = os.path.join(OBJ, s + ".o")
        tasks.append(([HIPCC] + HIP_FLAGS + extra_flags + ["-c", os.path.join(CSRC, s), "-o", o], o))
    for s in CPP_SOURCES:
        o = os.path.join(OBJ, s + ".o")
        tasks.append((["g++"] + CPP_FLAGS + ["-c", os.path.join(CSRC, s), "-o", o], o))
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        outs = list(ex.map(lambda t: _run(t[0]), tasks))
    if verbose:
        for o in outs:
            if o.strip():
                print(o)
    _run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + [t[1] for t in tasks])
    return LIB


C_CLIENT_SRC = os.path.join(os.path.dirname(HERE), "tests", "c_client", "abi_client.c")
C_CLIENT = os.path.join(os.path.dirname(HERE), "tests", "c_client", "abi_client")


def build_c_client():
    """The plain C (C99, gcc) client of the ABI that the GPU tests run: shows that the header and
    the library are usable without Python or torch."""
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    _run(["gcc", "-std=c99", "-Wall", "-Werror", "-O1", "-D__HIP_PLATFORM_AMD__=1",
          "-I" + os.path.join(rocm, "include"), C_CLIENT_SRC, "-o", C_CLIENT,
          "-L" + HERE, "-lw2v_shard", "-L" + os.path.join(rocm, "lib"), "-lamdhip64",
          "-Wl,-rpath,$ORIGIN/../../paper_1606_08495_amd", "-Wl,-rpath," + os.path.join(rocm, "lib")])
    return C_CLIENT


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
    print(build_c_client())
