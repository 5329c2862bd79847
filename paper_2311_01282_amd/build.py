"""Build libfdattn.so for gfx950 with hipcc (cross-compiles without a GPU).

    python -m paper_2311_01282_amd.build

Objects go to ``paper_2311_01282_amd/_build/``; the library is written next to
this file so it travels with the source tree.
"""
import concurrent.futures
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
BUILD = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libfdattn.so")
SOURCES = ["fd_api.hip", "fd_row_kernels.hip", "fd_reduce_kernels.hip", "fd_gqa_kernels.hip",
           "fd_stats_kernels.hip", "fd_prefill_kernels.hip"]
# the benchmark's streaming-read probe: a library of its own, not part of libfdattn
PROBE_LIB = os.path.join(HERE, "libfdprobe.so")
PROBE_SOURCES = ["fd_probe.hip"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
    # packed-fp32 VALU forms are kept out of the generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def hipcc():
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def _compile(src, extra):
    obj = os.path.join(BUILD, os.path.splitext(src)[0] + ".o")
    cmd = [hipcc()] + FLAGS + list(extra) + ["-c", os.path.join(CSRC, src), "-o", obj]
    subprocess.check_call(cmd)
    return obj


def _link(lib, objs):
    tmp = lib + ".tmp%d" % os.getpid()
    subprocess.check_call([hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs)
    os.replace(tmp, lib)


# the phase-probe variant of the library (per-phase device timestamps in the per-row fused kernel;
# see paper_2311_01282_amd/phase_probe.py): same sources, -DFD_PHASE_PROBE, objects of its own
PHASE_LIB = os.path.join(HERE, "libfdattn_phase.so")


def build_phase_probe(verbose=False):
    os.makedirs(BUILD, exist_ok=True)

    def one(src):
        obj = os.path.join(BUILD, os.path.splitext(src)[0] + ".phase.o")
        subprocess.check_call([hipcc()] + FLAGS + ["-DFD_PHASE_PROBE", "-c", os.path.join(CSRC, src), "-o", obj])
        return obj
    with concurrent.futures.ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(one, SOURCES))
    _link(PHASE_LIB, objs)
    if verbose:
        print("built", PHASE_LIB)
    return PHASE_LIB


def build(extra_flags=(), verbose=False):
    os.makedirs(BUILD, exist_ok=True)
    with concurrent.futures.ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(lambda s: _compile(s, extra_flags), SOURCES + PROBE_SOURCES))
    _link(LIB, objs[:len(SOURCES)])
    _link(PROBE_LIB, objs[len(SOURCES):])
    if verbose:
        print("built", LIB, PROBE_LIB)
    return LIB


if __name__ == "__main__":
    if sys.argv[1:] == ["--phase-probe"]:
        build_phase_probe(verbose=True)
    else:
        build(extra_flags=sys.argv[1:], verbose=True)
