"""Build step: compile the HIP sources into ``libmla_decode.so`` (in-tree, beside this file)."""
from __future__ import annotations

import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(_HERE)
SOURCES = [os.path.join(_HERE, "csrc", "mla_decode.hip")]
LIB_PATH = os.path.join(_HERE, "libmla_decode.so")
# measurement only (the streaming-read ceiling the benchmark reports): its own library, no part of the product
# measurement only: the product source with time stamps at its phase boundaries (bench.py --timeline)
TIMELINE_LIB_PATH = os.path.join(_HERE, "libmla_decode_timeline.so")
PROBE_SOURCES = [os.path.join(_HERE, "csrc", "hbm_probe.hip")]
PROBE_LIB_PATH = os.path.join(_HERE, "libhbm_probe.so")
# measurement only: one LDS access pattern per launch, for the bank-conflict counters (bench.py --lds-probe)
LDS_PROBE_SOURCES = [os.path.join(_HERE, "csrc", "lds_probe.hip")]
LDS_PROBE_LIB_PATH = os.path.join(_HERE, "liblds_probe.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed-fp32 code generation is switched off for every HIP translation unit
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I" + os.path.join(ROOT, "include"),
]


def _compile(sources, lib_path, verbose, extra=()):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = lib_path + ".tmp.%d" % os.getpid()
    cmd = [hipcc] + HIPCC_FLAGS + list(extra) + sources + ["-o", tmp]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(line for line in res.stdout.splitlines() if "packed-fp32-ops" not in line)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    os.replace(tmp, lib_path)
    return lib_path


def build_library(verbose: bool = False) -> str:
    """Run hipcc (cross-compiles for gfx950 without a GPU).  Returns the library path."""
    return _compile(SOURCES, LIB_PATH, verbose)


def build_timeline(verbose: bool = False) -> str:
    """The product source compiled with -DMLA_TIMELINE (measurement only).  Returns the library path."""
    return _compile(SOURCES, TIMELINE_LIB_PATH, verbose, extra=["-DMLA_TIMELINE"])


def build_lds_probe(verbose: bool = False) -> str:
    """The LDS access-pattern probe of the benchmark (measurement only).  Returns the library path."""
    return _compile(LDS_PROBE_SOURCES, LDS_PROBE_LIB_PATH, verbose)


def build_probe(verbose: bool = False) -> str:
    """The streaming-read probe of the benchmark (measurement only).  Returns the library path."""
    return _compile(PROBE_SOURCES, PROBE_LIB_PATH, verbose)


if __name__ == "__main__":
    print(build_library(verbose=True))
    print(build_probe(verbose=True))
    print(build_timeline(verbose=True))
    print(build_lds_probe(verbose=True))
