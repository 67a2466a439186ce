"""Build step: compiles csrc/*.hip into libtokenlake.so (gfx950) next to this file.

Usage:  python -m paper_2508_17219_amd.build
"""
from __future__ import annotations

import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "libtokenlake.so")
PROBE_LIB = os.path.join(HERE, "probe", "libtlprobe.so")      # bench.py's MFMA-only probe, a library of its own

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "-fPIC", "-shared", "--offload-arch=gfx950",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-unknown-warning-option",
]


def sources():
    return sorted(glob.glob(os.path.join(HERE, "csrc", "*.hip")))


def _hipcc(srcs, target, verbose, extra_flags=()):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + HIPCC_FLAGS + list(extra_flags) + [
        "-I", os.path.join(ROOT, "include"), "-I", os.path.join(HERE, "csrc"),
    ] + srcs + ["-o", target + ".tmp"]
    if verbose:
        print("[build]", " ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if verbose and out.strip():
        print(out, flush=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed (%d)\n%s" % (res.returncode, out))
    os.replace(target + ".tmp", target)
    return target


def build(verbose: bool = True, extra_flags=()) -> str:
    """Compile the library and the benchmark's probe (always recompiles); returns the library's path."""
    _hipcc(sources(), LIB, verbose, extra_flags)
    build_probe(verbose)
    return LIB


def build_probe(verbose: bool = True) -> str:
    return _hipcc([os.path.join(HERE, "probe", "mfma_probe.hip"), os.path.join(HERE, "probe", "issue_probe.hip")], PROBE_LIB, verbose)


def ensure_built(verbose: bool = True) -> str:
    """Build only if no library is there (tests, the smoke run and the benchmark call this; after a
    change to a source, run the build itself)."""
    return LIB if os.path.exists(LIB) else build(verbose)


if __name__ == "__main__":
    build()
    sys.exit(0)
