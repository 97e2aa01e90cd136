"""Builds libterngrad.so in-tree with hipcc for gfx950 (and, for bench.py, the bandwidth probes of
bench_probe.hip as a library of their own: a measurement instrument, no part of the product).

    python -m paper_1705_07878_amd.build
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libterngrad.so")
ROOT = os.path.dirname(HERE)
PROBE_SRC = os.path.join(ROOT, "bench_probe.hip")
PROBE_LIB = os.path.join(ROOT, "libbench_probe.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off",                       # fp32 products and sums are rounded separately
    "-fno-fast-math",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


def sources():
    return [os.path.join(CSRC, "terngrad.hip")]


def headers():
    hs = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".hpp")]
    hs.append(os.path.join(os.path.dirname(HERE), "include", "terngrad.h"))
    return hs


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(f) > t for f in sources() + headers())


def _hipcc(srcs, lib, verbose, extra=()):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + HIPCC_FLAGS + list(extra) + list(srcs) + ["-o", lib]
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)


def build(force: bool = True, verbose: bool = True) -> str:
    """Compiles the library (always, unless force=False and it is up to date)."""
    if not force and not is_stale():
        return LIB
    _hipcc(sources(), LIB, verbose)
    return LIB


def build_probe(force: bool = True, verbose: bool = True) -> str:
    """Compiles the bench-only probe library next to bench.py."""
    if not force and os.path.exists(PROBE_LIB) and all(
            os.path.getmtime(f) <= os.path.getmtime(PROBE_LIB) for f in [PROBE_SRC] + headers()):
        return PROBE_LIB
    _hipcc([PROBE_SRC], PROBE_LIB, verbose, extra=["-I", ROOT])
    return PROBE_LIB


if __name__ == "__main__":
    build()
    build_probe()
    print("built", LIB, PROBE_LIB)
    sys.exit(0)
