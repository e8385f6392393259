"""Build step of the HIP library for gfx950, output in-tree next to the binding.

The host code and the kernels of every block size are translation units of their own, compiled side by side
(one hipcc process each) and linked into libtsenor.so.
"""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor
from pathlib import Path

PKG = Path(__file__).resolve().parent
ROOT = PKG.parent
CSRC = PKG / "csrc"
SOURCES = [CSRC / "tsenor.hip"] + [CSRC / f"launch_m{m}.hip" for m in (64, 32, 16, 8, 4)]
OUTPUT = PKG / "libtsenor.so"
OBJ_DIR = PKG / "_build"
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # packed fp32 instructions are kept out of every kernel
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # no implicit fused multiply-add: every rounding is the one written in the source (the kernels ask for
    # fma() where they want it), so a host evaluation of the importance gives the same bits
    "-ffp-contract=off",
    f"-I{ROOT / 'include'}",
]

# measurement aid, a program of its own: issue rate of single vector instructions (see its header)
PROBE_SOURCE = CSRC / "issue_rate_probe.hip"
PROBE_OUTPUT = PKG / "issue_rate_probe.bin"
PROBE_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(map(str, cmd)), flush=True)
    subprocess.run(list(map(str, cmd)), check=True)


def build(verbose: bool = False, jobs: int | None = None) -> Path:
    """Compile libtsenor.so (always recompiles every source)."""
    OBJ_DIR.mkdir(exist_ok=True)
    jobs = jobs or min(len(SOURCES), os.cpu_count() or 1, 16)
    objects = [OBJ_DIR / (s.stem + f".{os.getpid()}.o") for s in SOURCES]
    try:
        with ThreadPoolExecutor(max_workers=jobs) as pool:
            list(pool.map(lambda so: _run([HIPCC, *FLAGS, "-c", "-o", so[1], so[0]], verbose), zip(SOURCES, objects)))
        tmp = OUTPUT.with_suffix(OUTPUT.suffix + f".tmp{os.getpid()}")
        _run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objects], verbose)
        os.replace(tmp, OUTPUT)
    finally:
        for o in objects:
            o.unlink(missing_ok=True)
    return OUTPUT


def build_probe(verbose: bool = False) -> Path:
    """Compile the issue-rate probe (not part of the library; run by hand for profiles/issue_rates_mi355x.md)."""
    tmp = PROBE_OUTPUT.with_suffix(PROBE_OUTPUT.suffix + f".tmp{os.getpid()}")
    _run([HIPCC, *PROBE_FLAGS, "-o", tmp, PROBE_SOURCE], verbose)
    os.replace(tmp, PROBE_OUTPUT)
    return PROBE_OUTPUT


if __name__ == "__main__":
    import sys

    print(build(verbose=True))
    if "--probe" in sys.argv[1:]:
        print(build_probe(verbose=True))
