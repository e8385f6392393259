"""Build step of the HIP library: one hipcc invocation for gfx950, output in-tree next to the binding."""
from __future__ import annotations

import os
import subprocess
from pathlib import Path

PKG = Path(__file__).resolve().parent
ROOT = PKG.parent
SOURCES = [PKG / "csrc" / "tsenor.hip"]
OUTPUT = PKG / "libtsenor.so"
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed fp32 instructions are kept out of every kernel
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # no implicit fused multiply-add: every rounding is the one written in the source (the kernels ask for
    # fma() where they want it), so a host evaluation of the importance gives the same bits
    "-ffp-contract=off",
    f"-I{ROOT / 'include'}",
]


# measurement aid, a program of its own: issue rate of single vector instructions (see its header)
PROBE_SOURCE = PKG / "csrc" / "issue_rate_probe.hip"
PROBE_OUTPUT = PKG / "issue_rate_probe.bin"
PROBE_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def build(verbose: bool = False) -> Path:
    """Compile every HIP source: libtsenor.so and the issue-rate probe (always recompiles)."""
    for flags, sources, output in ((FLAGS, SOURCES, OUTPUT), (PROBE_FLAGS, [PROBE_SOURCE], PROBE_OUTPUT)):
        tmp = output.with_suffix(output.suffix + f".tmp{os.getpid()}")
        cmd = [HIPCC, *flags, "-o", str(tmp), *map(str, sources)]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)
        os.replace(tmp, output)
    return OUTPUT


if __name__ == "__main__":
    print(build(verbose=True))
