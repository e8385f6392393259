"""Seeded synthetic inputs shared by the tests, the benchmark and the smoke check.

Holds input generation only: no arithmetic of the mask-finding method lives
here.  Every workload is a stand-in for the LLaMA weight matrices the paper
prunes (Sec. 5); shapes are the 8B / 70B projection shapes and the value
distributions are the ones the build's baseline names.  All draws come from
``numpy.random.Generator(Philox(seed))`` so that host and device see the same
bits.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np

TAU_ABSOLUTE = 0
TAU_REL_MATRIX_MAX = 1


@dataclass(frozen=True)
class Workload:
    name: str
    rows: int
    cols: int
    N: int
    M: int
    tau: float            # coefficient c of the REL_MATRIX_MAX mode, or the literal tau in ABSOLUTE mode
    iters: int            # T
    dtype: str            # "f32" or "bf16": storage type of W handed to the library
    dist: str             # "normal", "wanda", "student_t"
    seed: int
    tau_mode: int = TAU_REL_MATRIX_MAX

    def scaled(self, rows: int, cols: int, name: str | None = None) -> "Workload":
        """Same recipe on a smaller matrix (for cases the CPU oracle finishes in seconds)."""
        return replace(self, rows=rows, cols=cols, name=name or f"{self.name}[{rows}x{cols}]")


CONFIGS = {
    "cfg1_2of4_512": Workload("cfg1_2of4_512", 512, 512, 2, 4, 0.01, 200, "f32", "normal", 1001),
    "cfg2_8of16_4096": Workload("cfg2_8of16_4096", 4096, 4096, 8, 16, 0.01, 300, "f32", "normal", 1002),
    "cfg3_16of32_4096x14336": Workload("cfg3_16of32_4096x14336", 4096, 14336, 16, 32, 0.005, 300, "bf16", "wanda", 1003),
    "cfg5_32of64_8192x28672": Workload("cfg5_32of64_8192x28672", 8192, 28672, 32, 64, 0.002, 500, "f32", "student_t", 1005),
}

# one decoder layer of the 8B shape set: (name, rows, cols)
LAYER_SHAPES_8B = (
    ("q", 4096, 4096), ("k", 1024, 4096), ("v", 1024, 4096), ("o", 4096, 4096),
    ("gate", 14336, 4096), ("up", 14336, 4096), ("down", 4096, 14336),
)


def layer_workloads(layer: int = 0):
    """The seven matrices of one 8B decoder layer, fp32, Wanda-style importance, 16:32."""
    return [Workload(f"cfg4_layer{layer}_{n}", r, c, 16, 32, 0.005, 300, "f32", "wanda", 1004 + 97 * layer + k)
            for k, (n, r, c) in enumerate(LAYER_SHAPES_8B)]


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round to nearest, ties to even); returns the uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns to float32 (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def generate(w: Workload):
    """Returns dict(W_f32, W_store, col_scale): the float32 values the method sees, the array in the
    storage type handed to the library (float32, or uint16 bf16 bit patterns) and the optional
    per-column scale (float32, length cols) of the Wanda-style importance |W_ij| * c_j."""
    rng = np.random.Generator(np.random.Philox(w.seed))
    shape = (w.rows, w.cols)
    col_scale = None
    if w.dist == "normal":
        W = rng.standard_normal(shape, dtype=np.float32)
    elif w.dist == "wanda":
        W = (np.float32(0.02) * rng.standard_normal(shape, dtype=np.float32)).astype(np.float32)
        col_scale = rng.lognormal(0.0, 1.0, w.cols).astype(np.float32)
    elif w.dist == "student_t":
        W = (0.02 * rng.standard_t(3.0, shape)).astype(np.float32)
    else:
        raise ValueError(w.dist)
    if w.dtype == "bf16":
        store = f32_to_bf16_bits(W)
        W = bf16_bits_to_f32(store)
    elif w.dtype == "f32":
        store = W
    else:
        raise ValueError(w.dtype)
    return {"W_f32": W, "W_store": store, "col_scale": col_scale}
