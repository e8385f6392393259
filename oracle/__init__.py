"""CPU oracle for transposable N:M mask finding.  TEST INFRASTRUCTURE ONLY.

Thin ctypes wrapper around ``tsenor_oracle.c`` (plain C, double precision, the
paper's Algorithm 1 and Algorithm 2 step by step) plus the exact checkers in
``oracle.exact``.  Only tests, the smoke check and the benchmark's cpu_baseline
leg may import this package; it shares nothing with the HIP path and never
imports it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from pathlib import Path

import numpy as np

_DIR = Path(__file__).resolve().parent
_SRC = _DIR / "tsenor_oracle.c"
_LIB = _DIR / "libtsenor_oracle.so"

TAU_ABSOLUTE = 0
TAU_REL_MATRIX_MAX = 1


def build(force: bool = False) -> Path:
    """Compile the C oracle with gcc (-O2, no fast-math, OpenMP over blocks)."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        tmp = _LIB.with_suffix(f".so.tmp{os.getpid()}")
        subprocess.run(
            ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
             "-o", str(tmp), str(_SRC), "-lm"],
            check=True,
        )
        os.replace(tmp, _LIB)
    return _LIB


def build_sanitized() -> Path:
    """The same source with AddressSanitizer and UndefinedBehaviorSanitizer (gcc, -O1, frame pointers kept).
    Loaded instead of the ordinary build by a process that names it in TSENOR_ORACLE_LIBRARY (and preloads the
    sanitizer runtimes): how the tests run the pins over instrumented code."""
    out = _DIR / "libtsenor_oracle_sanitized.so"
    tmp = out.with_suffix(f".so.tmp{os.getpid()}")
    subprocess.run(
        ["gcc", "-O1", "-g", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
         "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
         "-o", str(tmp), str(_SRC), "-lm"],
        check=True,
    )
    os.replace(tmp, out)
    return out


_lib = None


def loaded_library() -> str:
    """Path of the shared library the oracle calls go to."""
    _load()
    return _lib._name


def _load():
    global _lib
    if _lib is None:
        override = os.environ.get("TSENOR_ORACLE_LIBRARY")
        if override:
            lib = ctypes.CDLL(override)
        else:
            build()
            lib = ctypes.CDLL(str(_LIB))
        i64, dbl, i32 = ctypes.c_int64, ctypes.c_double, ctypes.c_int
        p = ctypes.c_void_p
        lib.tsenor_oracle_importance.argtypes = [p, i64, i64, i64, p, p]
        lib.tsenor_oracle_importance.restype = i32
        lib.tsenor_oracle_tau_eff.argtypes = [p, i64, i64, dbl, i32]
        lib.tsenor_oracle_tau_eff.restype = dbl
        lib.tsenor_oracle_dykstra.argtypes = [p, i64, i64, i32, i32, dbl, i32, i32, p, p]
        lib.tsenor_oracle_dykstra.restype = i32
        lib.tsenor_oracle_dykstra_adaptive.argtypes = [p, i64, i64, i32, i32, dbl, i32, i32, dbl, i32, p, p]
        lib.tsenor_oracle_dykstra_adaptive.restype = i32
        lib.tsenor_oracle_round.argtypes = [p, p, i64, i64, i32, i32, i32, i32, p, p]
        lib.tsenor_oracle_round.restype = i32
        lib.tsenor_oracle_swap_scores.argtypes = [p, p, i32, i32, i32, p]
        lib.tsenor_oracle_swap_scores.restype = i32
        lib.tsenor_oracle_mask.argtypes = [p, i64, i64, i64, p, i32, i32, dbl, i32, i32, i32, i32, i32, p, p, p, p]
        lib.tsenor_oracle_mask.restype = i32
        lib.tsenor_oracle_importance_ex.argtypes = [p, p, ctypes.c_float, i64, i64, i64, p, i32, p, p]
        lib.tsenor_oracle_importance_ex.restype = i32
        lib.tsenor_oracle_objective.argtypes = [p, p, i64, i64, i32]
        lib.tsenor_oracle_objective.restype = dbl
        lib.tsenor_oracle_num_threads.restype = i32
        lib.tsenor_oracle_set_threads.argtypes = [i32]
        _lib = lib
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def num_threads() -> int:
    return int(_load().tsenor_oracle_num_threads())


def set_threads(n: int) -> None:
    _load().tsenor_oracle_set_threads(int(n))


def importance(W, col_scale=None) -> np.ndarray:
    """imp = |W| (times col_scale[j]) as one float32 multiply per weight."""
    W = _f32(W)
    cs = None if col_scale is None else _f32(col_scale)
    out = np.empty_like(W)
    rc = _load().tsenor_oracle_importance(_ptr(W), W.shape[0], W.shape[1], W.shape[1], _ptr(cs), _ptr(out))
    if rc:
        raise ValueError(f"tsenor_oracle_importance failed: {rc}")
    return out


def importance_ex(W, *, add=None, add_scale: float = 0.0, col_scale=None, square: bool = False):
    """Importance with the transforms of Sec. 4 / Proposition 1: x = W + add_scale*add, |x| * col_scale, optionally
    squared, every step one float32 operation.  Returns (importance, x)."""
    W = _f32(W)
    a = None if add is None else _f32(add)
    cs = None if col_scale is None else _f32(col_scale)
    imp, val = np.empty_like(W), np.empty_like(W)
    rc = _load().tsenor_oracle_importance_ex(_ptr(W), _ptr(a), float(add_scale), W.shape[0], W.shape[1], W.shape[1],
                                             _ptr(cs), int(square), _ptr(imp), _ptr(val))
    if rc:
        raise ValueError(f"tsenor_oracle_importance_ex failed: {rc}")
    return imp, val


def objective(mask_, imp, M: int) -> float:
    """Objective of Eq. (1): the importance the mask keeps, summed in double."""
    mask_ = np.ascontiguousarray(mask_, dtype=np.uint8)
    imp = _f32(imp)
    return float(_load().tsenor_oracle_objective(_ptr(mask_), _ptr(imp), imp.shape[0], imp.shape[1], int(M)))


def pack_bits(mask_) -> np.ndarray:
    """Bit-packed mask: bit (j & 7) of byte j >> 3 of row i is S_ij."""
    return np.packbits(np.ascontiguousarray(mask_, dtype=np.uint8), axis=1, bitorder="little")


def solve_ex(W, N: int, M: int, tau: float, T: int, *, add=None, add_scale: float = 0.0, col_scale=None,
             square: bool = False, tau_mode: int = TAU_ABSOLUTE, L: int = 10, strict_paper: bool = False,
             cols_first: bool = False, prev_mask=None):
    """The whole path with the importance transforms, the objective and the safeguard of App. A.1
    (Assumption 1: if the previous mask keeps strictly more importance than the one found, it is returned).
    Returns dict(mask, pruned, packed, objective, objective_prev, used_prev, stats, tau_eff, log_S)."""
    imp, val = importance_ex(W, add=add, add_scale=add_scale, col_scale=col_scale, square=square)
    te = tau_eff(imp, tau, tau_mode)
    log_S = dykstra(imp, N, M, te, T, cols_first=cols_first)
    m, stats = round_plan(log_S, imp, N, M, L=L, strict_paper=strict_paper)
    obj = objective(m, imp, M)
    obj_prev, used_prev = 0.0, False
    if prev_mask is not None:
        prev_mask = np.ascontiguousarray(prev_mask, dtype=np.uint8)
        obj_prev = objective(prev_mask, imp, M)
        if obj_prev > obj:
            m, used_prev = prev_mask.copy(), True
    return {"mask": m, "pruned": val * m, "packed": pack_bits(m), "objective": obj_prev if used_prev else obj,
            "objective_new": obj, "objective_prev": obj_prev, "used_prev": used_prev, "stats": stats, "tau_eff": te,
            "log_S": log_S}


def tau_eff(imp, tau: float, tau_mode: int = TAU_ABSOLUTE) -> float:
    imp = _f32(imp)
    return float(_load().tsenor_oracle_tau_eff(_ptr(imp), imp.shape[0], imp.shape[1], float(tau), int(tau_mode)))


def dykstra(imp, N: int, M: int, tau_eff_value: float, T: int, cols_first: bool = False, return_log_Q: bool = False):
    """Algorithm 1 on every MxM block of ``imp``; returns log S^(T) (and log Q^(T))."""
    imp = _f32(imp)
    rows, cols = imp.shape
    log_S = np.empty((rows, cols), dtype=np.float64)
    log_Q = np.empty((rows, cols), dtype=np.float64) if return_log_Q else None
    rc = _load().tsenor_oracle_dykstra(_ptr(imp), rows, cols, N, M, float(tau_eff_value), T, int(cols_first),
                                       _ptr(log_S), _ptr(log_Q))
    if rc:
        raise ValueError(f"tsenor_oracle_dykstra failed: {rc}")
    return (log_S, log_Q) if return_log_Q else log_S


ADAPTIVE_CHECK_EVERY = 4


def dykstra_adaptive(imp, N: int, M: int, tau_eff_value: float, T: int, tol: float, cols_first: bool = False,
                     check_every: int = ADAPTIVE_CHECK_EVERY):
    """Algorithm 1 with T read as a bound: a block stops after a `check_every`-th iteration in which every row
    and column scaling factor was within `tol` of 1.  Returns (log S, iterations done per block)."""
    imp = _f32(imp)
    rows, cols = imp.shape
    log_S = np.empty((rows, cols), dtype=np.float64)
    done = np.zeros((rows // M) * (cols // M), dtype=np.int32)
    rc = _load().tsenor_oracle_dykstra_adaptive(_ptr(imp), rows, cols, N, M, float(tau_eff_value), T,
                                                int(cols_first), float(tol), int(check_every), _ptr(log_S),
                                                _ptr(done))
    if rc:
        raise ValueError(f"tsenor_oracle_dykstra_adaptive failed: {rc}")
    return log_S, done


def round_plan(key, imp, N: int, M: int, L: int = 10, strict_paper: bool = False):
    """Algorithm 2 on every block: greedy on ``key`` then local search scored on ``imp``.

    Returns (mask uint8, stats[4] = missing-after-greedy, non-positive swaps applied,
    blocks needing more than L rounds, units still missing at return)."""
    key = np.ascontiguousarray(key, dtype=np.float64)
    imp = _f32(imp)
    rows, cols = imp.shape
    mask = np.empty((rows, cols), dtype=np.uint8)
    stats = np.zeros(4, dtype=np.int64)
    rc = _load().tsenor_oracle_round(_ptr(key), _ptr(imp), rows, cols, N, M, L, int(strict_paper), _ptr(mask),
                                     _ptr(stats))
    if rc:
        raise ValueError(f"tsenor_oracle_round failed: {rc}")
    return mask, stats


def simple_round(key, N: int, M: int) -> np.ndarray:
    """The "Simple" rounding arm of App. B.2.1, written out as its definition: in every block keep the N
    largest entries of each row (row-wise N:M rounding of the plan), then, of what is left, the N largest of
    each column.  Ties go to the lower index.  Rows may end up with fewer than N entries."""
    key = np.ascontiguousarray(key, dtype=np.float64)
    rows, cols = key.shape
    out = np.zeros((rows, cols), dtype=np.uint8)
    for r0 in range(0, rows, M):
        for c0 in range(0, cols, M):
            blk = key[r0:r0 + M, c0:c0 + M]
            kept = np.zeros((M, M), dtype=bool)
            for i in range(M):
                order = sorted(range(M), key=lambda j: (-blk[i, j], j))
                kept[i, order[:N]] = True
            final = np.zeros((M, M), dtype=np.uint8)
            for j in range(M):
                cand = [i for i in range(M) if kept[i, j]]
                cand.sort(key=lambda i: (-blk[i, j], i))
                for i in cand[:N]:
                    final[i, j] = 1
            out[r0:r0 + M, c0:c0 + M] = final
    return out


def swap_scores(imp_block, S_block, i: int, j: int) -> np.ndarray:
    """Eq. (5) score matrix of one block for deficient row i and column j (0-based)."""
    imp_block = _f32(imp_block)
    S_block = np.ascontiguousarray(S_block, dtype=np.uint8)
    M = imp_block.shape[0]
    out = np.empty((M, M), dtype=np.float64)
    rc = _load().tsenor_oracle_swap_scores(_ptr(imp_block), _ptr(S_block), M, i, j, _ptr(out))
    if rc:
        raise ValueError(f"tsenor_oracle_swap_scores failed: {rc}")
    return out


def mask(W, N: int, M: int, tau: float, T: int, *, col_scale=None, tau_mode: int = TAU_ABSOLUTE, L: int = 10,
         strict_paper: bool = False, cols_first: bool = False, return_plan: bool = False):
    """The whole path on a float32 matrix W.  Returns dict(mask, stats, tau_eff[, log_S])."""
    W = _f32(W)
    rows, cols = W.shape
    cs = None if col_scale is None else _f32(col_scale)
    out = np.empty((rows, cols), dtype=np.uint8)
    plan = np.empty((rows, cols), dtype=np.float64) if return_plan else None
    te = ctypes.c_double(0.0)
    stats = np.zeros(4, dtype=np.int64)
    rc = _load().tsenor_oracle_mask(_ptr(W), rows, cols, cols, _ptr(cs), N, M, float(tau), int(tau_mode), T, L,
                                    int(strict_paper), int(cols_first), _ptr(out), _ptr(plan),
                                    ctypes.cast(ctypes.byref(te), ctypes.c_void_p), _ptr(stats))
    if rc:
        raise ValueError(f"tsenor_oracle_mask failed: {rc}")
    res = {"mask": out, "stats": stats, "tau_eff": te.value}
    if return_plan:
        res["log_S"] = plan
    return res
