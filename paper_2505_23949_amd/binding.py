"""ctypes binding of libtsenor.so (declared in include/tsenor.h).

Argument marshalling only: every step of the path runs in the HIP kernels of the
library.  PyTorch supplies device memory (``tensor.data_ptr()``) and the current
HIP stream; nothing here computes on tensors.  Loading fails loudly if the
library has not been built (``python -c "import __graft_entry__ as g; g.build()"``).
"""
from __future__ import annotations

import ctypes
from pathlib import Path

_PKG = Path(__file__).resolve().parent
LIB_PATH = _PKG / "libtsenor.so"

TSENOR_OK = 0
TSENOR_ERR_NULL = -1
TSENOR_ERR_SHAPE = -2
TSENOR_ERR_NM = -3
TSENOR_ERR_UNSUPPORTED = -4
TSENOR_ERR_PARAM = -5
TSENOR_ERR_WORKSPACE = -6
TSENOR_ERR_HIP = -7
TSENOR_ERR_TOO_LARGE = -8

TSENOR_F32 = 0
TSENOR_BF16 = 1
TSENOR_TAU_ABSOLUTE = 0
TSENOR_TAU_REL_MATRIX_MAX = 1
TSENOR_FLAG_STRICT_PAPER = 1 << 0
TSENOR_FLAG_COLS_FIRST = 1 << 1
TSENOR_FLAG_FP32_ITERATIONS = 1 << 2
TSENOR_FLAG_GREEDY_ONE_LANE = 1 << 3
TSENOR_FLAG_GREEDY_M_LANES = 1 << 4
TSENOR_FLAG_TILES_LARGE = 1 << 5
TSENOR_FLAG_TILES_SMALL = 1 << 6
TSENOR_FLAG_SIMPLE_ROUNDING = 1 << 7
TSENOR_ADAPTIVE_CHECK_EVERY = 4
TSENOR_IMPORTANCE_ABS = 0
TSENOR_IMPORTANCE_SQUARE = 1

EXPORTS = (
    "tsenor_workspace_bytes", "tsenor_mask_ex", "tsenor_mask_batched", "tsenor_mask", "tsenor_mask_ex_static",
    "tsenor_mask_ex_profile", "tsenor_last_hip_error",
    "tsenor_status_string", "tsenor_version",
)


class tsenor_problem(ctypes.Structure):
    _fields_ = [
        ("W", ctypes.c_void_p),
        ("dtype", ctypes.c_int32),
        ("rows", ctypes.c_int64),
        ("cols", ctypes.c_int64),
        ("ld", ctypes.c_int64),
        ("col_scale", ctypes.c_void_p),
        ("N", ctypes.c_int32),
        ("M", ctypes.c_int32),
        ("tau", ctypes.c_double),
        ("tau_mode", ctypes.c_int32),
        ("iters", ctypes.c_int32),
        ("local_search_steps", ctypes.c_int32),
        ("flags", ctypes.c_uint32),
        ("mask", ctypes.c_void_p),
        ("plan_out", ctypes.c_void_p),
        ("tau_eff_out", ctypes.c_void_p),
        ("stats_out", ctypes.c_void_p),
        ("add", ctypes.c_void_p),
        ("add_scale", ctypes.c_float),
        ("importance", ctypes.c_int32),
        ("packed_out", ctypes.c_void_p),
        ("pruned_out", ctypes.c_void_p),
        ("objective_out", ctypes.c_void_p),
        ("prev_mask", ctypes.c_void_p),
        ("tol", ctypes.c_double),
        ("iters_done_out", ctypes.c_void_p),
    ]


class TsenorError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        detail = f", hipError_t {load().tsenor_last_hip_error()}" if status == TSENOR_ERR_HIP else ""
        super().__init__(f"{where}: {status_string(status)} (status {status}{detail})")


_lib = None


def load() -> ctypes.CDLL:
    """Load the HIP library; raises if it is missing (there is no fallback path)."""
    global _lib
    if _lib is None:
        if not LIB_PATH.exists():
            raise ImportError(f"{LIB_PATH} is not built; run __graft_entry__.build() first")
        # PyTorch brings its own copy of the HIP runtime; it has to be in the process before this library is
        # loaded, so that both use the same one (device pointers and streams of one runtime mean nothing to another)
        import torch  # noqa: F401

        lib = ctypes.CDLL(str(LIB_PATH))
        P = ctypes.POINTER(tsenor_problem)
        lib.tsenor_workspace_bytes.argtypes = [P, ctypes.c_int]
        lib.tsenor_workspace_bytes.restype = ctypes.c_size_t
        lib.tsenor_mask_ex.argtypes = [P, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
        lib.tsenor_mask_ex.restype = ctypes.c_int
        lib.tsenor_mask_batched.argtypes = [P, ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
        lib.tsenor_mask_batched.restype = ctypes.c_int
        lib.tsenor_mask.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int, ctypes.c_int,
                                    ctypes.c_float, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
        lib.tsenor_mask.restype = ctypes.c_int
        lib.tsenor_mask_ex_static.argtypes = [P, ctypes.c_void_p]
        lib.tsenor_mask_ex_static.restype = ctypes.c_int
        lib.tsenor_mask_ex_profile.argtypes = [P, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_int,
                                               ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_double)]
        lib.tsenor_mask_ex_profile.restype = ctypes.c_int
        lib.tsenor_status_string.argtypes = [ctypes.c_int]
        lib.tsenor_status_string.restype = ctypes.c_char_p
        lib.tsenor_version.restype = ctypes.c_int
        lib.tsenor_last_hip_error.restype = ctypes.c_int
        _lib = lib
    return _lib


def status_string(status: int) -> str:
    return load().tsenor_status_string(int(status)).decode()


def version() -> int:
    return int(load().tsenor_version())


def _stream_handle(stream=None):
    import torch

    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _dtype_code(W) -> int:
    import torch

    if W.dtype == torch.float32:
        return TSENOR_F32
    if W.dtype == torch.bfloat16:
        return TSENOR_BF16
    raise TypeError(f"W must be float32 or bfloat16, got {W.dtype}")


def make_problem(W, N, M, tau, iters, *, mask, col_scale=None, tau_mode=TSENOR_TAU_ABSOLUTE,
                 local_search_steps=10, flags=0, plan_out=None, tau_eff_out=None, stats_out=None, add=None,
                 add_scale=0.0, importance=TSENOR_IMPORTANCE_ABS, packed_out=None, pruned_out=None,
                 objective_out=None, prev_mask=None, tol=0.0, iters_done_out=None) -> tsenor_problem:
    """Fill a tsenor_problem from device tensors (no copies; the tensors must outlive the call)."""
    if W.dim() != 2 or W.stride(1) != 1:
        raise ValueError("W must be a 2-D tensor with unit column stride")
    p = tsenor_problem()
    p.W = W.data_ptr()
    p.dtype = _dtype_code(W)
    p.rows, p.cols, p.ld = W.shape[0], W.shape[1], W.stride(0)
    p.col_scale = None if col_scale is None else col_scale.data_ptr()
    p.N, p.M = int(N), int(M)
    p.tau = float(tau)
    p.tau_mode = int(tau_mode)
    p.iters = int(iters)
    p.local_search_steps = int(local_search_steps)
    p.flags = int(flags)
    p.mask = mask.data_ptr()
    p.plan_out = None if plan_out is None else plan_out.data_ptr()
    p.tau_eff_out = None if tau_eff_out is None else tau_eff_out.data_ptr()
    p.stats_out = None if stats_out is None else stats_out.data_ptr()
    if add is not None:
        if add.dtype != W.dtype or add.shape != W.shape or add.stride() != W.stride():
            raise ValueError("add must have W's dtype, shape and strides")
        p.add = add.data_ptr()
        p.add_scale = float(add_scale)
    p.importance = int(importance)
    p.packed_out = None if packed_out is None else packed_out.data_ptr()
    p.pruned_out = None if pruned_out is None else pruned_out.data_ptr()
    p.objective_out = None if objective_out is None else objective_out.data_ptr()
    p.prev_mask = None if prev_mask is None else prev_mask.data_ptr()
    p.tol = float(tol)
    p.iters_done_out = None if iters_done_out is None else iters_done_out.data_ptr()
    return p


def tsenor_workspace_bytes(problems) -> int:
    arr = (tsenor_problem * len(problems))(*problems)
    return int(load().tsenor_workspace_bytes(arr, len(problems)))


def tsenor_mask_batched(problems, workspace, stream=None) -> None:
    """Enqueue the path for every problem on ``stream``; ``workspace`` is a uint8 device tensor."""
    arr = (tsenor_problem * len(problems))(*problems)
    rc = load().tsenor_mask_batched(arr, len(problems), ctypes.c_void_p(workspace.data_ptr()),
                                    workspace.numel() * workspace.element_size(), _stream_handle(stream))
    if rc != TSENOR_OK:
        raise TsenorError(rc, "tsenor_mask_batched")


def tsenor_mask_ex(problem, workspace, stream=None) -> None:
    rc = load().tsenor_mask_ex(ctypes.byref(problem), ctypes.c_void_p(workspace.data_ptr()),
                               workspace.numel() * workspace.element_size(), _stream_handle(stream))
    if rc != TSENOR_OK:
        raise TsenorError(rc, "tsenor_mask_ex")


STATIC_SCRATCH_BYTES = 48 << 20


def tsenor_mask_ex_static(problem, stream=None) -> None:
    """tsenor_mask_ex on the library's own fixed scratch (no allocation anywhere in the call)."""
    rc = load().tsenor_mask_ex_static(ctypes.byref(problem), _stream_handle(stream))
    if rc != TSENOR_OK:
        raise TsenorError(rc, "tsenor_mask_ex_static")


NUM_STAGES = 4
STAGE_NAMES = ("reset+absmax", "dykstra+sort", "greedy", "local_search+write")


def tsenor_mask_ex_profile(problem, workspace, repeats, stream=None, want_clock=False):
    """Run the path ``repeats`` times, synchronise, return the mean per-stage durations in ms (and, if asked for,
    the shader clock in MHz that the Dykstra kernel's first wave saw over its iteration loop)."""
    ms = (ctypes.c_float * NUM_STAGES)()
    mhz = ctypes.c_double(0.0)
    rc = load().tsenor_mask_ex_profile(ctypes.byref(problem), ctypes.c_void_p(workspace.data_ptr()),
                                       workspace.numel() * workspace.element_size(), _stream_handle(stream),
                                       int(repeats), ms, ctypes.byref(mhz) if want_clock else None)
    if rc != TSENOR_OK:
        raise TsenorError(rc, "tsenor_mask_ex_profile")
    return ([float(x) for x in ms], float(mhz.value)) if want_clock else [float(x) for x in ms]


def tsenor_mask(W, N, M, tau, iters, mask=None, stream=None):
    """The paper's problem statement on an fp32 matrix: importance |W|, K = tau |W|. Returns the mask tensor."""
    import torch

    if W.dtype != torch.float32 or not W.is_contiguous():
        raise TypeError("tsenor_mask takes a contiguous float32 matrix")
    if mask is None:
        mask = torch.empty(W.shape, dtype=torch.uint8, device=W.device)
    rc = load().tsenor_mask(ctypes.c_void_p(W.data_ptr()), W.shape[0], W.shape[1], int(N), int(M), float(tau),
                            int(iters), ctypes.c_void_p(mask.data_ptr()), _stream_handle(stream))
    if rc != TSENOR_OK:
        raise TsenorError(rc, "tsenor_mask")
    return mask


def solve(W, N, M, tau, iters, *, col_scale=None, tau_mode=TSENOR_TAU_ABSOLUTE, local_search_steps=10, flags=0,
          want_plan=False, want_stats=False, workspace=None, stream=None, add=None, add_scale=0.0,
          importance=TSENOR_IMPORTANCE_ABS, want_packed=False, want_pruned=False, want_objective=False,
          prev_mask=None, tol=0.0, want_iters_done=False):
    """Allocate outputs and scratch with torch, call tsenor_mask_ex once, return dict(mask[, plan, stats, tau_eff])."""
    import torch

    dev = W.device
    mask = torch.empty(W.shape, dtype=torch.uint8, device=dev)
    plan = torch.empty(W.shape, dtype=torch.float64, device=dev) if want_plan else None
    stats = torch.zeros(4, dtype=torch.int64, device=dev) if want_stats else None
    tau_eff = torch.zeros(1, dtype=torch.float64, device=dev)
    packed = torch.empty((W.shape[0], W.shape[1] // 8), dtype=torch.uint8, device=dev) if want_packed else None
    pruned = torch.empty(W.shape, dtype=W.dtype, device=dev) if want_pruned else None
    objective = torch.zeros(2, dtype=torch.float64, device=dev) if want_objective else None
    iters_done = (torch.zeros((W.shape[0] // M) * (W.shape[1] // M), dtype=torch.int32, device=dev)
                  if want_iters_done else None)
    p = make_problem(W, N, M, tau, iters, mask=mask, col_scale=col_scale, tau_mode=tau_mode,
                     local_search_steps=local_search_steps, flags=flags, plan_out=plan, tau_eff_out=tau_eff,
                     stats_out=stats, add=add, add_scale=add_scale, importance=importance, packed_out=packed,
                     pruned_out=pruned, objective_out=objective, prev_mask=prev_mask, tol=tol,
                     iters_done_out=iters_done)
    need = tsenor_workspace_bytes([p])
    if need == 0:
        # invalid arguments: let the entry point name the reason
        tsenor_mask_ex(p, torch.empty(256, dtype=torch.uint8, device=dev), stream)
    if workspace is None or workspace.numel() < need:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    tsenor_mask_ex(p, workspace, stream)
    out = {"mask": mask, "tau_eff": tau_eff, "workspace": workspace}
    if want_plan:
        out["plan"] = plan
    if want_stats:
        out["stats"] = stats
    if want_packed:
        out["packed"] = packed
    if want_pruned:
        out["pruned"] = pruned
    if want_objective:
        out["objective"] = objective
    if want_iters_done:
        out["iters_done"] = iters_done
    return out
