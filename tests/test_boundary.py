"""CPU-only checks of the C-ABI boundary: exports, argument validation, workspace sizes (no compute calls)."""
import ctypes
import os
import re
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2505_23949_amd import binding

    if not binding.LIB_PATH.exists():
        from paper_2505_23949_amd import build

        build.build()
    return binding.load()


def _problem(**kw):
    from paper_2505_23949_amd import binding as b

    p = b.tsenor_problem()
    p.W, p.mask = 0x1000, 0x2000          # never dereferenced: validation happens on the host
    p.dtype = b.TSENOR_F32
    p.rows, p.cols, p.ld = 64, 128, 128
    p.N, p.M = 8, 16
    p.tau, p.tau_mode = 0.01, b.TSENOR_TAU_REL_MATRIX_MAX
    p.iters, p.local_search_steps, p.flags = 10, 10, 0
    for k, v in kw.items():
        setattr(p, k, v)
    return p


def test_every_declared_entry_point_is_exported(lib):
    from paper_2505_23949_amd import binding

    import glob

    headers = sorted(glob.glob(os.path.join(ROOT, "include", "*.h")))
    assert len(headers) >= 2
    text = "".join(re.sub(r"/\*.*?\*/", "", open(h).read(), flags=re.S) for h in headers)
    declared = set(re.findall(r"\b(tsenor_[a-z_]+)\s*\(", text))
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None


def test_struct_layout_matches_header():
    import tempfile

    from paper_2505_23949_amd import binding

    # ask the C compiler for the layout of the struct the header declares and compare with the ctypes mirror
    fields = [f[0] for f in binding.tsenor_problem._fields_]
    prog = '#include <stdio.h>\n#include <stddef.h>\n#include "tsenor.h"\nint main(void){\n'
    prog += 'printf("%zu\\n", sizeof(tsenor_problem));\n'
    prog += "".join(f'printf("%zu\\n", offsetof(tsenor_problem, {f}));\n' for f in fields) + "return 0;}\n"
    with tempfile.TemporaryDirectory() as d:
        src, exe = os.path.join(d, "layout.c"), os.path.join(d, "layout")
        open(src, "w").write(prog)
        subprocess.run(["gcc", "-std=c99", "-I", os.path.join(ROOT, "include"), "-o", exe, src], check=True)
        out = [int(x) for x in subprocess.run([exe], capture_output=True, text=True, check=True).stdout.split()]
    assert out[0] == ctypes.sizeof(binding.tsenor_problem)
    assert out[1:] == [getattr(binding.tsenor_problem, f).offset for f in fields]


def test_validation_errors(lib):
    from paper_2505_23949_amd import binding as b

    def call(p, ws=0x10000, nbytes=1 << 40):
        return lib.tsenor_mask_ex(ctypes.byref(p), ctypes.c_void_p(ws), nbytes, None)

    assert call(_problem(W=None)) == b.TSENOR_ERR_NULL
    assert call(_problem(mask=None)) == b.TSENOR_ERR_NULL
    assert lib.tsenor_mask_ex(None, ctypes.c_void_p(0x10000), 1 << 40, None) == b.TSENOR_ERR_NULL
    for bad in (dict(rows=0), dict(cols=-16), dict(rows=72), dict(cols=100), dict(ld=64), dict(rows=1 << 32)):
        assert call(_problem(**bad)) == b.TSENOR_ERR_SHAPE, bad
    assert call(_problem(N=-1)) == b.TSENOR_ERR_NM
    assert call(_problem(N=17)) == b.TSENOR_ERR_NM
    for bad in (dict(M=5), dict(M=128), dict(dtype=7), dict(tau_mode=3), dict(flags=1 << 9)):
        assert call(_problem(**bad)) == b.TSENOR_ERR_UNSUPPORTED, bad
    for bad in (dict(tau=0.0), dict(tau=-1.0), dict(tau=float("nan")), dict(tau=float("inf")), dict(iters=-1),
                dict(local_search_steps=-2), dict(tau=1e-4)):
        assert call(_problem(**bad)) == b.TSENOR_ERR_PARAM, bad
    assert call(_problem(tau=1e-4, tau_mode=b.TSENOR_TAU_ABSOLUTE), ws=0) == b.TSENOR_ERR_WORKSPACE
    good = _problem()
    need = lib.tsenor_workspace_bytes(ctypes.byref(good), 1)
    assert need > 0
    assert call(good, ws=0) == b.TSENOR_ERR_WORKSPACE
    assert call(good, ws=0x10010) == b.TSENOR_ERR_WORKSPACE          # not 256-byte aligned
    assert call(good, nbytes=need - 1) == b.TSENOR_ERR_WORKSPACE
    stage = (ctypes.c_float * b.NUM_STAGES)()
    assert lib.tsenor_mask_ex_profile(ctypes.byref(good), ctypes.c_void_p(0x10000), 1 << 40, None, 0, stage, None) \
        == b.TSENOR_ERR_PARAM
    assert lib.tsenor_mask_ex_profile(ctypes.byref(good), ctypes.c_void_p(0x10000), 1 << 40, None, 1, None, None) \
        == b.TSENOR_ERR_NULL
    assert lib.tsenor_mask(None, 64, 64, 8, 16, 0.1, 10, ctypes.c_void_p(0x2000), None) == b.TSENOR_ERR_NULL
    assert lib.tsenor_mask(ctypes.c_void_p(0x1000), 64, 60, 8, 16, 0.1, 10, ctypes.c_void_p(0x2000), None) \
        == b.TSENOR_ERR_SHAPE


def test_limits_checked_before_any_launch(lib):
    from paper_2505_23949_amd import binding as b

    # fewer than 2^31 blocks of one size in a call: 2^39 weights of 4x4 blocks are 2^35 blocks
    huge = _problem(M=4, N=2, rows=1 << 20, cols=1 << 19, ld=1 << 19)
    assert lib.tsenor_workspace_bytes(ctypes.byref(huge), 1) > 0           # a valid problem on its own
    assert lib.tsenor_mask_ex(ctypes.byref(huge), ctypes.c_void_p(0x10000), 1 << 62, None) == b.TSENOR_ERR_SHAPE
    # the second problem of a batch is checked before the first one is enqueued
    arr = (b.tsenor_problem * 2)(_problem(), _problem(N=99))
    assert lib.tsenor_mask_batched(arr, 2, ctypes.c_void_p(0x10000), 1 << 40, None) == b.TSENOR_ERR_NM
    # the entry point on the library's fixed scratch refuses what does not fit, before it touches the device
    big = _problem(M=32, N=16, rows=8192, cols=8192, ld=8192)
    assert lib.tsenor_workspace_bytes(ctypes.byref(big), 1) > b.STATIC_SCRATCH_BYTES
    assert lib.tsenor_mask_ex_static(ctypes.byref(big), None) == b.TSENOR_ERR_TOO_LARGE
    assert lib.tsenor_mask_ex_static(None, None) == b.TSENOR_ERR_NULL
    assert lib.tsenor_mask_ex_static(ctypes.byref(_problem(M=5)), None) == b.TSENOR_ERR_UNSUPPORTED
    assert b"TSENOR_STATIC_SCRATCH_BYTES" in lib.tsenor_status_string(b.TSENOR_ERR_TOO_LARGE)
    assert lib.tsenor_last_hip_error() == 0


def test_workspace_bytes(lib):
    from paper_2505_23949_amd import binding as b

    for M, rows, cols in [(4, 512, 512), (16, 4096, 4096), (32, 4096, 14336), (64, 8192, 28672)]:
        p = _problem(M=M, N=M // 2, rows=rows, cols=cols, ld=cols)
        need = lib.tsenor_workspace_bytes(ctypes.byref(p), 1)
        blocks = rows * cols // (M * M)
        # header + partial maxima of the pre-pass (1024 floats) + one uint16 per weight (greedy scan order)
        # + M row bit masks per block (32- or 64-bit words) + two doubles per block (objective of the mask
        # found and of the caller's previous mask)
        lower = 256 + 4096 + 2 * rows * cols + blocks * M * (8 if M > 32 else 4) + 16 * blocks
        assert lower <= need <= lower + 768
    arr = (b.tsenor_problem * 2)(_problem(), _problem(M=32, N=16, rows=64, cols=64, ld=64))
    assert lib.tsenor_workspace_bytes(arr, 2) == sum(lib.tsenor_workspace_bytes(ctypes.byref(x), 1) for x in arr)
    assert lib.tsenor_workspace_bytes(ctypes.byref(_problem(M=5)), 1) == 0
    assert lib.tsenor_workspace_bytes(None, 1) == 0


def test_status_strings_and_version(lib):
    from paper_2505_23949_amd import binding as b

    seen = set()
    for code in range(0, -8, -1):
        s = b.status_string(code)
        assert s and s != "unknown status"
        seen.add(s)
    assert len(seen) == 8 and b.status_string(-99) == "unknown status"
    assert b.version() >= 100


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in r.stderr


def test_product_path_never_touches_the_oracle():
    pkg = os.path.join(ROOT, "paper_2505_23949_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text and "tsenor_oracle" not in text, f
    for dirpath, _, files in os.walk(os.path.join(ROOT, "oracle")):
        for f in files:
            if f.endswith((".py", ".c")):
                assert "paper_2505_23949_amd" not in open(os.path.join(dirpath, f)).read(), f


def test_bf16_round_trip_of_the_input_generator():
    import numpy as np

    from paper_2505_23949_amd import synth

    x = np.array([1.0, 1.00390625, 1.01171875, -0.0, 3.3895314e38, 1e-40], dtype=np.float32)
    bits = synth.f32_to_bf16_bits(x)
    back = synth.bf16_bits_to_f32(bits)
    # 1 + 2^-8 is a tie and rounds to even (1.0); 1 + 3*2^-8 is a tie and rounds up to 1 + 2^-6
    assert back[0] == 1.0 and back[1] == 1.0 and back[2] == np.float32(1.015625)
    assert np.array_equal(synth.f32_to_bf16_bits(back), bits)
    g = synth.generate(synth.CONFIGS["cfg3_16of32_4096x14336"].scaled(64, 64))
    assert g["W_store"].dtype == np.uint16 and np.array_equal(synth.bf16_bits_to_f32(g["W_store"]), g["W_f32"])
    g2 = synth.generate(synth.CONFIGS["cfg3_16of32_4096x14336"].scaled(64, 64))
    assert np.array_equal(g["W_store"], g2["W_store"]) and np.array_equal(g["col_scale"], g2["col_scale"])


def test_validation_of_the_extended_fields(lib):
    from paper_2505_23949_amd import binding as b

    def call(p):
        return lib.tsenor_mask_ex(ctypes.byref(p), ctypes.c_void_p(0), 0, None)   # stops at the workspace check

    assert call(_problem(importance=2)) == b.TSENOR_ERR_UNSUPPORTED
    assert call(_problem(flags=b.TSENOR_FLAG_GREEDY_ONE_LANE | b.TSENOR_FLAG_GREEDY_M_LANES)) == b.TSENOR_ERR_PARAM
    assert call(_problem(flags=b.TSENOR_FLAG_GREEDY_M_LANES)) == b.TSENOR_ERR_WORKSPACE
    assert call(_problem(flags=b.TSENOR_FLAG_TILES_LARGE | b.TSENOR_FLAG_TILES_SMALL)) == b.TSENOR_ERR_PARAM
    assert call(_problem(flags=b.TSENOR_FLAG_TILES_SMALL)) == b.TSENOR_ERR_WORKSPACE
    assert call(_problem(tol=-1.0)) == b.TSENOR_ERR_PARAM
    assert call(_problem(tol=float("nan"))) == b.TSENOR_ERR_PARAM
    assert call(_problem(tol=1e-3, flags=b.TSENOR_FLAG_FP32_ITERATIONS)) == b.TSENOR_ERR_WORKSPACE
    assert call(_problem(tol=1e-3)) == b.TSENOR_ERR_WORKSPACE
    assert call(_problem(N=0, iters_done_out=0x4000)) == b.TSENOR_ERR_UNSUPPORTED
    assert call(_problem(add=0x3000, add_scale=float("inf"))) == b.TSENOR_ERR_PARAM
    assert call(_problem(add=0x3000, add_scale=0.5)) == b.TSENOR_ERR_WORKSPACE
    odd = dict(M=4, N=2, rows=8, cols=12, ld=12)
    assert call(_problem(**odd)) == b.TSENOR_ERR_WORKSPACE
    for field in ("packed_out", "pruned_out", "prev_mask"):
        assert call(_problem(**odd, **{field: 0x4000})) == b.TSENOR_ERR_SHAPE
    assert call(_problem(N=16, objective_out=0x4000)) == b.TSENOR_ERR_UNSUPPORTED
    assert call(_problem(N=0, prev_mask=0x4000)) == b.TSENOR_ERR_UNSUPPORTED
