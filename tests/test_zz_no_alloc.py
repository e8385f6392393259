"""The entry point that allocates nothing (tsenor_mask_ex_static) against tsenor_mask_ex, through the C ABI.

Two calls in a row on the library's fixed scratch, the second with a smaller input: every output must equal,
bit for bit, what tsenor_mask_ex gives with a caller-provided workspace (same kernels, same arithmetic), and the
first must also equal the CPU oracle.  Collected last, so that a failure here hides no other test.
"""
import ctypes

import numpy as np
import pytest

import oracle
from paper_2505_23949_amd import synth

pytestmark = pytest.mark.gpu


def _problem(binding, torch, w, dev, scratch_filler=None):
    g = synth.generate(w)
    if w.dtype == "bf16":
        W = torch.from_numpy(g["W_store"].view(np.int16)).to(dev).view(torch.bfloat16)
    else:
        W = torch.from_numpy(g["W_store"]).to(dev)
    cs = None if g["col_scale"] is None else torch.from_numpy(g["col_scale"]).to(dev)
    out = {
        "mask": torch.zeros(W.shape, dtype=torch.uint8, device=dev),
        "plan": torch.zeros(W.shape, dtype=torch.float64, device=dev),
        "stats": torch.zeros(4, dtype=torch.int64, device=dev),
        "tau_eff": torch.zeros(1, dtype=torch.float64, device=dev),
        "packed": torch.zeros((w.rows, w.cols // 8), dtype=torch.uint8, device=dev),
        "objective": torch.zeros(2, dtype=torch.float64, device=dev),
    }
    p = binding.make_problem(W, w.N, w.M, w.tau, w.iters, mask=out["mask"], col_scale=cs, tau_mode=w.tau_mode,
                             plan_out=out["plan"], stats_out=out["stats"], tau_eff_out=out["tau_eff"],
                             packed_out=out["packed"], objective_out=out["objective"])
    return g, p, out, (W, cs)


def test_static_scratch_entry_point_matches_the_workspace_one():
    import torch

    from paper_2505_23949_amd import binding

    assert torch.cuda.is_available(), "GPU tests need a GPU"
    lib = binding.load()
    dev = torch.device("cuda:0")
    # first a 16:32 matrix of 60 blocks, then a smaller 8:16 one: the second call finds the first one's
    # leftovers in the scratch
    cases = [synth.CONFIGS["cfg3_16of32_4096x14336"].scaled(192, 320, "static_first"),
             synth.CONFIGS["cfg2_8of16_4096"].scaled(48, 80, "static_second_smaller")]
    for w in cases:
        print(f"[case] static scratch {w.name} {w.rows}x{w.cols} {w.N}:{w.M}", flush=True)
        g, p_static, got, keep_a = _problem(binding, torch, w, dev)
        _, p_ws, want, keep_b = _problem(binding, torch, w, dev)
        binding.tsenor_mask_ex_static(p_static)
        work = torch.empty(binding.tsenor_workspace_bytes([p_ws]), dtype=torch.uint8, device=dev)
        binding.tsenor_mask_ex(p_ws, work)
        torch.cuda.synchronize()
        for name in want:
            assert torch.equal(got[name], want[name]), (w.name, name)
        ref = oracle.mask(g["W_f32"], w.N, w.M, w.tau, w.iters, col_scale=g["col_scale"], tau_mode=w.tau_mode,
                          return_plan=True)
        assert np.array_equal(got["mask"].cpu().numpy(), ref["mask"])
        assert np.abs(got["plan"].cpu().numpy() - np.exp(ref["log_S"])).max() <= 1e-9
        assert np.array_equal(got["stats"].cpu().numpy(), ref["stats"])

    # sizes beyond the fixed scratch are refused before anything is enqueued
    big = binding.tsenor_problem()
    big.W, big.mask = 0x1000, 0x2000                       # never dereferenced
    big.dtype, big.rows, big.cols, big.ld = binding.TSENOR_F32, 8192, 8192, 8192
    big.N, big.M, big.tau, big.tau_mode, big.iters = 16, 32, 0.01, binding.TSENOR_TAU_REL_MATRIX_MAX, 10
    assert binding.tsenor_workspace_bytes([big]) > binding.STATIC_SCRATCH_BYTES
    assert lib.tsenor_mask_ex_static(ctypes.byref(big), None) == binding.TSENOR_ERR_TOO_LARGE
    assert lib.tsenor_mask_ex_static(None, None) == binding.TSENOR_ERR_NULL
    big.M = 5
    assert lib.tsenor_mask_ex_static(ctypes.byref(big), None) == binding.TSENOR_ERR_UNSUPPORTED
