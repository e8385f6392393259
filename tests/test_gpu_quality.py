"""Solution quality of the HIP path against the exact optimum, and the ablation arms of App. B.2.1.

The arms are reached through the library's own parameters: rounding the entropy solution (T > 0) or the
importance itself (T = 0), with the full Algorithm 2, with greedy selection only (strict mode, L = 0) or with
the simple row-then-column rounding (TSENOR_FLAG_SIMPLE_ROUNDING).
The exact optimum of every block comes from the LP relaxation of Eq. (3) (integral: a capacitated bipartite
b-matching), solved on the CPU.  Relative error = (f(S*) - f(S)) / f(S*) as in Fig. 3 / Fig. 5.

Inputs are synthetic stand-ins for the LLaMA blocks of the paper, so the assertions are the orderings the
paper reports (Sec. 3.3, App. B.2.1), not its percentages.
"""
import numpy as np
import pytest

import oracle
from oracle import exact
from paper_2505_23949_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dev():
    import torch

    from paper_2505_23949_amd import binding

    assert torch.cuda.is_available(), "GPU tests need a GPU"
    binding.load()
    return torch.device("cuda:0")


def _relative_errors(mask, imp, opt, M, feasible=True):
    got = (exact.blocks(mask, M) * exact.blocks(imp, M)).sum(axis=(1, 2))
    if feasible:
        # (the LP solver stops at a relative tolerance of ~1e-9; a mask with short rows, as greedy selection
        # alone can leave, is outside the feasible set and may exceed the optimum)
        assert np.all(got <= opt * (1 + 1e-7)), "a feasible mask cannot beat the exact optimum"
    return (opt - got) / opt


@pytest.mark.parametrize("N,M,block_rows,block_cols", [(2, 4, 16, 32), (4, 8, 8, 16), (8, 16, 6, 12), (16, 32, 3, 8),
                                                       (32, 64, 2, 3)])
def test_ablation_arms_against_the_exact_optimum(dev, N, M, block_rows, block_cols):
    import torch

    from paper_2505_23949_amd import binding

    w = synth.Workload(f"quality_{N}of{M}", block_rows * M, block_cols * M, N, M, 0.005, 300, "f32", "wanda", 3100 + M)
    g = synth.generate(w)
    W = torch.from_numpy(g["W_store"]).to(dev)
    cs = torch.from_numpy(g["col_scale"]).to(dev)
    imp = oracle.importance(g["W_f32"], g["col_scale"]).astype(np.float64)
    opt = np.array([exact.lp_optimum(b, N)[0] for b in exact.blocks(imp, M)])

    def arm(iters, greedy_only, simple=False):
        kw = dict(local_search_steps=0, flags=binding.TSENOR_FLAG_STRICT_PAPER) if greedy_only else {}
        if simple:
            kw = dict(flags=binding.TSENOR_FLAG_SIMPLE_ROUNDING)
        res = binding.solve(W, N, M, w.tau, iters, col_scale=cs, tau_mode=w.tau_mode, want_stats=simple, **kw)
        torch.cuda.synchronize()
        mask = res["mask"].cpu().numpy()
        if simple:
            # the arm itself against its definition: row-wise then column-wise top-N of the oracle's plan
            te = oracle.tau_eff(imp.astype(np.float32), w.tau, w.tau_mode)
            key = oracle.dykstra(imp.astype(np.float32), N, M, te, iters) if iters else imp
            want = oracle.simple_round(key, N, M)
            assert np.array_equal(mask, want)
            missing = N * mask.shape[0] * mask.shape[1] // M - int(mask.sum())
            assert res["stats"].cpu().numpy().tolist() == [missing, 0, 0, missing]
        elif not greedy_only:
            assert exact.is_transposable_nm(mask, N, M)
        return _relative_errors(mask, imp, opt, M, feasible=not (greedy_only or simple)).mean()

    print(f"[case] ablation arms {N}:{M}, {len(opt)} blocks", flush=True)
    entropy_optround = arm(300, False)      # the method
    entropy_greedy = arm(300, True)         # "Entropy + Greedy"
    direct_optround = arm(0, False)         # Algorithm 2 on the importance itself
    direct_greedy = arm(0, True)            # greedy selection on the importance itself
    entropy_simple = arm(300, False, simple=True)   # "Entropy" of Fig. 3 / "Entropy + Simple" of Fig. 5
    direct_simple = arm(0, False, simple=True)
    print(f"  mean relative error: entropy+optround {entropy_optround:.5f}, entropy+greedy {entropy_greedy:.5f}, "
          f"entropy+simple {entropy_simple:.5f}, optround {direct_optround:.5f}, greedy {direct_greedy:.5f}, "
          f"simple {direct_simple:.5f}", flush=True)
    # the rounding of Algorithm 2 beats simple rounding by a wide margin on either key (Sec. 5.1, App. B.2.1)
    assert entropy_optround < 0.5 * entropy_simple
    assert direct_optround < 0.5 * direct_simple
    assert entropy_greedy < entropy_simple and direct_greedy < direct_simple
    # local search improves on greedy selection, with and without the entropy solution (App. B.2.1)
    assert entropy_optround < entropy_greedy
    assert direct_optround < direct_greedy
    # rounding the entropy solution beats rounding the importance directly (Sec. 3.3 (i), App. B.2.1)
    assert entropy_optround < direct_optround
    # the full method is close to optimal on these inputs
    assert entropy_optround < 0.01


def test_cfg1_relative_error_against_brute_force(dev):
    # the 2:4 workload at full size: every one of its 16384 blocks against the best of the 90 feasible masks.
    # The paper prints no number for M = 4 (its figures start at M = 8), so the magnitudes are this build's own
    # ("parity unpinned"); what is pinned is the sign (a feasible mask never beats the optimum) and that Algorithm 2
    # with the entropy solution is no worse than greedy selection alone.
    import torch

    from paper_2505_23949_amd import binding

    w = synth.CONFIGS["cfg1_2of4_512"]
    g = synth.generate(w)
    W = torch.from_numpy(g["W_store"]).to(dev)
    imp = oracle.importance(g["W_f32"], None).astype(np.float64)
    masks90 = exact.feasible_masks(w.M, w.N)
    assert len(masks90) == 90
    blocks = exact.blocks(imp, w.M).reshape(-1, w.M * w.M)
    opt = (blocks @ masks90.reshape(90, -1).T.astype(np.float64)).max(axis=1)
    res = binding.solve(W, w.N, w.M, w.tau, w.iters, tau_mode=w.tau_mode)
    greedy = binding.solve(W, w.N, w.M, w.tau, w.iters, tau_mode=w.tau_mode, local_search_steps=0,
                           flags=binding.TSENOR_FLAG_STRICT_PAPER)
    torch.cuda.synchronize()
    mask = res["mask"].cpu().numpy()
    assert exact.is_transposable_nm(mask, w.N, w.M)
    err = _relative_errors(mask, imp, opt, w.M)
    err_greedy = _relative_errors(greedy["mask"].cpu().numpy(), imp, opt, w.M, feasible=False)
    optimal = float((err <= 1e-12).mean())
    print(f"[case] cfg1 2:4, {len(opt)} blocks against brute force: mean relative error {err.mean():.6f}, "
          f"max {err.max():.4f}, optimal blocks {optimal:.4f}; greedy selection only: mean {err_greedy.mean():.6f}",
          flush=True)
    assert err.min() >= -1e-12
    assert err.mean() <= err_greedy.mean()
    assert optimal >= 0.9 and err.mean() < 0.005


def test_cfg2_relative_error_against_the_lp_on_a_block_sample(dev):
    # the 8:16 workload at full size: the GPU's mask of every 64th block (1024 blocks) against the exact optimum
    # of Eq. (3) (the metric of Sec. 5.1 / Fig. 3; the paper's values exist only as curves, so the magnitude is
    # "parity unpinned" and only the sign and the order of the arms are asserted)
    import torch

    from paper_2505_23949_amd import binding

    w = synth.CONFIGS["cfg2_8of16_4096"]
    g = synth.generate(w)
    W = torch.from_numpy(g["W_store"]).to(dev)
    res = binding.solve(W, w.N, w.M, w.tau, w.iters, tau_mode=w.tau_mode)
    greedy = binding.solve(W, w.N, w.M, w.tau, w.iters, tau_mode=w.tau_mode, local_search_steps=0,
                           flags=binding.TSENOR_FLAG_STRICT_PAPER)
    direct = binding.solve(W, w.N, w.M, w.tau, 0, tau_mode=w.tau_mode)
    torch.cuda.synchronize()
    imp = oracle.importance(g["W_f32"], None).astype(np.float64)
    pick = np.arange(0, (w.rows // w.M) * (w.cols // w.M), 64)
    assert len(pick) == 1024
    imp_b = exact.blocks(imp, w.M)[pick]
    print(f"[case] cfg2 8:16: exact optimum of {len(pick)} sampled blocks", flush=True)
    opt = np.array([exact.lp_optimum(b, w.N)[0] for b in imp_b])

    def errors(mask, feasible=True):
        got = (exact.blocks(mask, w.M)[pick] * imp_b).sum(axis=(1, 2))
        if feasible:
            assert np.all(got <= opt * (1 + 1e-7))
        return (opt - got) / opt

    mask = res["mask"].cpu().numpy()
    assert exact.is_transposable_nm(mask, w.N, w.M)
    e_full, e_greedy, e_direct = errors(mask), errors(greedy["mask"].cpu().numpy(), False), \
        errors(direct["mask"].cpu().numpy())
    print(f"  mean relative error: entropy + Algorithm 2 {e_full.mean():.6f} (max {e_full.max():.5f}), "
          f"entropy + greedy only {e_greedy.mean():.6f}, Algorithm 2 on the importance {e_direct.mean():.6f}", flush=True)
    assert e_full.mean() < e_greedy.mean() and e_full.mean() < e_direct.mean()
    assert e_full.mean() < 0.01


def test_a_converged_plan_rounds_better(dev):
    # the error as a function of the iteration budget: a plan far from convergence (10 iterations) rounds
    # worse than the importance itself, a converged one (1000) much better than either
    import torch

    from paper_2505_23949_amd import binding

    N, M = 8, 16
    w = synth.Workload("quality_iters", 8 * M, 16 * M, N, M, 0.005, 0, "f32", "normal", 3200)
    g = synth.generate(w)
    W = torch.from_numpy(g["W_store"]).to(dev)
    imp = oracle.importance(g["W_f32"], None).astype(np.float64)
    opt = np.array([exact.lp_optimum(b, N)[0] for b in exact.blocks(imp, M)])
    errs = []
    for iters in (0, 10, 100, 1000):
        res = binding.solve(W, N, M, w.tau, iters, tau_mode=w.tau_mode)
        torch.cuda.synchronize()
        errs.append(_relative_errors(res["mask"].cpu().numpy(), imp, opt, M).mean())
    print(f"[case] mean relative error after 0/10/100/1000 iterations: {errs}", flush=True)
    assert errs[3] < errs[2] < errs[1]
    assert errs[3] < 0.5 * errs[0]
