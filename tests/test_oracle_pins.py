"""Pins of the CPU oracle against what the paper and the mathematics fix (no GPU).

Each test names the passage it checks.  A plausible mistake in the oracle
(a dropped dual term, a wrong sign, a transposed operand, a wrong tie-break)
fails at least one of them.
"""
import itertools

import numpy as np
import pytest

import oracle
from oracle import exact


def _arr(rows, dtype=np.float64):
    return np.array([[float(t) for t in r] for r in rows], dtype=dtype)


# ----------------------------------------------------------------------------------------------
# Fig. 2: the printed worked example (greedy mask, swap-score matrix, final mask, both objectives)
# ----------------------------------------------------------------------------------------------

def test_fig2_greedy_selection(golden_fig2):
    W = _arr(golden_fig2["abs_w"], np.float32)
    want = _arr(golden_fig2["greedy_mask"]).astype(np.uint8)
    got, stats = oracle.round_plan(W.astype(np.float64), W, 2, 4, L=0, strict_paper=True)
    assert np.array_equal(got, want)
    assert stats[0] == 1 and stats[3] == 1          # one unit missing: row 4 and column 4 hold one entry
    assert round(float((got * W.astype(np.float64)).sum()), 2) == float(golden_fig2["greedy_objective"][0][0])


def test_fig2_swap_scores(golden_fig2):
    W = _arr(golden_fig2["abs_w"], np.float32)
    S = _arr(golden_fig2["greedy_mask"]).astype(np.uint8)
    got = oracle.swap_scores(W, S, 3, 3)            # (i, j) = (4, 4) in the paper's 1-based indices
    want = np.array([[-np.inf if t == "-inf" else float(t) for t in r] for r in golden_fig2["swap_scores"]])
    assert np.array_equal(np.isinf(got), np.isinf(want))
    fin = ~np.isinf(want)
    assert np.allclose(got[fin], want[fin], atol=5e-3)   # printed to two decimals
    bi, bj = np.unravel_index(np.argmax(got), got.shape)
    assert [bi + 1, bj + 1] == [int(t) for t in golden_fig2["best_swap_1based"][0]]


def test_fig2_local_search_result(golden_fig2):
    W = _arr(golden_fig2["abs_w"], np.float32)
    want = _arr(golden_fig2["final_mask"]).astype(np.uint8)
    for strict in (True, False):
        got, stats = oracle.round_plan(W.astype(np.float64), W, 2, 4, L=10, strict_paper=strict)
        assert np.array_equal(got, want)
        assert stats[3] == 0
    assert round(float((want * W.astype(np.float64)).sum()), 2) == float(golden_fig2["final_objective"][0][0])


def test_fig2_final_mask_is_the_brute_force_optimum(golden_fig2):
    W = _arr(golden_fig2["abs_w"], np.float32)
    masks = exact.feasible_masks(4, 2)
    assert len(masks) == 90                          # all transposable 2:4 patterns of a 4x4 block
    assert round(exact.brute_force_optimum(W, 2, masks), 2) == float(golden_fig2["final_objective"][0][0])


# ----------------------------------------------------------------------------------------------
# Exact optimum of Eq. (2)/(3): the heuristic never beats it, the two exact solvers agree
# ----------------------------------------------------------------------------------------------

def test_exact_solvers_agree_on_small_blocks():
    rng = np.random.default_rng(7)
    masks = exact.feasible_masks(4, 2)
    for _ in range(25):
        blk = np.abs(rng.standard_normal((4, 4))).astype(np.float32)
        lp, vertex = exact.lp_optimum(blk, 2)
        assert abs(lp - exact.brute_force_optimum(blk, 2, masks)) < 1e-9
        assert np.allclose(vertex, np.round(vertex), atol=1e-9)      # Sec. 3.1: vertices are integral
    m63 = exact.feasible_masks(6, 3)
    blk = np.abs(rng.standard_normal((6, 6)))
    assert abs(exact.lp_optimum(blk, 3)[0] - exact.brute_force_optimum(blk, 3, m63)) < 1e-9


def test_full_path_vs_brute_force_2of4():
    rng = np.random.Generator(np.random.Philox(11))
    W = rng.standard_normal((64, 64), dtype=np.float32)
    res = oracle.mask(W, 2, 4, 0.01, 200, tau_mode=oracle.TAU_REL_MATRIX_MAX)
    assert exact.is_transposable_nm(res["mask"], 2, 4)
    masks = exact.feasible_masks(4, 2)
    imp_b = exact.blocks(np.abs(W), 4).astype(np.float64)
    got = (exact.blocks(res["mask"], 4) * imp_b).sum(axis=(1, 2))
    opt = np.array([exact.brute_force_optimum(b, 2, masks) for b in imp_b])
    assert np.all(got <= opt + 1e-9)
    assert np.mean(got >= opt - 1e-9) > 0.9          # near-optimal on most blocks (paper: 1-10% error at worst)
    assert np.mean((opt - got) / opt) < 0.01


@pytest.mark.parametrize("N,M,blocks", [(4, 8, 16), (8, 16, 6)])
def test_full_path_vs_lp_optimum(N, M, blocks):
    rng = np.random.Generator(np.random.Philox(100 + M))
    W = rng.standard_normal((M, M * blocks), dtype=np.float32)
    res = oracle.mask(W, N, M, 0.01, 300, tau_mode=oracle.TAU_REL_MATRIX_MAX)
    assert exact.is_transposable_nm(res["mask"], N, M)
    greedy_only, _ = oracle.round_plan(np.abs(W).astype(np.float64), np.abs(W), N, M, L=0, strict_paper=True)
    imp_b = exact.blocks(np.abs(W), M).astype(np.float64)
    got = (exact.blocks(res["mask"], M) * imp_b).sum(axis=(1, 2))
    opt = np.array([exact.lp_optimum(b, N)[0] for b in imp_b])
    assert np.all(got <= opt + 1e-9)
    assert np.mean((opt - got) / opt) < 0.02
    # Sec. 3.3 (i): rounding the entropy solution beats greedy on |W| itself, on average
    g = (exact.blocks(greedy_only, M) * imp_b).sum(axis=(1, 2))
    assert got.mean() > g.mean()


# ----------------------------------------------------------------------------------------------
# Algorithm 1: closed forms, special cases, the linear-domain statement, optimality conditions
# ----------------------------------------------------------------------------------------------

def _alg1_linear(absW, N, tau, T):
    """Algorithm 1 exactly as stated (linear domain, S and Q as matrices)."""
    S = np.exp(tau * absW.astype(np.float64))
    Q = np.ones_like(S)
    ones = np.ones(S.shape[0])
    for _ in range(T):
        S = np.diag(N / (S @ ones)) @ S
        S = S @ np.diag(N / (S.T @ ones))
        S_new = np.minimum(S * Q, 1.0)
        Q = Q * (S / S_new)
        S = S_new
    return S, Q


@pytest.mark.parametrize("N,M", [(2, 4), (4, 8), (3, 5), (8, 16)])
def test_log_domain_equals_linear_domain_algorithm1(N, M):
    rng = np.random.default_rng(3 * M + N)
    blk = np.abs(rng.standard_normal((M, M))).astype(np.float32)
    for tau, T in [(0.5, 1), (3.0, 2), (6.0, 7), (12.0, 60)]:
        S_lin, Q_lin = _alg1_linear(blk, N, tau, T)
        log_S, log_Q = oracle.dykstra(blk, N, M, tau, T, return_log_Q=True)
        assert np.allclose(np.exp(log_S), S_lin, rtol=1e-10, atol=1e-300)
        assert np.allclose(np.exp(log_Q), Q_lin, rtol=1e-10)
        assert (np.exp(log_Q) > 1 + 1e-9).any() or tau < 3   # the cap is active in the harder settings


def _sinkhorn_knopp(Kmat, N, T):
    """Textbook matrix scaling of exp(K) to marginals (N, ..., N): u, v updates, no cap."""
    G = np.exp(Kmat)
    v = np.ones(G.shape[1])
    for _ in range(T):
        u = N / (G @ v)
        v = N / (G.T @ u)
    return u[:, None] * G * v[None, :]


@pytest.mark.parametrize("M", [4, 7, 16])
def test_reduces_to_sinkhorn_when_cap_cannot_bind(M):
    # N = 1: every entry is at most its row sum 1, so the box constraint never binds and Q stays 1.
    rng = np.random.default_rng(M)
    blk = np.abs(rng.standard_normal((M, M))).astype(np.float32)
    tau, T = 4.0, 25
    log_S, log_Q = oracle.dykstra(blk, 1, M, tau, T, return_log_Q=True)
    assert np.allclose(np.exp(log_S), _sinkhorn_knopp(tau * blk.astype(np.float64), 1, T), rtol=1e-11)
    assert np.allclose(log_Q, 0.0, atol=1e-12)
    assert np.allclose(np.exp(log_S).sum(axis=0), 1.0, rtol=1e-12)   # last scaling was the column one


def test_two_by_two_closed_form():
    # M = 2, N = 1: the fixed point is [[p, 1-p], [1-p, p]] with p = sigmoid(tau (w11 + w22 - w12 - w21) / 2)
    blk = np.array([[0.9, 0.2], [0.4, 0.3]], dtype=np.float32)
    tau = 3.0
    b = blk.astype(np.float64)
    p = 1.0 / (1.0 + np.exp(-tau * (b[0, 0] + b[1, 1] - b[0, 1] - b[1, 0]) / 2.0))
    S = np.exp(oracle.dykstra(blk, 1, 2, tau, 400))
    assert np.allclose(S, [[p, 1 - p], [1 - p, p]], atol=1e-12)


def test_uniform_and_full_blocks():
    blk = np.full((8, 8), 0.37, dtype=np.float32)
    log_S, log_Q = oracle.dykstra(blk, 3, 8, 5.0, 1, return_log_Q=True)
    assert np.allclose(np.exp(log_S), 3 / 8, rtol=1e-13) and np.allclose(log_Q, 0.0, atol=1e-13)
    rng = np.random.default_rng(0)
    blk = np.abs(rng.standard_normal((4, 4))).astype(np.float32)
    S = np.exp(oracle.dykstra(blk, 4, 4, 2.0, 3000))
    assert np.allclose(S, 1.0, atol=1e-6)           # N = M: the only feasible plan is all ones


def test_projection_closed_forms_and_order():
    rng = np.random.default_rng(5)
    blk = np.abs(rng.standard_normal((8, 8))).astype(np.float32)
    tau = 6.0
    # first iteration, written out: rows scaled to N, columns scaled to N, then the cap with Q = 1
    S0 = np.exp(tau * blk.astype(np.float64))
    S1 = S0 * (4 / S0.sum(axis=1, keepdims=True))
    S2 = S1 * (4 / S1.sum(axis=0, keepdims=True))
    log_S, log_Q = oracle.dykstra(blk, 4, 8, tau, 1, return_log_Q=True)
    assert np.allclose(np.exp(log_S), np.minimum(S2, 1.0), rtol=1e-12)
    assert np.allclose(np.exp(log_Q), np.maximum(S2, 1.0), rtol=1e-12)
    assert (S2 > 1).any() and log_S.max() == 0.0
    # columns first is the same algorithm on the transposed block
    a = oracle.dykstra(blk, 4, 8, tau, 9, cols_first=True)
    b = oracle.dykstra(np.ascontiguousarray(blk.T), 4, 8, tau, 9)
    assert np.allclose(a, b.T, rtol=0, atol=1e-13)
    assert not np.allclose(a, oracle.dykstra(blk, 4, 8, tau, 9), atol=1e-6)


@pytest.mark.parametrize("N,M", [(2, 4), (3, 6), (8, 16)])
def test_dual_structure_at_every_iteration(N, M):
    # log S + log Q - K is a sum of a row term and a column term after every iteration (Dykstra with a
    # single dual for the box, App. A.1), S <= 1, Q >= 1 and Q > 1 only where S = 1.
    rng = np.random.default_rng(N * M)
    blk = np.abs(rng.standard_normal((M, M))).astype(np.float32)
    tau = 8.0
    K = tau * blk.astype(np.float64)
    for T in (1, 2, 3, 10, 50):
        log_S, log_Q = oracle.dykstra(blk, N, M, tau, T, return_log_Q=True)
        D = log_S + log_Q - K
        mixed = D[:-1, :-1] - D[:-1, 1:] - D[1:, :-1] + D[1:, 1:]
        assert np.abs(mixed).max() < 1e-10
        assert log_S.max() <= 0.0 and log_Q.min() >= 0.0
        assert np.all((log_Q == 0.0) | (log_S == 0.0))


def test_converged_plan_solves_the_regularised_problem():
    from scipy.optimize import minimize

    rng = np.random.default_rng(21)
    M, N, tau = 4, 2, 5.0
    blk = np.abs(rng.standard_normal((M, M))).astype(np.float32)
    S = np.exp(oracle.dykstra(blk, N, M, tau, 20000))
    assert np.allclose(S.sum(axis=0), N, atol=1e-9) and np.allclose(S.sum(axis=1), N, atol=1e-9)
    assert (S > 1 - 1e-12).any()                     # the cap is active at the optimum of this instance
    b = blk.astype(np.float64)

    def neg_obj(x):                                  # Eq. (4): <S,|W|> + H(S)/tau, to be maximised
        x = np.clip(x, 1e-300, None)
        return -(np.dot(x, b.ravel()) - np.sum(x * np.log(x)) / tau)

    def neg_grad(x):
        x = np.clip(x, 1e-300, None)
        return -(b.ravel() - (np.log(x) + 1.0) / tau)

    A = np.zeros((2 * M - 1, M * M))                 # the 2M marginal equations have rank 2M - 1
    for i in range(M):
        A[i, i * M:(i + 1) * M] = 1.0
    for j in range(M - 1):
        A[M + j, j::M] = 1.0
    r = minimize(neg_obj, np.full(M * M, N / M), jac=neg_grad, bounds=[(1e-10, 1.0)] * (M * M),
                 constraints=[{"type": "eq", "fun": lambda x: A @ x - N, "jac": lambda x: A}],
                 method="SLSQP", options={"ftol": 1e-15, "maxiter": 5000})
    assert r.success
    assert neg_obj(S.ravel()) <= r.fun + 1e-9        # at least as good as the generic solver's point
    assert np.allclose(S, r.x.reshape(M, M), atol=1e-6)


@pytest.mark.parametrize("N,M", [(2, 4), (4, 8)])
def test_regularisation_error_bound(N, M):
    # H <= M N ln(M/N) on the feasible set and H(S*) = 0, so <S_tau,|W|> >= OPT - M N ln(M/N) / tau.
    rng = np.random.default_rng(M)
    blk = np.abs(rng.standard_normal((M, M))).astype(np.float32)
    opt = exact.lp_optimum(blk, N)[0]
    for tau in (2.0, 10.0, 40.0):
        S = np.exp(oracle.dykstra(blk, N, M, tau, 20000))
        val = float((S * blk.astype(np.float64)).sum())
        assert val <= opt + 1e-7
        assert val >= opt - M * N * np.log(M / N) / tau - 1e-7


def test_equivariances():
    rng = np.random.default_rng(9)
    M, N, tau, T = 8, 4, 7.0, 40
    blk = np.abs(rng.standard_normal((M, M))).astype(np.float32)
    base = oracle.dykstra(blk, N, M, tau, T)
    # (tau, W) -> (tau / a, a W) with a a power of two is the same problem bit for bit
    assert np.array_equal(base, oracle.dykstra(blk * np.float32(4.0), N, M, tau / 4.0, T))
    # permuting columns permutes the plan
    pc = rng.permutation(M)
    assert np.allclose(oracle.dykstra(np.ascontiguousarray(blk[:, pc]), N, M, tau, T), base[:, pc], atol=1e-12)
    pr = rng.permutation(M)
    assert np.allclose(oracle.dykstra(np.ascontiguousarray(blk[pr]), N, M, tau, T), base[pr], atol=1e-12)
    # blocks are independent: the plan of a tiled matrix is the tiling of the plans
    big = np.block([[blk, blk.T], [blk[::-1].copy(), blk]]).astype(np.float32)
    out = oracle.dykstra(big, N, M, tau, T)
    assert np.array_equal(out[:M, :M], base) and np.array_equal(out[M:, M:], base)
    assert np.array_equal(out[:M, M:], oracle.dykstra(np.ascontiguousarray(blk.T), N, M, tau, T))


# ----------------------------------------------------------------------------------------------
# Algorithm 2: invariants, orderings, tie-breaks, modes
# ----------------------------------------------------------------------------------------------

def _greedy_reference(key, N):
    """Greedy selection by direct definition: scan (key desc, flat index asc)."""
    M = key.shape[0]
    order = sorted(range(M * M), key=lambda k: (-key.flat[k], k))
    S = np.zeros((M, M), dtype=np.uint8)
    for k in order:
        i, j = divmod(k, M)
        if S[i].sum() < N and S[:, j].sum() < N:
            S[i, j] = 1
    return S


def _local_search_reference(S, imp, N, max_rounds=None, strict=False):
    """Local search by direct definition of Eq. (5), lowest-index deficient row/column and arg-max."""
    S = S.copy()
    M = S.shape[0]
    imp = imp.astype(np.float64)
    rounds = 0
    while True:
        rdef = [i for i in range(M) if S[i].sum() < N]
        cdef = [j for j in range(M) if S[:, j].sum() < N]
        if not rdef or (max_rounds is not None and rounds >= max_rounds):
            return S
        i, j = rdef[0], cdef[0]
        best, arg = None, None
        for ip, jp in itertools.product(range(M), range(M)):
            if S[ip, jp] == 1 and S[i, jp] == 0 and S[ip, j] == 0:
                sc = imp[i, jp] + imp[ip, j] - imp[ip, jp]
                if best is None or sc > best:
                    best, arg = sc, (ip, jp)
        rounds += 1
        if arg is None or (strict and not best > 0):
            return S
        S[arg] = 0
        S[arg[0], j] = 1
        S[i, arg[1]] = 1


@pytest.mark.parametrize("N,M", [(2, 4), (4, 8), (8, 16), (5, 12), (16, 32)])
def test_rounding_matches_direct_definition(N, M):
    rng = np.random.default_rng(1000 + M)
    nb = 6
    imp = np.abs(rng.standard_normal((M, M * nb))).astype(np.float32)
    key = rng.random((M, M * nb))
    key[rng.random(key.shape) < 0.25] = 0.75         # many exact ties, as at the cap
    got_g, _ = oracle.round_plan(key, imp, N, M, L=0, strict_paper=True)
    got_s, st_s = oracle.round_plan(key, imp, N, M, L=2, strict_paper=True)
    got_d, st_d = oracle.round_plan(key, imp, N, M, L=10)
    for b in range(nb):
        sl = slice(b * M, (b + 1) * M)
        g = _greedy_reference(key[:, sl], N)
        assert np.array_equal(got_g[:, sl], g)
        assert np.array_equal(got_s[:, sl], _local_search_reference(g, imp[:, sl], N, max_rounds=2, strict=True))
        assert np.array_equal(got_d[:, sl], _local_search_reference(g, imp[:, sl], N))
    assert exact.is_transposable_nm(got_d, N, M) and st_d[3] == 0
    # a positive swap never lowers the objective (Sec. 3.3)
    obj = lambda m: float((m * imp.astype(np.float64)).sum())
    assert obj(got_s) >= obj(got_g)


def test_local_search_always_reaches_feasibility_from_adversarial_keys():
    # keys that make greedy strand capacity: large on one diagonal band only
    rng = np.random.default_rng(77)
    for N, M in [(2, 4), (3, 6), (4, 8), (8, 16)]:
        for _ in range(20):
            key = rng.random((M, M)) ** 8
            imp = np.abs(rng.standard_normal((M, M))).astype(np.float32)
            m, st = oracle.round_plan(key, imp, N, M, L=1)
            assert exact.is_transposable_nm(m, N, M)
            assert st[3] == 0


def test_tie_break_is_ascending_flat_index():
    key = np.zeros((4, 4))
    imp = np.ones((4, 4), dtype=np.float32)
    m, st = oracle.round_plan(key, imp, 2, 4, L=0, strict_paper=True)
    # scanning (0,0),(0,1),(0,2)... fills rows 0-1 in columns 0-1 and rows 2-3 in columns 2-3
    want = np.array([[1, 1, 0, 0], [1, 1, 0, 0], [0, 0, 1, 1], [0, 0, 1, 1]], dtype=np.uint8)
    assert np.array_equal(m, want) and st[0] == 0


# ----------------------------------------------------------------------------------------------
# Input transform, tau modes, the composed path
# ----------------------------------------------------------------------------------------------

def test_importance_and_tau_modes():
    rng = np.random.default_rng(2)
    W = rng.standard_normal((8, 16)).astype(np.float32)
    c = rng.lognormal(0, 1, 16).astype(np.float32)
    assert np.array_equal(oracle.importance(W), np.abs(W))
    imp = oracle.importance(W, c)
    assert imp.dtype == np.float32 and np.array_equal(imp, np.abs(W) * c[None, :])
    assert oracle.tau_eff(imp, 0.25, oracle.TAU_ABSOLUTE) == 0.25
    assert oracle.tau_eff(imp, 0.005, oracle.TAU_REL_MATRIX_MAX) == 1.0 / (0.005 * float(imp.max()))
    assert oracle.tau_eff(np.zeros((4, 4), np.float32), 0.005, oracle.TAU_REL_MATRIX_MAX) == 0.0


def test_composed_path_equals_its_steps():
    rng = np.random.Generator(np.random.Philox(5))
    W = (0.02 * rng.standard_normal((32, 64))).astype(np.float32)
    c = rng.lognormal(0, 1, 64).astype(np.float32)
    res = oracle.mask(W, 8, 16, 0.005, 120, col_scale=c, tau_mode=oracle.TAU_REL_MATRIX_MAX, return_plan=True)
    imp = oracle.importance(W, c)
    te = oracle.tau_eff(imp, 0.005, oracle.TAU_REL_MATRIX_MAX)
    log_S = oracle.dykstra(imp, 8, 16, te, 120)
    m, st = oracle.round_plan(log_S, imp, 8, 16)
    assert res["tau_eff"] == te
    assert np.array_equal(res["log_S"], log_S) and np.array_equal(res["mask"], m)
    assert np.array_equal(res["stats"], st)
    assert exact.is_transposable_nm(m, 8, 16)
    # degenerate N
    assert oracle.mask(W, 0, 16, 0.005, 5)["mask"].sum() == 0
    assert oracle.mask(W, 16, 16, 0.005, 5)["mask"].all()


def test_log_domain_survives_large_logits():
    # the paper's default entropy weight gives logits up to 1/0.005 = 200: exp() of them overflows
    # nothing in the log-domain form, and the plan is still a valid sub-stochastic matrix
    rng = np.random.Generator(np.random.Philox(8))
    W = rng.standard_t(3.0, (32, 32)).astype(np.float32)
    res = oracle.mask(W, 16, 32, 0.002, 300, tau_mode=oracle.TAU_REL_MATRIX_MAX, return_plan=True)
    S = np.exp(res["log_S"])
    assert np.isfinite(res["log_S"]).all() and S.max() <= 1.0
    assert np.abs(S.sum(axis=0) - 16).max() < 0.5 and np.abs(S.sum(axis=1) - 16).max() < 0.5
    assert exact.is_transposable_nm(res["mask"], 16, 32)


# ----------------------------------------------------------------------------------------------
# Importance transforms of Sec. 4 / Proposition 1, objective of Eq. (1), safeguard of App. A.1
# ----------------------------------------------------------------------------------------------

def test_importance_transforms_are_single_float_operations():
    rng = np.random.default_rng(31)
    W = rng.standard_normal((8, 16)).astype(np.float32)
    V = rng.standard_normal((8, 16)).astype(np.float32)
    c = rng.lognormal(0, 1, 16).astype(np.float32)
    f32 = np.float32
    x = (W + (f32(0.37) * V).astype(f32)).astype(f32)
    imp, val = oracle.importance_ex(W, add=V, add_scale=0.37, col_scale=c, square=True)
    a = (np.abs(x) * c).astype(f32)
    assert np.array_equal(val, x) and np.array_equal(imp, (a * a).astype(f32))
    imp2, val2 = oracle.importance_ex(W, col_scale=c)
    assert np.array_equal(val2, W) and np.array_equal(imp2, oracle.importance(W, c))
    # (W + V/rho)^2 of Proposition 1 with rho = 4
    imp3, _ = oracle.importance_ex(W, add=V, add_scale=0.25, square=True)
    assert np.allclose(imp3, (W.astype(np.float64) + V / 4.0) ** 2, rtol=1e-6)


def test_objective_packing_and_safeguard():
    rng = np.random.default_rng(32)
    W = rng.standard_normal((16, 32)).astype(np.float32)
    imp = oracle.importance(W)
    res = oracle.solve_ex(W, 4, 8, 0.01, 100, tau_mode=oracle.TAU_REL_MATRIX_MAX)
    m = res["mask"]
    assert abs(res["objective"] - float((m * imp.astype(np.float64)).sum())) < 1e-9
    assert np.array_equal(res["pruned"], W * m)
    bits = np.unpackbits(res["packed"], axis=1, bitorder="little")
    assert np.array_equal(bits, m) and res["packed"][0, 0] == sum(int(m[0, k]) << k for k in range(8))
    # a previous mask that is worse is ignored, one that is better (the exact optimum) replaces the result
    worse, _ = oracle.round_plan(-imp.astype(np.float64), imp, 4, 8)          # greedy on the smallest weights
    r1 = oracle.solve_ex(W, 4, 8, 0.01, 100, tau_mode=oracle.TAU_REL_MATRIX_MAX, prev_mask=worse)
    assert not r1["used_prev"] and np.array_equal(r1["mask"], m) and r1["objective_prev"] < r1["objective"]
    best = np.zeros_like(m)
    for b in range(8):
        r0, c0 = (b // 4) * 8, (b % 4) * 8
        best[r0:r0 + 8, c0:c0 + 8] = np.round(exact.lp_optimum(imp[r0:r0 + 8, c0:c0 + 8], 4)[1]).astype(np.uint8)
    r2 = oracle.solve_ex(W, 4, 8, 0.01, 0, tau_mode=oracle.TAU_REL_MATRIX_MAX, L=0, strict_paper=True, prev_mask=best)
    assert r2["objective_prev"] >= r2["objective_new"]
    if r2["objective_prev"] > r2["objective_new"]:
        assert r2["used_prev"] and np.array_equal(r2["mask"], best) and r2["objective"] == r2["objective_prev"]
        assert np.array_equal(r2["pruned"], W * best)


def test_simple_rounding_arm():
    # App. B.2.1 "Simple": row-wise then column-wise N:M rounding.  Pins: a hand-worked 4x4 case, the bounds
    # every result obeys, and agreement with the full method where the answer is forced.
    key = np.array([[9, 8, 1, 0], [7, 6, 5, 0], [4, 3, 2, 1], [9, 9, 9, 9]], dtype=np.float64)
    # rows keep {0,1}, {0,1}, {0,1}, {0,1} (the tie in the last row goes to the lower columns); column 0 then
    # keeps its two largest of 9, 7, 4, 9 -> rows 0 and 3 (the tie 9 = 9 is no issue: both are kept), column 1
    # of 8, 6, 3, 9 -> rows 3 and 0
    want = np.array([[1, 1, 0, 0], [0, 0, 0, 0], [0, 0, 0, 0], [1, 1, 0, 0]], dtype=np.uint8)
    assert np.array_equal(oracle.simple_round(key, 2, 4), want)
    rng = np.random.Generator(np.random.Philox(4321))
    key = rng.standard_normal((16, 24))
    got = oracle.simple_round(key, 3, 8)
    b = exact.blocks(got, 8)
    assert b.sum(axis=2).max() <= 3 and b.sum(axis=1).max() <= 3
    # every column that was offered at least N row-survivors is full
    kb = exact.blocks(key, 8)
    for blk, m in zip(kb, b):
        survivors = np.zeros_like(m)
        for i in range(8):
            survivors[i, np.argsort(-blk[i], kind="stable")[:3]] = 1
        assert np.array_equal(m.sum(axis=0), np.minimum(survivors.sum(axis=0), 3))
        assert np.all(m <= survivors)
    # a key whose N largest entries per row already form a transposable pattern is returned as that pattern
    perm = np.kron(np.eye(2), np.ones((2, 2)))
    assert np.array_equal(oracle.simple_round(perm + 0.01 * rng.random((4, 4)), 2, 4), perm.astype(np.uint8))


def test_early_exit_variant_of_algorithm1():
    # "maximum iterations" read as a bound.  Pins: tol = 0 is the fixed-T result bit for bit; the count is a
    # multiple of the check interval (or T); a looser tolerance never needs more iterations; the stopped state
    # equals the fixed-T state at that count; its marginals are within the tolerance; a uniform block is a
    # fixed point and stops at the first check.
    rng = np.random.Generator(np.random.Philox(9090))
    N, M, T = 4, 8, 400
    imp = np.abs(rng.standard_normal((2 * M, 3 * M))).astype(np.float32)
    te = oracle.tau_eff(imp, 0.02, oracle.TAU_REL_MATRIX_MAX)
    fixed = oracle.dykstra(imp, N, M, te, T)
    same, done0 = oracle.dykstra_adaptive(imp, N, M, te, T, 0.0)
    assert np.array_equal(same, fixed) and np.all(done0 == T)
    prev = None
    for tol in (1e-2, 1e-4, 1e-6):
        log_S, done = oracle.dykstra_adaptive(imp, N, M, te, T, tol)
        assert np.all((done % oracle.ADAPTIVE_CHECK_EVERY == 0) | (done == T))
        if prev is not None:
            assert np.all(done >= prev)
        prev = done
        for b, (blk, n) in enumerate(zip(exact.blocks(log_S, M), done)):
            r0, c0 = (b // 3) * M, (b % 3) * M
            ref = oracle.dykstra(imp[r0:r0 + M, c0:c0 + M], N, M, te, int(n))
            assert np.array_equal(blk, ref)
            if n < T:
                S = np.exp(blk)
                assert np.abs(S.sum(axis=0) - N).max() <= 2 * tol * N and np.abs(S.sum(axis=1) - N).max() <= 2 * tol * N
        assert (done < T).any()
    flat = np.full((M, M), 0.7, dtype=np.float32)
    _, done = oracle.dykstra_adaptive(flat, N, M, 1.0, 100, 1e-12)
    assert done[0] == oracle.ADAPTIVE_CHECK_EVERY
    _, done = oracle.dykstra_adaptive(flat, N, M, 1.0, 100, 1e-12, check_every=7)
    assert done[0] == 7
