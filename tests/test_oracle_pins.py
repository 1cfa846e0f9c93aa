"""Pins for the fp64 oracle: every check compares it with something other than itself
(hand-worked fixtures, closed forms, library routines, exhaustive search)."""
import json
import os

import numpy as np
import pytest

import csat_inputs as gen
from oracle import csat_oracle as orc
from tests.brute_force import l0_support_search, lasso_by_kkt_enumeration


def _load(golden_dir, name):
    with open(os.path.join(golden_dir, name)) as f:
        return json.load(f)


# ------------------------------------------------------------------ golden fixtures
def test_golden_ista_iterates(golden_dir):
    for case in _load(golden_dir, "ista_hand_worked.json")["cases"]:
        Phi = np.array(case["Phi"])
        y = np.array(case["y"])[None, :]
        _, trace, _ = orc.ista_trace(y, Phi, case["lambda"], case["mu"], len(case["iterates"]))
        for t, want in enumerate(case["iterates"]):
            np.testing.assert_allclose(trace[t][0], want, rtol=0, atol=1e-12, err_msg=case["name"])


def test_golden_measure_and_attention(golden_dir):
    g = _load(golden_dir, "attention_hand_worked.json")
    Kc, Vc = orc.measure(g["measure"]["Phi"], g["measure"]["K"], g["measure"]["K"])
    np.testing.assert_allclose(Kc, g["measure"]["Kc"], atol=1e-14)
    np.testing.assert_allclose(Vc, g["measure"]["Kc"], atol=1e-14)
    for key in ("compressed_attention", "scale"):
        c = g[key]
        A, Z = orc.compressed_attention(c["Q"], c["Kc"], c["Vc"])
        np.testing.assert_allclose(A, c["A"], atol=1e-14)
        np.testing.assert_allclose(Z, c["Z"], atol=1e-13)


# ------------------------------------------------------------------ exact attention vs a library routine
def test_attention_exact_matches_torch_sdpa():
    import torch
    rng = np.random.default_rng(0)
    Q, K, V = rng.standard_normal((3, 17, 8)), rng.standard_normal((3, 23, 8)), rng.standard_normal((3, 23, 8))
    want = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(Q), torch.from_numpy(K), torch.from_numpy(V)).numpy()
    np.testing.assert_allclose(orc.attention_exact(Q, K, V), want, rtol=1e-12, atol=1e-13)


def test_identity_phi_reduces_to_exact_attention():
    import torch
    rng = np.random.default_rng(1)
    n, d = 19, 8
    Q, K, V = (rng.standard_normal((2, n, d)) for _ in range(3))
    Phi = gen.make_phi("identity", n, n)
    Kc, Vc = orc.measure(Phi, K, V)
    np.testing.assert_array_equal(Kc, K)
    A, Z = orc.compressed_attention(Q, Kc, Vc)
    want = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(Q), torch.from_numpy(K), torch.from_numpy(V)).numpy()
    np.testing.assert_allclose(Z, want, rtol=1e-12, atol=1e-13)
    # whole block: Phi = I, lambda = 0, mu = 1: the first iterate is x = y = attention row, a fixed point
    for T in (1, 4):
        out = orc.forward(Q, K, V, Phi, lam=0.0, mu=1.0, iters=T)
        np.testing.assert_allclose(out["C"], want, rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(out["X"], out["A"], rtol=0, atol=1e-15)


# ------------------------------------------------------------------ measurement stage
def test_measure_against_explicit_loops_and_linearity():
    rng = np.random.default_rng(2)
    m, n, d = 5, 9, 3
    Phi, K, V = rng.standard_normal((m, n)), rng.standard_normal((n, d)), rng.standard_normal((n, d))
    Kc, Vc = orc.measure(Phi, K, V)
    for l in range(m):
        for c in range(d):
            assert Kc[l, c] == pytest.approx(sum(Phi[l, j] * K[j, c] for j in range(n)), abs=1e-13)
            assert Vc[l, c] == pytest.approx(sum(Phi[l, j] * V[j, c] for j in range(n)), abs=1e-13)
    K2 = rng.standard_normal((n, d))
    Kc2, _ = orc.measure(Phi, 2.0 * K - 3.0 * K2, V)
    Kc_b, _ = orc.measure(Phi, K2, V)
    np.testing.assert_allclose(Kc2, 2.0 * Kc - 3.0 * Kc_b, atol=1e-12)
    # batched form equals per-head form
    Kb = rng.standard_normal((4, n, d))
    Kcb, _ = orc.measure(Phi, Kb, Kb)
    for h in range(4):
        np.testing.assert_allclose(Kcb[h], orc.measure(Phi, Kb[h], Kb[h])[0], atol=1e-13)


def test_measurement_ensembles():
    m, n = 64, 4096
    G = gen.make_phi("gaussian", m, n, seed=0)
    assert abs(G.var() * m - 1.0) < 0.02 and abs(G.mean()) < 1e-3
    x = np.random.default_rng(3).standard_normal((n, 64))
    ratio = (np.linalg.norm(G @ x, axis=0) ** 2 / np.linalg.norm(x, axis=0) ** 2).mean()
    assert abs(ratio - 1.0) < 0.05                       # E||Phi x||^2 = ||x||^2
    R = gen.make_phi("rademacher", m, n, seed=0)
    np.testing.assert_allclose(np.abs(R), 1.0 / np.sqrt(m), rtol=1e-15)
    np.testing.assert_allclose(np.linalg.norm(R, axis=0), 1.0, rtol=1e-12)   # unit-norm columns
    assert abs(R.mean()) * np.sqrt(m) < 0.01
    # seeded: same seed same draw, other seed other draw
    np.testing.assert_array_equal(G, gen.make_phi("gaussian", m, n, seed=0))
    assert not np.array_equal(G, gen.make_phi("gaussian", m, n, seed=1))


def test_opnorm_against_svd():
    rng = np.random.default_rng(4)
    Phi = rng.standard_normal((7, 30))
    assert orc.phi_opnorm_sq(Phi) == pytest.approx(np.linalg.svd(Phi, compute_uv=False)[0] ** 2, rel=1e-12)
    Qm, _ = np.linalg.qr(rng.standard_normal((12, 12)))
    assert orc.phi_opnorm_sq(Qm) == pytest.approx(1.0, rel=1e-12)
    assert orc.phi_opnorm_sq(3.0 * Qm[:5]) == pytest.approx(9.0, rel=1e-12)


# ------------------------------------------------------------------ compressed attention
def test_compressed_attention_invariants_and_cost():
    from scipy.special import softmax
    rng = np.random.default_rng(5)
    n_q, n, d, m = 11, 40, 6, 7
    Q, K, V = rng.standard_normal((n_q, d)), rng.standard_normal((n, d)), rng.standard_normal((n, d))
    Phi = gen.make_phi("gaussian", m, n)
    Kc, Vc = orc.measure(Phi, K, V)
    A, Z = orc.compressed_attention(Q, Kc, Vc)
    assert A.shape == (n_q, m) and Z.shape == (n_q, d)
    assert (A >= 0).all()
    np.testing.assert_allclose(A.sum(-1), 1.0, rtol=1e-14)
    # explicit-loop scores: cost is exactly n_q * m * d multiply-accumulates, shape (n_q, m)
    S, macs = orc.compressed_scores_counted(Q, Kc)
    assert macs == n_q * m * d and S.shape == (n_q, m)
    np.testing.assert_allclose(A, softmax(S, axis=-1), rtol=1e-12)
    # shift invariance of the row softmax: adding a constant to the logits changes nothing
    np.testing.assert_allclose(softmax(S + 3.7, axis=-1), A, rtol=1e-12)
    # Q = 0: uniform weights, Z_i is the mean compressed value row
    A0, Z0 = orc.compressed_attention(np.zeros_like(Q), Kc, Vc)
    np.testing.assert_allclose(A0, 1.0 / m, rtol=1e-15)
    np.testing.assert_allclose(Z0, np.broadcast_to(Vc.mean(0), Z0.shape), rtol=1e-13)
    # permuting the measurements (rows of Phi) permutes A's columns and leaves Z unchanged
    p = rng.permutation(m)
    Kp, Vp = orc.measure(Phi[p], K, V)
    Ap, Zp = orc.compressed_attention(Q, Kp, Vp)
    np.testing.assert_allclose(Ap, A[:, p], rtol=1e-12)
    np.testing.assert_allclose(Zp, Z, rtol=1e-12, atol=1e-14)
    # the 1/sqrt(d_k) scale: doubling Q with 4x d (zero padded) leaves logits unchanged
    Qp = np.concatenate([2.0 * Q, np.zeros((n_q, 3 * d))], axis=1)
    Kcp = np.concatenate([Kc, np.ones((m, 3 * d))], axis=1)
    Ap2, _ = orc.compressed_attention(Qp, Kcp, np.concatenate([Vc, Vc, Vc, Vc], axis=1))
    np.testing.assert_allclose(Ap2, A, rtol=1e-12)


# ------------------------------------------------------------------ ISTA decoder
def test_soft_threshold_definition():
    u = np.array([-2.0, -0.5, -0.1, 0.0, 0.1, 0.5, 2.0])
    np.testing.assert_allclose(orc.soft_threshold(u, 0.5), [-1.5, 0, 0, 0, 0, 0, 1.5], atol=0)
    # a tie |u| == theta maps to zero and is not in the support
    assert not orc.support(orc.soft_threshold(np.array([0.5, -0.5]), 0.5)).any()


def _basis_pursuit(Phi, y):
    """min ||x||_1 s.t. Phi x = y as a linear programme (x = p - q, p, q >= 0), solved by scipy."""
    from scipy.optimize import linprog
    m, n = Phi.shape
    res = linprog(np.ones(2 * n), A_eq=np.hstack([Phi, -Phi]), b_eq=y, bounds=(0, None), method="highs")
    assert res.status == 0
    return res.x[:n] - res.x[n:]


@pytest.mark.parametrize("seed", range(6))
def test_planted_sparse_support_matches_exhaustive_search(seed):
    m, n, k = 14, 20, 2
    Phi, Xs, sups = gen.planted_sparse(seed, m, n, k, rows=3)
    Y = Xs @ Phi.T
    mu = 1.0 / orc.phi_opnorm_sq(Phi)
    X = orc.ista(Y, Phi, lam=1e-3, mu=mu, iters=20000)
    checked = 0
    for r in range(3):
        brute, res = l0_support_search(Phi, Y[r], k)
        assert res < 1e-10
        np.testing.assert_array_equal(brute, sups[r])                 # the search finds the planted set
        # exact l1 recovery holds only when this draw of Phi is good enough for this support:
        # the paper's basis-pursuit programme, solved exactly, says whether it is
        bp = _basis_pursuit(Phi, Y[r])
        if np.abs(bp - Xs[r]).max() > 1e-7:
            continue
        # ... and the l1-penalised form keeps the support for every lambda > 0 when the
        # textbook irrepresentable condition max_j |Phi_j^T Phi_S (Phi_S^T Phi_S)^-1 sign(x_S)| < 1 holds
        S = sups[r]
        cert = Phi.T @ (Phi[:, S] @ np.linalg.solve(Phi[:, S].T @ Phi[:, S], np.sign(Xs[r, S])))
        if np.abs(np.delete(cert, S)).max() > 0.95:
            continue
        checked += 1
        np.testing.assert_array_equal(np.flatnonzero(orc.support(X[r])), brute)
        np.testing.assert_allclose(X[r], bp, atol=5e-3)               # lambda-sized shrinkage bias only
    assert checked >= 1


@pytest.mark.parametrize("seed", range(5))
def test_ista_converges_to_exhaustive_kkt_solution(seed):
    rng = np.random.default_rng(100 + seed)
    m, n, lam = 5, 8, 0.15
    Phi = rng.standard_normal((m, n)) / np.sqrt(m)
    y = rng.standard_normal(m)
    want = lasso_by_kkt_enumeration(Phi, y, lam)
    assert want is not None
    mu = 1.0 / orc.phi_opnorm_sq(Phi)
    X = orc.ista(y[None], Phi, lam, mu, iters=30000)
    np.testing.assert_allclose(X[0], want, atol=1e-9)
    np.testing.assert_array_equal(orc.support(X[0]), want != 0)


def test_ista_matches_sklearn_lasso():
    from sklearn.linear_model import Lasso
    rng = np.random.default_rng(7)
    m, n, lam = 30, 80, 0.05
    Phi = rng.standard_normal((m, n)) / np.sqrt(m)
    y = Phi[:, [3, 17, 40]] @ np.array([1.0, -0.7, 0.4]) + 0.01 * rng.standard_normal(m)
    # scikit-learn minimises 1/(2 m) ||y - Phi w||^2 + alpha ||w||_1  ->  alpha = lam / m
    sk = Lasso(alpha=lam / m, fit_intercept=False, tol=1e-14, max_iter=200000).fit(Phi, y).coef_
    mu = 1.0 / orc.phi_opnorm_sq(Phi)
    X = orc.ista(y[None], Phi, lam, mu, iters=50000)
    np.testing.assert_allclose(X[0], sk, atol=1e-8)


def test_ista_objective_monotone_and_zero_solution():
    rng = np.random.default_rng(8)
    m, n, lam = 16, 48, 0.1
    Phi = rng.standard_normal((m, n)) / np.sqrt(m)
    Y = rng.standard_normal((4, m))
    mu = 1.0 / orc.phi_opnorm_sq(Phi)
    _, trace, _ = orc.ista_trace(Y, Phi, lam, mu, 60)
    obj = np.stack([orc.lasso_objective(Y, Phi, X, lam) for X in trace])
    assert (np.diff(obj, axis=0) <= 1e-13).all()
    assert (obj[0] <= orc.lasso_objective(Y, Phi, np.zeros((4, n)), lam) + 1e-13).all()
    # lambda >= ||Phi^T y||_inf: zero is optimal and every iterate stays zero
    big = np.abs(Y @ Phi).max() * 1.0001
    _, trace0, _ = orc.ista_trace(Y, Phi, big, mu, 5)
    assert all((X == 0).all() for X in trace0)


def test_ista_orthogonal_phi_closed_form():
    rng = np.random.default_rng(9)
    n, lam = 10, 0.3
    Qm, _ = np.linalg.qr(rng.standard_normal((n, n)))
    Y = rng.standard_normal((3, n))
    want = orc.soft_threshold(Y @ Qm, lam)           # x = S_lambda(Phi^T y), mu = 1
    for T in (1, 2, 7):
        np.testing.assert_allclose(orc.ista(Y, Qm, lam, 1.0, T), want, atol=1e-13)
    np.testing.assert_allclose(orc.ista(Y, np.eye(n), lam, 1.0, 3), orc.soft_threshold(Y, lam), atol=0)


def test_ista_equals_lista_form_and_is_permutation_equivariant():
    rng = np.random.default_rng(10)
    m, n, lam = 12, 30, 0.05
    Phi = rng.standard_normal((m, n)) / np.sqrt(m)
    Y = rng.standard_normal((5, m))
    mu = 0.9 / orc.phi_opnorm_sq(Phi)
    X = orc.ista(Y, Phi, lam, mu, 25)
    np.testing.assert_allclose(orc.lista_form(Y, Phi, lam, mu, 25), X, atol=1e-12)
    p = rng.permutation(n)
    np.testing.assert_allclose(orc.ista(Y, Phi[:, p], lam, mu, 25), X[:, p], atol=1e-13)
    # rows are independent problems
    np.testing.assert_allclose(orc.ista(Y[2:3], Phi, lam, mu, 25), X[2:3], atol=1e-14)


# ------------------------------------------------------------------ whole block
def test_forward_identities():
    rng = np.random.default_rng(11)
    BH, n_q, n, d, m = 2, 9, 24, 4, 8
    Q, K, V = rng.standard_normal((BH, n_q, d)), rng.standard_normal((BH, n, d)), rng.standard_normal((BH, n, d))
    Phi = gen.make_phi("gaussian", m, n)
    mu = 1.0 / orc.phi_opnorm_sq(Phi)
    # lambda = 0, one iteration: x = mu Phi^T y, so C^ = mu (Phi V)^T y = mu Z
    o1 = orc.forward(Q, K, V, Phi, lam=0.0, mu=mu, iters=1)
    np.testing.assert_allclose(o1["C"], mu * o1["Z"], rtol=1e-12, atol=1e-14)
    # no decoder iterations: the block returns the compressed output
    o0 = orc.forward(Q, K, V, Phi, lam=0.1, mu=mu, iters=0)
    np.testing.assert_array_equal(o0["C"], o0["Z"])
    # explicit per-row synthesis: C^_i = sum_j x_ij V_j
    o = orc.forward(Q, K, V, Phi, lam=0.05, mu=mu, iters=6)
    for h in range(BH):
        for i in range(n_q):
            want = sum(o["X"][h, i, j] * V[h, j] for j in range(n))
            np.testing.assert_allclose(o["C"][h, i], want, atol=1e-13)
    # permuting keys/values together with Phi's columns changes nothing downstream
    p = rng.permutation(n)
    op = orc.forward(Q, K[:, p], V[:, p], Phi[:, p], lam=0.05, mu=mu, iters=6)
    np.testing.assert_allclose(op["C"], o["C"], rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(op["X"], o["X"][:, :, p], atol=1e-13)
    # row sampling computes the same rows
    rows = np.array([7, 1, 4])
    os_ = orc.forward(Q, K, V, Phi, lam=0.05, mu=mu, iters=6, rows=rows)
    np.testing.assert_allclose(os_["X"], o["X"][:, rows], atol=1e-15)
    np.testing.assert_allclose(os_["C"], o["C"][:, rows], atol=1e-15)


def test_separate_key_and_value_matrices():
    """K~ = Phi_K K, V~ = Phi_V V with two different matrices (section 3); the decoder uses Phi_V."""
    import torch
    rng = np.random.default_rng(12)
    BH, n, d, m = 2, 12, 4, 12
    Q, K, V = rng.standard_normal((BH, n, d)), rng.standard_normal((BH, n, d)), rng.standard_normal((BH, n, d))
    PhiV = gen.make_phi("gaussian", m, n, seed=1)
    PhiK = gen.make_phi("rademacher", m, n, seed=2)
    mu = 1.0 / orc.phi_opnorm_sq(PhiV)
    # the same matrix twice is the shared case
    a, b = orc.forward(Q, K, V, PhiV, 0.05, mu, 4), orc.forward(Q, K, V, PhiV, 0.05, mu, 4, Phi_K=PhiV)
    for k in ("Kc", "Vc", "A", "Z", "X", "C"):
        np.testing.assert_array_equal(a[k], b[k])
    # each matrix lands on its own operand (explicit sums)
    o = orc.forward(Q, K, V, PhiV, 0.05, mu, 4, Phi_K=PhiK)
    for l in range(m):
        np.testing.assert_allclose(o["Kc"][1, l], sum(PhiK[l, j] * K[1, j] for j in range(n)), atol=1e-13)
        np.testing.assert_allclose(o["Vc"][1, l], sum(PhiV[l, j] * V[1, j] for j in range(n)), atol=1e-13)
    # Phi_K = I: the scores are the exact ones, so Z is exact attention over the measured values Phi_V V
    oi = orc.forward(Q, K, V, PhiV, 0.05, mu, 0, Phi_K=np.eye(n))
    t = lambda x: torch.from_numpy(np.ascontiguousarray(x))
    want = torch.nn.functional.scaled_dot_product_attention(t(Q), t(K), t(PhiV @ V)).numpy()
    np.testing.assert_allclose(oi["Z"], want, rtol=1e-11, atol=1e-13)
    # Phi_V = I with another Phi_K: V~ = V, and the decoder (Phi = I, lambda = 0) returns A~ itself, C^ = A~ V = Z
    ov = orc.forward(Q, K, V, np.eye(n), 0.0, 1.0, 3, Phi_K=PhiK)
    np.testing.assert_allclose(ov["X"], ov["A"], atol=1e-14)
    np.testing.assert_allclose(ov["C"], ov["Z"], atol=1e-13)
    # lambda = 0, one iteration: C^ = mu Z whatever Phi_K is (the decoder's matrix is Phi_V)
    o1 = orc.forward(Q, K, V, PhiV, 0.0, mu, 1, Phi_K=PhiK)
    np.testing.assert_allclose(o1["C"], mu * o1["Z"], rtol=1e-12, atol=1e-14)
    # column-wise reading: Y is formed with Phi_V and decoded through it; Phi_V = I, lambda = 0 returns Z
    r = orc.forward_rd(Q, K, V, PhiV, 0.05, mu, 3, Phi_K=PhiK)
    np.testing.assert_allclose(r["Y"], PhiV @ r["Z"], atol=1e-13)
    np.testing.assert_array_equal(r["Kc"], o["Kc"])
    ri = orc.forward_rd(Q, K, V, np.eye(n), 0.0, 1.0, 2, Phi_K=PhiK)
    np.testing.assert_allclose(ri["C"], ri["Z"], atol=1e-13)


def test_lista_with_given_weights(golden_dir):
    """lista(): hand-worked layers, the analytic weights (= ISTA), closed forms."""
    g = json.load(open(os.path.join(golden_dir, "lista_hand_worked.json")))
    for L in (1, 2):
        X, _ = orc.lista(np.array(g["y"]), np.array(g["S"]), np.array(g["B"]), g["thetas"][:L])
        np.testing.assert_allclose(X[0], g["x_after_layer"][L - 1], rtol=0, atol=1e-15)
    rng = np.random.default_rng(5)
    m, n, rows = 9, 21, 4
    Phi = gen.make_phi("gaussian", m, n)
    Y = rng.standard_normal((rows, m))
    mu, lam = 1.0 / orc.phi_opnorm_sq(Phi), 0.07
    # analytic weights reproduce the ISTA iterates
    S, Bm = np.eye(n) - mu * Phi.T @ Phi, mu * Phi.T
    for T in (1, 2, 9):
        X, U = orc.lista(Y, S, Bm, [mu * lam] * T)
        Xi, _, Ui = orc.ista_trace(Y, Phi, lam, mu, T)
        np.testing.assert_allclose(X, Xi, rtol=0, atol=1e-13)
        np.testing.assert_allclose(U, Ui, rtol=0, atol=1e-13)
    # S = 0: every layer forgets the previous one, the result is the shrinkage of B y by the last threshold
    Bm = rng.standard_normal((n, m))
    X, _ = orc.lista(Y, np.zeros((n, n)), Bm, [0.9, 0.1, 0.4])
    v = np.einsum("jl,rl->rj", Bm, Y)
    np.testing.assert_allclose(X, np.where(np.abs(v) > 0.4, v - 0.4 * np.sign(v), 0.0), rtol=0, atol=1e-14)
    # diagonal S, B = first m columns of the identity, thresholds 0: scalar geometric recursions
    sdiag = rng.uniform(-0.9, 0.9, n)
    Bm = np.eye(n, m)
    X, _ = orc.lista(Y, np.diag(sdiag), Bm, [0.0] * 6)
    geo = sum(sdiag ** k for k in range(6))
    np.testing.assert_allclose(X[:, :m], Y * geo[:m], rtol=1e-13, atol=1e-14)
    assert not X[:, m:].any()
    # thresholds are per layer: order matters
    Bm = rng.standard_normal((n, m))
    Xa, _ = orc.lista(Y, S, Bm, [0.5, 0.05])
    Xb, _ = orc.lista(Y, S, Bm, [0.05, 0.5])
    assert np.abs(Xa - Xb).max() > 1e-3


def test_omp_pins():
    """omp(): library routine, exhaustive search on planted problems, closed forms, invariants."""
    from sklearn.linear_model import orthogonal_mp
    rng = np.random.default_rng(31)
    m, n, k = 12, 30, 3
    Phi = gen.make_phi("gaussian", m, n)
    Y = rng.standard_normal((6, m))
    X, picks, margins = orc.omp(Y, Phi, k)
    # scikit-learn's implementation of the same algorithm (Cholesky-based), column by column
    for i in range(Y.shape[0]):
        ref = orthogonal_mp(Phi, Y[i], n_nonzero_coefs=k, precompute=False)
        np.testing.assert_allclose(X[i], ref, rtol=1e-9, atol=1e-11)
        assert sorted(picks[i]) == sorted(np.flatnonzero(ref))
        # the residual is orthogonal to every picked column, and exactly k coordinates are set
        r = Y[i] - Phi @ X[i]
        assert np.abs(Phi[:, picks[i]].T @ r).max() < 1e-12
        assert np.count_nonzero(X[i]) == k and len(set(picks[i])) == k
    assert (margins >= 0).all() and (margins <= 1).all()
    # planted k-sparse, noiseless: the picked support is the exhaustive l0 search's and the fit is exact
    hits = 0
    for seed in range(6):
        r2 = np.random.default_rng(100 + seed)
        Phi2 = r2.standard_normal((10, 16)) / np.sqrt(10)
        sup = np.sort(r2.choice(16, size=2, replace=False))
        y = Phi2[:, sup] @ (np.array([1.5, -1.0]) * r2.choice([-1, 1], size=2))
        Xp, pk, _ = orc.omp(y[None], Phi2, 2)
        best, res = l0_support_search(Phi2, y, 2)
        assert res < 1e-12 and list(best) == list(sup)
        if sorted(pk[0]) == list(sup):              # greedy recovery holds for most, not all, draws
            hits += 1
            np.testing.assert_allclose(Phi2 @ Xp[0], y, atol=1e-12)
    assert hits >= 4
    # one pick: closed form
    X1, p1, _ = orc.omp(Y, Phi, 1)
    for i in range(Y.shape[0]):
        c = Phi.T @ Y[i]
        j = int(np.argmax(np.abs(c)))
        assert p1[i, 0] == j
        np.testing.assert_allclose(X1[i, j], c[j] / (Phi[:, j] @ Phi[:, j]), rtol=1e-13)
    # orthonormal columns: the k largest |Phi^T y| in decreasing order, coefficients are those correlations
    Po = np.linalg.qr(rng.standard_normal((m, m)))[0]                # m x m orthogonal: columns orthonormal
    Xo, po, _ = orc.omp(Y, Po, 4)
    for i in range(Y.shape[0]):
        c = Po.T @ Y[i]
        order = np.argsort(-np.abs(c))[:4]
        assert list(po[i]) == list(order)
        np.testing.assert_allclose(Xo[i, order], c[order], rtol=1e-12, atol=1e-14)
    # ties go to the lowest index: two identical columns
    Pt = Phi.copy()
    Pt[:, 7] = Pt[:, 3]
    _, pt, mt = orc.omp((2.0 * Pt[:, 3])[None], Pt, 1)
    assert pt[0, 0] == 3 and mt[0, 0] == 0.0


def test_omp_margins_against_an_independent_path():
    """omp()'s `margins` (how far the chosen correlation was ahead of the runner-up) decide which GPU rows are
    compared strictly, so they are pinned on their own: the support after t picks comes from scikit-learn's
    orthogonal_mp with t non-zeros, the residual from its coefficients, and the correlations of the unpicked
    columns from explicit loops; the margin is then (largest - second largest) / largest."""
    from sklearn.linear_model import orthogonal_mp
    rng = np.random.default_rng(57)
    m, n, k = 14, 26, 4
    Phi = rng.standard_normal((m, n)) / np.sqrt(m)
    Y = rng.standard_normal((5, m))
    _, picks, margins = orc.omp(Y, Phi, k)
    for i in range(Y.shape[0]):
        for t in range(k):
            if t == 0:
                picked, r = [], Y[i].copy()
            else:
                coef = orthogonal_mp(Phi, Y[i], n_nonzero_coefs=t, precompute=False)
                picked = list(np.flatnonzero(coef))
                r = Y[i] - Phi @ coef
            assert sorted(picked) == sorted(picks[i, :t])
            corr = []
            for j in range(n):
                if j in picked:
                    continue
                acc = 0.0
                for l in range(m):
                    acc += Phi[l, j] * r[l]
                corr.append((abs(acc), j))
            corr.sort(reverse=True)
            assert corr[0][1] == picks[i, t]
            want = (corr[0][0] - corr[1][0]) / corr[0][0]
            assert margins[i, t] == pytest.approx(want, rel=1e-9, abs=1e-12)
    # a planted mistake would show: the margin of the first pick is not that of the last
    assert np.abs(margins[:, 0] - margins[:, -1]).max() > 1e-3


def test_lasso_objective_against_explicit_sums_and_known_values():
    """lasso_objective(): explicit loops on a random case, the hand value of a 2 x 2 case, and the minimum
    property at scikit-learn's solution (no perturbation lowers it)."""
    from sklearn.linear_model import Lasso
    rng = np.random.default_rng(5)
    m, n, lam = 7, 11, 0.3
    Phi = rng.standard_normal((m, n))
    Y = rng.standard_normal((3, m))
    X = rng.standard_normal((3, n)) * (rng.random((3, n)) < 0.4)
    got = orc.lasso_objective(Y, Phi, X, lam)
    for i in range(3):
        sq, l1 = 0.0, 0.0
        for l in range(m):
            pred = 0.0
            for j in range(n):
                pred += Phi[l, j] * X[i, j]
            sq += (Y[i, l] - pred) ** 2
        for j in range(n):
            l1 += abs(X[i, j])
        assert got[i] == pytest.approx(0.5 * sq + lam * l1, rel=1e-12)
    # y = (3, 1), Phi = [[1, 2], [0, 1]], x = (1, -1): Phi x = (-1, -1), residual (4, 2): 1/2 * 20 + 0.5 * 2 = 11
    val = orc.lasso_objective(np.array([[3.0, 1.0]]), np.array([[1.0, 2.0], [0.0, 1.0]]), np.array([[1.0, -1.0]]), 0.5)
    assert val[0] == pytest.approx(11.0, rel=1e-14)
    sk = Lasso(alpha=lam / m, fit_intercept=False, tol=1e-14, max_iter=200000).fit(Phi, Y[0]).coef_
    best = orc.lasso_objective(Y[:1], Phi, sk[None], lam)[0]
    for _ in range(50):
        pert = sk + 1e-3 * rng.standard_normal(n)
        assert orc.lasso_objective(Y[:1], Phi, pert[None], lam)[0] >= best - 1e-12


def test_column_wise_reading_pins():
    """forward_rd: closed forms and library routines that fix the column-wise reading."""
    import torch
    from sklearn.linear_model import Lasso
    rng = np.random.default_rng(21)
    BH, n, d = 2, 18, 5
    Q, K, V = (rng.standard_normal((BH, n, d)) for _ in range(3))
    attn = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(Q), torch.from_numpy(K), torch.from_numpy(V)).numpy()
    # Phi = I, mu = 1: Y = Z = exact attention, and one step lands on the fixed point, the
    # element-wise shrinkage of the exact attention output
    lam = 0.07
    want = np.where(np.abs(attn) > lam, attn - lam * np.sign(attn), 0.0)
    for T in (1, 3):
        o = orc.forward_rd(Q, K, V, gen.make_phi("identity", n, n), lam=lam, mu=1.0, iters=T)
        np.testing.assert_allclose(o["Y"], attn, rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(o["C"], want, rtol=1e-12, atol=1e-13)
    # orthonormal rows (Phi Phi^T = I), lambda = 0, mu = 1: the first iterate is the minimum-norm
    # solution of Phi x = y and a fixed point
    m = 7
    Phi = np.linalg.qr(rng.standard_normal((n, m)))[0].T
    for T in (1, 4):
        o = orc.forward_rd(Q, K, V, Phi, lam=0.0, mu=1.0, iters=T)
        for h in range(BH):
            np.testing.assert_allclose(o["C"][h], np.linalg.pinv(Phi) @ o["Y"][h], rtol=1e-10, atol=1e-12)
    # Y is the measurement of Z, element by element
    Phi = gen.make_phi("gaussian", m, n)
    mu = 1.0 / orc.phi_opnorm_sq(Phi)
    o = orc.forward_rd(Q, K, V, Phi, lam=0.02, mu=mu, iters=400)
    for h in range(BH):
        for l in range(m):
            for k in range(d):
                assert abs(o["Y"][h, l, k] - sum(Phi[l, j] * o["Z"][h, j, k] for j in range(n))) < 1e-12
    # every decoded column converges to scikit-learn's Lasso solution for that column
    # (its objective is 1/(2m) ||y - Phi x||^2 + alpha ||x||_1, so alpha = lambda / m)
    Phi12 = gen.make_phi("gaussian", 12, n)
    o = orc.forward_rd(Q, K, V, Phi12, lam=0.3, mu=1.0 / orc.phi_opnorm_sq(Phi12), iters=50000)
    for h in range(BH):
        for k in range(d):
            ref = Lasso(alpha=0.3 / 12, fit_intercept=False, tol=1e-14, max_iter=200000).fit(Phi12, o["Y"][h, :, k]).coef_
            np.testing.assert_allclose(o["C"][h, :, k], ref, atol=1e-7)
            assert np.count_nonzero(ref) > 0
    # no iterations: C = Z; a column subset decodes the same columns; permuting the feature
    # columns of V permutes the output columns
    o6 = orc.forward_rd(Q, K, V, Phi, lam=0.02, mu=mu, iters=6)
    np.testing.assert_array_equal(orc.forward_rd(Q, K, V, Phi, 0.02, mu, 0)["C"], o6["Z"])
    cols = np.array([3, 0])
    np.testing.assert_allclose(orc.forward_rd(Q, K, V, Phi, 0.02, mu, 6, cols=cols)["C"], o6["C"][:, :, cols], atol=1e-15)
    p = rng.permutation(d)
    np.testing.assert_allclose(orc.forward_rd(Q, K, V[:, :, p], Phi, 0.02, mu, 6)["C"], o6["C"][:, :, p], atol=1e-13)
    with pytest.raises(ValueError):
        orc.forward_rd(Q[:, :5], K, V, Phi, 0.02, mu, 1)


# ------------------------------------------------------------------ the input generators
def test_bf16_rounding_matches_torch():
    import torch
    x = np.random.default_rng(12).standard_normal(10000).astype(np.float32) * 3
    x[:4] = [1.00390625, 1.01171875, -1.00390625, 0.0]          # exact ties: round to even
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    np.testing.assert_array_equal(gen.round_to_bf16(x), want)
    back = torch.from_numpy(gen.bf16_bits(want)).view(torch.bfloat16).to(torch.float32).numpy()
    np.testing.assert_array_equal(back, want)


def test_hadamard_ensemble_generator():
    """The structured ensemble against scipy's Hadamard matrix, and its frame property."""
    from scipy.linalg import hadamard
    m, n = 24, 50
    Phi, rows, signs = gen.make_hadamard_phi(m, n, seed=3)
    N = 64
    assert Phi.shape == (m, n) and len(signs) == N and len(rows) == m and len(set(rows.tolist())) == m
    assert (np.diff(rows) > 0).all() and set(np.unique(signs).tolist()) <= {-1, 1}
    H = hadamard(N).astype(np.float64)
    np.testing.assert_array_equal(Phi * np.sqrt(m), (H[rows] * signs[None, :])[:, :n])
    # with all N columns the rows are orthogonal with squared norm N/m: ||Phi||_2^2 = N/m exactly
    PhiN, _, _ = gen.make_hadamard_phi(m, N, seed=3)
    np.testing.assert_allclose(PhiN @ PhiN.T, (N / m) * np.eye(m), atol=1e-12)
    assert orc.phi_opnorm_sq(PhiN) == pytest.approx(N / m, rel=1e-12)
    assert orc.phi_opnorm_sq(Phi) <= N / m + 1e-9       # dropping columns cannot raise the norm


def test_workload_generators_shapes_and_structure():
    for name, w in gen.WORKLOADS.items():
        if name in ("cross_modal", "long_video"):
            w = gen.scaled(w, B=1, H=2)
        if name == "long_video":
            w = gen.scaled(w, n=2048 + 0, n_q=2048, frames=8)
        Q, K, V = gen.make_qkv(w)
        assert Q.shape == (w.B * w.H, w.n_q, w.d) and K.shape == V.shape == (w.B * w.H, w.n, w.d)
        if w.dtype == "bf16":
            np.testing.assert_array_equal(gen.round_to_bf16(K), K)
        if "frame_drift" in w.structure:
            P = w.patches
            diff = K[:, :P] - K[:, P:2 * P]                     # two frames differ by drift only
            assert 0.04 < diff.std() / np.sqrt(2) < 0.06
        if w.structure == "lowrank_image_text":
            s = np.linalg.svd(K[0, :w.patches].astype(np.float64), compute_uv=False)
            assert s[15] > 3 * s[16]                            # rank 16 plus small noise
        Phi = gen.make_workload_phi(w)
        assert Phi.shape == (w.m, w.n)
    # a head slice returns the same values as the full draw
    w = gen.WORKLOADS["image_text"]
    Qf, _, _ = gen.make_qkv(w)
    Qs, _, _ = gen.make_qkv(w, heads=slice(5, 7))
    np.testing.assert_array_equal(Qs, Qf[5:7])


def test_phi_fill_generator_pins():
    """The oracle's counter-based draw of Phi (section 3 names the Gaussian and Rademacher ensembles; the generator
    and the 1/sqrt(m) scaling are this build's choice).  Its words are SplitMix64's published outputs for the
    seeds 0 and 1234567; an element is the Box-Muller value of its two words, worked here with Python integers
    and the math module; any element can be drawn on its own; the ensembles have the moments they should."""
    import math
    assert [int(x) for x in orc.splitmix64_words(0, 0, 3)] == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]
    assert [int(x) for x in orc.splitmix64_words(1234567, 0, 3)] == [6457827717110365317, 3203168211198807973,
                                                                   9817491932198370423]
    # random access: words 1000 .. 1004 are the tail of words 0 .. 1004
    np.testing.assert_array_equal(orc.splitmix64_words(99, 1000, 5), orc.splitmix64_words(99, 0, 1005)[1000:])
    m, n = 5, 7
    P = orc.phi_fill("gaussian", 0, m, n)
    assert P.dtype == np.float32 and P.shape == (m, n)
    w1, w2 = 0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4                     # element (0, 0) of seed 0
    g00 = math.sqrt(-2.0 * math.log(((w1 >> 11) + 1) / 2.0 ** 53)) * math.cos(2.0 * math.pi * (w2 >> 11) / 2.0 ** 53)
    assert P[0, 0] == np.float32(g00 / math.sqrt(m))
    # element (r, c) comes from words 2 i and 2 i + 1 with i = r n + c, whatever the matrix around it
    i = 3 * n + 4
    wa, wb = (int(x) for x in orc.splitmix64_words(0, 2 * i, 2))
    g = math.sqrt(-2.0 * math.log(((wa >> 11) + 1) / 2.0 ** 53)) * math.cos(2.0 * math.pi * (wb >> 11) / 2.0 ** 53)
    assert abs(float(P[3, 4]) - g / math.sqrt(m)) <= 1e-7 * abs(g)
    R = orc.phi_fill("rademacher", 0, m, n)
    assert R[0, 0] == np.float32(-1.0 / math.sqrt(m))                   # top bit of 0xE220... is set
    np.testing.assert_array_equal(np.abs(R), np.full((m, n), np.float32(1.0 / math.sqrt(m))))
    # moments over 2^18 entries: mean 0 +- 4 sigma, variance 1/m, sign balance, no correlation between neighbours
    m, n = 64, 4096
    G = orc.phi_fill("gaussian", 11, m, n).astype(np.float64) * math.sqrt(m)
    N = G.size
    assert abs(G.mean()) < 4 / math.sqrt(N) and abs(G.var() - 1.0) < 4 * math.sqrt(2.0 / N)
    assert abs(np.mean(G ** 4) - 3.0) < 0.1                             # Gaussian kurtosis
    assert abs(np.mean(G[:, 1:] * G[:, :-1])) < 4 / math.sqrt(N)
    S = orc.phi_fill("rademacher", 11, m, n) * math.sqrt(m)
    assert abs(S.mean()) < 4 / math.sqrt(N) and abs(np.mean(S[:, 1:] * S[:, :-1])) < 4 / math.sqrt(N)
    assert not np.array_equal(orc.phi_fill("gaussian", 11, m, n), orc.phi_fill("gaussian", 12, m, n))
    # E[Phi Phi^T] = (n / m) I: off-diagonal entries of the Gram matrix are O(sqrt(n) / m)
    gram = (G / math.sqrt(m)) @ (G / math.sqrt(m)).T
    assert np.allclose(np.diag(gram), n / m, rtol=0.15) and np.abs(gram - np.diag(np.diag(gram))).max() < 6 * math.sqrt(n) / m
