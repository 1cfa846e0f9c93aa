"""Parity of the HIP path (through the C ABI) with the fp64 oracle on the same seeded inputs."""
import numpy as np
import pytest
import torch

import csat_inputs as gen
import paper_2507_02957_amd as csat
from oracle import csat_oracle as orc
from tests.gpu_harness import DEV, TOL, DeviceProblem, assert_close, assert_close_iterate, to_dev, to_np

pytestmark = pytest.mark.gpu


@pytest.fixture
def options():
    """Kernel-selection overrides through the context (csat_set_option), restored to the library's own choices
    when the test ends."""
    touched = []

    def set_option(key, value):
        csat.csat_set_option(key, value)
        touched.append(key)

    yield set_option
    for key in touched:
        csat.csat_set_option(key, 0)


def _mu(Phi):
    """Step size 1/||Phi||^2 computed once in fp64 and handed as the same float to both sides."""
    return float(np.float32(1.0 / orc.phi_opnorm_sq(Phi)))


def _support_check(name, Xg, ref, theta, band_rel=1e-5):
    """Supports must agree bit for bit except where the oracle's last pre-threshold value sits
    within band_rel*theta of the threshold (a tie that rounding may break either way)."""
    sg, so = Xg != 0, ref["X"] != 0
    ambiguous = np.abs(np.abs(ref["U"]) - theta) <= band_rel * theta
    diff = (sg != so) & ~ambiguous
    assert not diff.any(), f"{name}: {diff.sum()} support mismatches outside the tie band"
    return int(((sg != so) & ambiguous).sum()), int(ambiguous.sum())


def _small(name, **kw):
    base = dict(name=name, B=1, H=1, n_q=64, n=64, d=64, m=32, dtype="f32", phi_kind="gaussian", iters=5,
                lam=0.05, structure="iid", seed=11)
    base.update(kw)
    return gen.Workload(**base)


SMALL = [
    gen.WORKLOADS["tiny"],
    # several row/column tiles with ragged tails in every dimension; n, m not multiples of 8
    _small("ragged_f32", B=2, H=3, n_q=150, n=203, d=64, m=75, dtype="f32", iters=7),
    _small("ragged_bf16", B=2, H=3, n_q=150, n=203, d=64, m=75, dtype="bf16", iters=7),
    _small("cross_f32", B=1, H=2, n_q=77, n=300, d=128, m=136, dtype="f32", phi_kind="rademacher", iters=6,
           lam=0.02),
    _small("cross_bf16", B=1, H=2, n_q=77, n=300, d=128, m=136, dtype="bf16", phi_kind="rademacher", iters=6,
           lam=0.02),
    _small("one_row", n_q=1, n=40, d=8, m=8, dtype="f32", iters=3),
    _small("one_row_bf16", n_q=1, n=40, d=8, m=8, dtype="bf16", iters=3),
    # bf16, m > 416: the decoder runs as one large-tile GEMM pair per iteration (ragged 256-tiles in
    # rows and columns, sparse state, X requested); m % 4 != 0 takes the element-wise residual epilogue
    # in csat_recover, where Y is the caller's [rows, m] buffer
    _small("wide_m_bf16", B=1, H=2, n_q=300, n=520, d=64, m=452, dtype="bf16", iters=5, lam=0.008),
    _small("wide_m_odd_bf16", B=1, H=3, n_q=171, n=470, d=64, m=450, dtype="bf16", iters=4, lam=0.008),
    # fused decoder: a single and two iterations (first / last iteration special cases), the largest
    # m it takes (13 tiles), and the fewest chunks it takes (n = 65 -> 3)
    _small("fused_t1", B=2, H=3, n_q=150, n=203, d=64, m=75, dtype="bf16", iters=1),
    _small("fused_t2", B=2, H=3, n_q=150, n=203, d=64, m=75, dtype="bf16", iters=2),
    _small("fused_mt13", B=1, H=2, n_q=130, n=430, d=64, m=409, dtype="bf16", iters=4, lam=0.008),
    _small("fused_3chunks", B=1, H=2, n_q=40, n=65, d=64, m=33, dtype="bf16", iters=4),
    _small("generic_2chunks_bf16", B=1, H=2, n_q=40, n=64, d=64, m=33, dtype="bf16", iters=4),
    # softmax rows of 513..1024 scores (16 per lane in registers) and beyond 1024 (three passes over the row)
    _small("rows_600_bf16", B=1, H=2, n_q=70, n=700, d=64, m=600, dtype="bf16", iters=3, lam=0.004),
    _small("rows_1100_f32", B=1, H=1, n_q=40, n=1200, d=64, m=1100, dtype="f32", iters=2, lam=0.004),
    # the same beyond 1024 in bf16, on the large-tile GEMM pair (5 x 5 column tiles of the two products, split K)
    _small("rows_1100_bf16", B=1, H=2, n_q=150, n=1300, d=64, m=1100, dtype="bf16", iters=3, lam=0.004),
]


@pytest.mark.parametrize("w", SMALL, ids=lambda w: w.name)
def test_stagewise_and_forward_small(w):
    Q, K, V = gen.make_qkv(w)
    Phi = gen.make_workload_phi(w)
    mu = _mu(Phi)
    ref = orc.forward(Q, K, V, Phi, w.lam, mu, w.iters)
    p = DeviceProblem(w, Q, K, V, Phi)
    tol = TOL[w.dtype]
    Kc, Vc = p.measure()
    assert_close("Kc", to_np(Kc), ref["Kc"], tol)
    assert_close("Vc", to_np(Vc), ref["Vc"], tol)
    A, Z = p.attention(Kc, Vc)
    assert_close("A", to_np(A), ref["A"], tol)
    assert_close("Z", to_np(Z), ref["Z"], tol)
    X, C = p.recover(A, w.lam, mu, w.iters)
    assert_close("X (recover)", to_np(X), ref["X"], tol)
    assert_close("C (recover)", to_np(C), ref["C"], tol)
    C2, Z2, X2 = p.forward(w.lam, mu, w.iters)
    assert_close("Z (forward)", to_np(Z2), ref["Z"], tol)
    assert_close("X (forward)", to_np(X2), ref["X"], tol)
    assert_close("C (forward)", to_np(C2), ref["C"], tol)
    if w.dtype == "f32":
        flipped, band = _support_check(w.name, to_np(X2), ref, mu * w.lam)
        print(f"{w.name}: {flipped} of {band} tie-band coordinates differ in support")
    # only C requested: same values as with every optional output requested
    C3, _, _ = p.forward(w.lam, mu, w.iters, want_z=False, want_x=False)
    assert torch.equal(C3, C2)
    # deterministic: a second run is bit-identical
    C4, _, X4 = p.forward(w.lam, mu, w.iters)
    assert torch.equal(C4, C2) and torch.equal(X4, X2)


# the column-wise reading (self-attention shapes): lambda is on the scale of Z's entries
RD_SMALL = [
    _small("rd_f32", B=2, H=2, n_q=203, n=203, d=64, m=75, dtype="f32", iters=7, lam=0.6),
    _small("rd_bf16", B=2, H=2, n_q=203, n=203, d=64, m=75, dtype="bf16", iters=7, lam=0.6),      # fused decoder
    _small("rd_d128_bf16", B=1, H=3, n_q=300, n=300, d=128, m=136, dtype="bf16", phi_kind="rademacher", iters=6, lam=0.4),
    _small("rd_wide_m_bf16", B=1, H=5, n_q=520, n=520, d=64, m=452, dtype="bf16", iters=5, lam=0.1),   # GEMM-pair decoder
    _small("rd_tiny_n", B=1, H=2, n_q=40, n=40, d=64, m=16, dtype="f32", iters=3, lam=1.0),          # more columns than tokens
]


@pytest.mark.parametrize("w", RD_SMALL, ids=lambda w: w.name)
def test_column_wise_forward_small(w):
    Q, K, V = gen.make_qkv(w)
    Phi = gen.make_workload_phi(w)
    mu = _mu(Phi)
    ref = orc.forward_rd(Q, K, V, Phi, w.lam, mu, w.iters)
    density = float((ref["X"] != 0).mean())
    assert 0.02 < density < 0.98, f"degenerate test case, density {density}"
    p = DeviceProblem(w, Q, K, V, Phi)
    tol = TOL[w.dtype]
    C, Z = p.forward_rd(w.lam, mu, w.iters)
    assert_close("Z", to_np(Z), ref["Z"], tol)
    assert_close("C", to_np(C), ref["C"], tol)
    if w.dtype == "f32":
        sg, so = to_np(C) != 0, ref["C"] != 0
        ambiguous = np.swapaxes(np.abs(np.abs(ref["U"]) - mu * w.lam) <= 1e-5 * mu * w.lam, 1, 2)
        assert not ((sg != so) & ~ambiguous).any(), "support mismatch outside the tie band"
    C2, _ = p.forward_rd(w.lam, mu, w.iters, want_z=False)
    assert torch.equal(C2, C)
    # no iterations: C = Z; and the other reading still runs on the same (larger) workspace
    C0, Z0 = p.forward_rd(w.lam, mu, 0)
    assert torch.equal(C0, Z0)
    assert_close("Z (no decoder)", to_np(Z0), ref["Z"], tol)
    Ca, _, _ = p.forward(w.lam, mu, 2, want_z=False, want_x=False)
    assert_close("C (row-wise reading)", to_np(Ca), orc.forward(Q, K, V, Phi, w.lam, mu, 2)["C"], tol)


def test_column_wise_identity_and_errors_on_gpu():
    """Phi = I, mu = 1: the output is the element-wise shrinkage of exact attention."""
    w = _small("rd_identity", B=1, H=2, n_q=96, n=96, d=64, m=96, dtype="f32", iters=2, lam=0.05)
    Q, K, V = gen.make_qkv(w)
    Phi = gen.quantize(gen.make_phi("identity", w.n, w.n), "f32")
    attn = orc.attention_exact(Q, K, V)
    want = np.where(np.abs(attn) > w.lam, attn - w.lam * np.sign(attn), 0.0)
    p = DeviceProblem(w, Q, K, V, Phi)
    C, Z = p.forward_rd(w.lam, 1.0, 2)
    assert_close("Z", to_np(Z), attn, 1e-4)
    assert np.abs(to_np(C) - want).max() <= 1e-4 * np.abs(attn).max()
    # cross-attention shapes are refused before anything is launched
    wx = _small("rd_cross", B=1, H=1, n_q=32, n=64, d=64, m=16, dtype="f32")
    Qx, Kx, Vx = gen.make_qkv(wx)
    px = DeviceProblem(wx, Qx, Kx, Vx, gen.make_workload_phi(wx))
    with pytest.raises(csat.CsatError):
        px.forward_rd(0.1, 0.5, 1)


LISTA_SMALL = [
    _small("lista_f32", B=2, H=2, n_q=150, n=203, d=64, m=75, dtype="f32", iters=6),
    _small("lista_bf16", B=2, H=2, n_q=150, n=203, d=64, m=75, dtype="bf16", iters=6),
    _small("lista_big_tiles_bf16", B=1, H=2, n_q=300, n=520, d=64, m=136, dtype="bf16", iters=5, lam=0.03),
    _small("lista_one_row", n_q=1, n=40, d=8, m=8, dtype="f32", iters=3),
    # a single layer on the large-tile path (alpha^(0) = 0 and the caller's X in the same launch)
    _small("lista_1layer_bf16", B=2, H=2, n_q=150, n=203, d=64, m=75, dtype="bf16", iters=1),
    # the same layers on the element-wise epilogue (name ends in _elementwise: see the test)
    _small("lista_bf16_elementwise", B=2, H=2, n_q=150, n=203, d=64, m=75, dtype="bf16", iters=6),
]


@pytest.mark.parametrize("w", LISTA_SMALL, ids=lambda w: w.name)
def test_lista_decoder_small(w, options):
    """The unrolled decoder with given weights: the analytic ones (then it is ISTA) and a perturbed,
    'learned-like' set with a different threshold per layer."""
    if w.name.endswith("_elementwise"):
        options("lista", 1)
    Q, K, V = gen.make_qkv(w)
    Phi = gen.make_workload_phi(w)
    mu = _mu(Phi)
    tol = TOL[w.dtype]
    p = DeviceProblem(w, Q, K, V, Phi)
    A, _ = p.attention(*p.measure())
    Y = to_np(A).reshape(-1, w.m)
    rng = np.random.default_rng(77)
    Phi64 = Phi.astype(np.float64)
    S0, B0 = np.eye(w.n) - mu * Phi64.T @ Phi64, mu * Phi64.T
    sets = [("analytic", S0, B0, [mu * w.lam] * w.iters),
            ("perturbed", S0 + 0.02 * rng.standard_normal(S0.shape) / np.sqrt(w.n),
             B0 * (1.0 + 0.1 * rng.standard_normal(B0.shape)), [mu * w.lam * (1.5 - 0.2 * t) for t in range(w.iters)])]
    for name, S, Bw, thetas in sets:
        S, Bw = gen.quantize(S.astype(np.float32), w.dtype), gen.quantize(Bw.astype(np.float32), w.dtype)
        thetas = [float(np.float32(t)) for t in thetas]
        Xo, Uo = orc.lista(Y, S, Bw, thetas)
        Xo = Xo.reshape(p.BH, w.n_q, w.n)
        density = float((Xo != 0).mean())
        assert 0.005 < density < 0.99, f"degenerate case, density {density}"
        Xg, Cg = p.recover_lista(A, S, Bw, thetas)
        assert_close(f"X ({name})", to_np(Xg), Xo, tol)
        Vq = gen.quantize(V, w.dtype).astype(np.float64)
        assert_close(f"C ({name})", to_np(Cg), Xo @ Vq, tol)
        if w.dtype == "f32":
            th = thetas[-1]
            ambiguous = (np.abs(np.abs(Uo) - th) <= 1e-5 * th).reshape(Xo.shape)
            assert not (((to_np(Xg) != 0) != (Xo != 0)) & ~ambiguous).any(), "support mismatch outside the tie band"
        if name == "analytic":      # the same problem through the ISTA entry point
            Xi, _ = p.recover(A, w.lam, mu, w.iters, want_c=False)
            assert_close("X (ISTA entry) vs LISTA oracle", to_np(Xi), Xo, 4 * tol)
    # only C requested, and no layers at all
    _, C2 = p.recover_lista(A, S, Bw, thetas, want_x=False)
    assert torch.equal(C2, Cg)
    X0, C0 = p.recover_lista(A, S, Bw, [])
    assert not X0.any() and not C0.any()


OMP_SMALL = [
    (_small("omp_f32", B=2, H=2, n_q=150, n=203, d=64, m=75, dtype="f32"), 6),
    (_small("omp_bf16", B=2, H=2, n_q=150, n=203, d=64, m=75, dtype="bf16"), 6),
    (_small("omp_wide_bf16", B=1, H=2, n_q=300, n=520, d=64, m=452, dtype="bf16"), 12),
    (_small("omp_one_row", n_q=1, n=40, d=8, m=8, dtype="f32"), 8),                    # k = m: exact fit
    (_small("omp_k1", B=1, H=2, n_q=70, n=160, d=64, m=48, dtype="f32"), 1),
]


@pytest.mark.parametrize("w,k", OMP_SMALL, ids=lambda v: v.name if hasattr(v, "name") else str(v))
def test_omp_decoder_small(w, k):
    """Matching pursuit: picks are integers decided by floating-point correlations, so rows whose
    every pick wins by a clear margin in the oracle must agree exactly (order included); the others
    must still be valid least-squares fits on k distinct columns."""
    Q, K, V = gen.make_qkv(w)
    Phi = gen.make_workload_phi(w)
    tol = TOL[w.dtype]
    p = DeviceProblem(w, Q, K, V, Phi)
    A, _ = p.attention(*p.measure())
    Y = to_np(A).reshape(-1, w.m).astype(np.float64)
    Xo, picks_o, margins = orc.omp(Y, Phi, k)
    Xg, Pg, Cg = p.recover_omp(A, k)
    Xg, Pg = to_np(Xg).reshape(-1, w.n), Pg.cpu().numpy().astype(np.int64).reshape(-1, k)
    thr = 1e-3 if w.dtype == "f32" else 1e-2
    unclear = margins <= thr
    prefix = np.where(unclear.any(axis=1), unclear.argmax(axis=1), k)       # picks before the first close call
    for i in range(Pg.shape[0]):
        assert list(Pg[i, :prefix[i]]) == list(picks_o[i, :prefix[i]]), f"row {i}: picks differ before a close call"
    clear = prefix == k
    print(f"{w.name}: {clear.mean():.2f} of the rows have only clear picks, mean clear prefix {prefix.mean():.1f} of {k}")
    assert prefix.mean() >= min(2.0, k) and clear.sum() >= min(4, Pg.shape[0])
    np.testing.assert_array_equal(Pg[clear], picks_o[clear])
    assert_close("X (clear rows)", Xg[clear][None], Xo[clear][None], tol)
    Vq = gen.quantize(V, w.dtype).astype(np.float64)
    Co = (Xo.reshape(p.BH, w.n_q, w.n) @ Vq).reshape(-1, w.d)
    assert_close("C (clear rows)", to_np(Cg).reshape(-1, w.d)[clear][None], Co[clear][None], tol)
    # every row: k distinct picks, non-zeros exactly there, residual orthogonal to the picked columns
    Phi64 = Phi.astype(np.float64)
    for i in range(Xg.shape[0]):
        assert len(set(Pg[i])) == k and set(np.flatnonzero(Xg[i])) <= set(Pg[i])
        r = Y[i] - Phi64 @ Xg[i]
        assert np.abs(Phi64[:, Pg[i]].T @ r).max() <= 5e-3 * max(np.abs(Phi64.T @ Y[i]).max(), 1e-30)
    # outputs are optional one by one; no picks at all gives zeros
    X2, _, _ = p.recover_omp(A, k, want_picks=False, want_c=False)
    assert np.array_equal(to_np(X2).reshape(-1, w.n), Xg)
    X0, _, C0 = p.recover_omp(A, 0)
    assert not X0.any() and not C0.any()


KV_CASES = [
    _small("kv_f32", B=2, H=2, n_q=150, n=203, d=64, m=75, dtype="f32", iters=5),                     # small GEMM pair
    _small("kv_bf16", B=2, H=2, n_q=150, n=203, d=64, m=75, dtype="bf16", iters=5),                    # fused decoder
    _small("kv_wide_m_bf16", B=1, H=2, n_q=300, n=520, d=64, m=452, dtype="bf16", iters=4, lam=0.008),  # large-tile pair
]


@pytest.mark.parametrize("w", KV_CASES, ids=lambda w: w.name)
def test_separate_key_and_value_matrices(w):
    """K~ = Phi_K K and V~ = Phi_V V with two different draws; the decoder runs through Phi_V."""
    Q, K, V = gen.make_qkv(w)
    PhiV = gen.make_workload_phi(w)
    PhiK = gen.quantize(gen.make_phi("rademacher", w.m, w.n, seed=7), w.dtype)
    mu = _mu(PhiV)
    ref = orc.forward(Q, K, V, PhiV, w.lam, mu, w.iters, Phi_K=PhiK)
    p = DeviceProblem(w, Q, K, V, PhiV)
    PhiKd = to_dev(PhiK, w.dtype)
    tol = TOL[w.dtype]
    Kc, Vc = p.empty(p.BH, w.m, w.d), p.empty(p.BH, w.m, w.d)
    csat.csat_measure_kv(p.dims, PhiKd, p.Phi, p.K, p.V, Kc, Vc, p.ws)
    assert_close("Kc", to_np(Kc), ref["Kc"], tol)
    assert_close("Vc", to_np(Vc), ref["Vc"], tol)
    C, Z = p.empty(p.BH, w.n_q, w.d), p.empty(p.BH, w.n_q, w.d)
    X = p.empty(p.BH, w.n_q, w.n, dtype=torch.float32)
    csat.csat_forward_kv(p.dims, p.Q, p.K, p.V, PhiKd, p.Phi, w.lam, mu, w.iters, C, Z, X, p.ws)
    torch.cuda.synchronize()
    assert_close("Z", to_np(Z), ref["Z"], tol)
    assert_close("X", to_np(X), ref["X"], tol)
    assert_close("C", to_np(C), ref["C"], tol)
    if w.dtype == "f32":
        _support_check(w.name, to_np(X), ref, mu * w.lam)
    # the same pointer twice is the shared-matrix call, bit for bit
    C1, _, X1 = p.forward(w.lam, mu, w.iters)
    C2, X2 = torch.empty_like(C1), torch.empty_like(X1)
    csat.csat_forward_kv(p.dims, p.Q, p.K, p.V, p.Phi, p.Phi, w.lam, mu, w.iters, C2, None, X2, p.ws)
    torch.cuda.synchronize()
    assert torch.equal(C2, C1) and torch.equal(X2, X1)
    with pytest.raises(csat.CsatError) as e:
        csat.csat_forward_kv(p.dims, p.Q, p.K, p.V, None, p.Phi, w.lam, mu, w.iters, C2, None, X2, p.ws)
    assert e.value.status == -1


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_separate_matrices_column_wise(dtype):
    w = _small("kv_rd_" + dtype, B=2, H=2, n_q=203, n=203, d=64, m=75, dtype=dtype, iters=6, lam=0.6)
    Q, K, V = gen.make_qkv(w)
    PhiV = gen.make_workload_phi(w)
    PhiK = gen.quantize(gen.make_phi("gaussian", w.m, w.n, seed=9), w.dtype)
    mu = _mu(PhiV)
    ref = orc.forward_rd(Q, K, V, PhiV, w.lam, mu, w.iters, Phi_K=PhiK)
    density = float((ref["X"] != 0).mean())
    assert 0.02 < density < 0.98, f"degenerate test case, density {density}"
    p = DeviceProblem(w, Q, K, V, PhiV)
    C, Z = p.empty(p.BH, w.n, w.d), p.empty(p.BH, w.n, w.d)
    csat.csat_forward_rd_kv(p.dims, p.Q, p.K, p.V, to_dev(PhiK, w.dtype), p.Phi, w.lam, mu, w.iters, C, Z, p.ws)
    torch.cuda.synchronize()
    assert_close("Z", to_np(Z), ref["Z"], TOL[dtype])
    assert_close("C", to_np(C), ref["C"], TOL[dtype])



@pytest.mark.parametrize("segments", [2, 3, 7])
@pytest.mark.parametrize("thin", ["0", "1"])
def test_fused_decoder_segments_are_bit_identical(segments, thin, options):
    """The fused decoder hands its residual operands from one segment of the iterations to the next;
    however the iterations are cut, the arithmetic is the same, so the results must not change by a bit.
    Both work shapes: 128-row workgroups (thin = 0, what large launches get) and one 32-row tile per
    workgroup (what a launch this small gets by default)."""
    w = _small("segments_bf16", B=2, H=3, n_q=150, n=203, d=64, m=75, dtype="bf16", iters=7)
    Q, K, V = gen.make_qkv(w)
    Phi = gen.make_workload_phi(w)
    mu = _mu(Phi)
    p = DeviceProblem(w, Q, K, V, Phi)
    options("fused_thin", 1 if thin == "0" else 0)       # option value 1 = 128-row workgroups
    options("fused_segments", 1)
    C1, _, X1 = p.forward(w.lam, mu, w.iters)
    options("fused_segments", segments)
    Cs, _, Xs = p.forward(w.lam, mu, w.iters)
    assert torch.equal(Cs, C1) and torch.equal(Xs, X1)
    ref = orc.forward(Q, K, V, Phi, w.lam, mu, w.iters)
    assert_close("X", to_np(Xs), ref["X"], TOL[w.dtype])
    # the dense-state and the sparse-state variant give the same iterate (the library picks by problem size)
    for state in (1, 2):                                  # dense, sparse
        options("state", state)
        Cd, _, Xd = p.forward(w.lam, mu, w.iters)
        assert torch.equal(Xd, X1) and torch.equal(Cd, C1)


ATTN_CASES = [(m, dtype, d) for m in (75, 392, 600, 1100) for dtype, d in (("f32", 64), ("bf16", 64))] + [
    (136, "bf16", 128), (200, "f32", 72), (200, "bf16", 72), (513, "bf16", 128), (8, "f32", 8), (33, "bf16", 16)]


@pytest.mark.parametrize("m,dtype,d", ATTN_CASES)
def test_compressed_attention_in_one_kernel(m, dtype, d, options):
    """Scores, row softmax and output product in one kernel (the softmax inside the score tile): A~ and Z against
    the oracle for rows that fit the registers in one sweep (m <= 512) and for longer rows (two sweeps), ragged
    row tiles, every head dimension the tests use; and against the three-kernel path kept behind an option."""
    n = max(m + 57, 130)
    w = _small(f"attn_m{m}_{dtype}_d{d}", B=1, H=3, n_q=77, n=n, d=d, m=m, dtype=dtype, iters=0, seed=60 + m)
    Q, K, V = gen.make_qkv(w)
    Phi = gen.make_workload_phi(w)
    ref = orc.forward(Q, K, V, Phi, 0.0, 1.0, 0)
    tol = TOL[dtype]
    p = DeviceProblem(w, Q, K, V, Phi)
    Kc, Vc = p.measure()
    options("attention", 2)              # the one kernel whatever the shape (by default a short query side takes three)
    A, Z = p.attention(Kc, Vc)
    assert_close("A", to_np(A), ref["A"], tol)
    assert_close("Z", to_np(Z), ref["Z"], tol)
    assert torch.allclose(A.view(-1, m).sum(-1), torch.ones(A.numel() // m, device=DEV), atol=1e-5)
    Z1 = p.empty(p.BH, w.n_q, w.d)
    csat.csat_compressed_attention(p.dims, p.Q, Kc, Vc, None, Z1, p.ws)          # A~ not requested
    torch.cuda.synchronize()
    assert torch.equal(Z1, Z)
    options("attention", 1)
    A3, Z3 = p.attention(Kc, Vc)
    assert_close("A (three kernels)", to_np(A3), ref["A"], tol)
    assert_close("A, one kernel vs three", to_np(A), to_np(A3), 2 * tol)
    assert_close("Z, one kernel vs three", to_np(Z), to_np(Z3), 2 * tol)
    # the whole block (the (hi | lo) pair of K~ in bf16 mode) on either path
    C3, Zf3, _ = p.forward(0.0, 1.0, 0, want_x=False)
    options("attention", 2)
    C1, Zf1, _ = p.forward(0.0, 1.0, 0, want_x=False)
    assert torch.equal(C1, Zf1)
    assert_close("Z (forward)", to_np(Zf1), ref["Z"], tol)
    assert_close("Z (forward), one kernel vs three", to_np(Zf1), to_np(Zf3), 2 * tol)


MEASURE_CASES = [(203, 75, 64), (520, 452, 64), (64, 33, 64), (300, 136, 128), (512, 200, 128), (1600, 392, 64),
                 (72, 8, 64), (1000, 96, 128)]


@pytest.mark.parametrize("n,m,d", MEASURE_CASES)
def test_measurement_in_one_kernel(n, m, d, options):
    """bf16 with d = 64 or 128 measures K~ and V~ in one kernel that reads K and V as they are (Phi as the caller
    holds it when n % 8 == 0, else its padded copy) and writes every copy of K~ and V~ the attention stage reads.
    Against the oracle, and against the two-GEMM path kept behind an option: the stage call, and the whole block
    with Z (which goes through the fragments of K~ and of V~: the attention kernel forms Z from them itself)."""
    w = _small(f"measure_n{n}_m{m}_d{d}", B=1, H=3, n_q=min(n, 150), n=n, d=d, m=m, dtype="bf16", iters=3, seed=80 + m)
    Q, K, V = gen.make_qkv(w)
    Phi = gen.make_workload_phi(w)
    mu = _mu(Phi)
    ref = orc.forward(Q, K, V, Phi, w.lam, mu, w.iters)
    tol = TOL["bf16"]
    p = DeviceProblem(w, Q, K, V, Phi)
    Kc, Vc = p.measure()
    assert_close("Kc", to_np(Kc), ref["Kc"], tol)
    assert_close("Vc", to_np(Vc), ref["Vc"], tol)
    C, Z, X = p.forward(w.lam, mu, w.iters)
    assert_close("Z", to_np(Z), ref["Z"], tol)
    assert_close("C", to_np(C), ref["C"], tol)
    Cn, _, Xn = p.forward(w.lam, mu, w.iters, want_z=False)        # V~ not computed
    assert torch.equal(Cn, C) and torch.equal(Xn, X)
    # V~ transposed for a product GEMM behind the attention kernel instead of as that kernel's fragments
    options("measure", 2)
    Ct, Zt, Xt = p.forward(w.lam, mu, w.iters)
    assert_close("Z, product in the attention kernel vs as a GEMM", to_np(Z), to_np(Zt), 2 * tol)
    assert torch.equal(Ct, C) and torch.equal(Xt, X)            # A~ does not depend on how Z is formed
    options("measure", 1)
    Kg, Vg = p.measure()
    assert_close("Kc, one kernel vs GEMMs", to_np(Kc), to_np(Kg), tol)
    assert_close("Vc, one kernel vs GEMMs", to_np(Vc), to_np(Vg), tol)
    Cg, Zg, Xg = p.forward(w.lam, mu, w.iters)
    assert_close("Z, one kernel vs GEMMs", to_np(Z), to_np(Zg), 2 * tol)
    assert_close("C, one kernel vs GEMMs", to_np(C), to_np(Cg), 2 * tol)
    assert_close("Z (GEMMs)", to_np(Zg), ref["Z"], tol)


def test_decoder_give_up_is_reported(options):
    """The fused decoder bounds its wait for a hand-over between segments.  A wait that runs out must not pass
    for a result: csat_decoder_status reports it and X and C of that call hold NaN.  The failure is forced from
    the host (the error record is pre-set, as if an earlier unit had given up), so every kernel still exits
    normally; the next ordinary call on the same workspace is clean again."""
    w = _small("give_up_bf16", B=2, H=3, n_q=150, n=203, d=64, m=75, dtype="bf16", iters=7)
    Q, K, V = gen.make_qkv(w)
    Phi = gen.make_workload_phi(w)
    mu = _mu(Phi)
    p = DeviceProblem(w, Q, K, V, Phi)
    C0, _, X0 = p.forward(w.lam, mu, w.iters)
    assert csat.csat_decoder_status(p.ws) == 0
    for thin in (0, 1):
        options("fused_thin", thin)
        options("fused_segments", 3)
        options("inject_decoder_error", 1)
        C, _, X = p.forward(w.lam, mu, w.iters)
        assert csat.csat_decoder_status(p.ws) == csat.CSAT_ERR_TIMEOUT
        assert torch.isnan(X).all() and torch.isnan(C.float()).all()
        options("inject_decoder_error", 0)
        C1, _, X1 = p.forward(w.lam, mu, w.iters)
        assert csat.csat_decoder_status(p.ws) == 0
        assert torch.equal(C1, C0) and torch.equal(X1, X0)
    # a wait limit of zero polls: a unit gives up unless the segment before it is already done.  Whether any
    # unit does depends on timing; either the call is reported failed and poisoned, or it is the usual result.
    options("fused_spin_limit", -1)
    options("fused_segments", 7)
    C2, _, X2 = p.forward(w.lam, mu, w.iters)
    if csat.csat_decoder_status(p.ws) == 0:
        assert torch.equal(C2, C0) and torch.equal(X2, X0)
    else:
        assert torch.isnan(X2).all() and torch.isnan(C2.float()).all()
    # the GEMM-pair decoder has no hand-over: its status is always clean, also behind a failed call
    options("fused_spin_limit", 0)
    options("inject_decoder_error", 1)
    p.forward(w.lam, mu, w.iters)
    options("inject_decoder_error", 0)
    options("decoder", 1)
    Cg, _, Xg = p.forward(w.lam, mu, w.iters)
    assert csat.csat_decoder_status(p.ws) == 0
    assert_close("X (GEMM pair)", to_np(Xg), to_np(X0), 2 * TOL[w.dtype])


FUSED_CASES = [w for w in SMALL if w.dtype == "bf16" and w.m <= 416 and w.n > 64]


@pytest.mark.parametrize("w", FUSED_CASES, ids=lambda w: w.name)
def test_fused_decoder_with_128_row_workgroups(w, options):
    """Launches this small get one 32-row tile per workgroup by default; large ones get 128-row workgroups.
    The small cases again on that shape, element by element against the oracle, and bit for bit against the
    default shape (same arithmetic per row)."""
    Q, K, V = gen.make_qkv(w)
    Phi = gen.make_workload_phi(w)
    mu = _mu(Phi)
    ref = orc.forward(Q, K, V, Phi, w.lam, mu, w.iters)
    p = DeviceProblem(w, Q, K, V, Phi)
    C1, _, X1 = p.forward(w.lam, mu, w.iters)
    options("fused_thin", 1)
    C0, Z0, X0 = p.forward(w.lam, mu, w.iters)
    assert_close("X", to_np(X0), ref["X"], TOL[w.dtype])
    assert_close("C", to_np(C0), ref["C"], TOL[w.dtype])
    assert torch.equal(X0, X1) and torch.equal(C0, C1)


WIDE_FUSED_CASES = [      # (n_q, n, m, iterations, 128-row workgroups)
    (300, 1000, 448, 3, 0),     # 14 tiles of m; one 32-row tile per workgroup
    (160, 704, 512, 4, 1),      # 16 tiles, all full
    (77, 4096, 512, 3, 1),      # cross_modal's rows
    (130, 777, 470, 2, 1),      # 15 tiles, the last ragged; ragged last chunk; two iterations
    (96, 520, 500, 1, 1),       # a single iteration
]


@pytest.mark.parametrize("n_q,n,m,iters,groups128", WIDE_FUSED_CASES)
def test_fused_decoder_with_14_to_16_tiles_of_m(n_q, n, m, iters, groups128, options):
    """bf16 and 416 < m <= 512: the residual accumulators fill the accumulator file and the decoder runs on the
    one-chunk schedule.  Launches with enough rows get it by default; here it is forced onto small ones.  Against the
    oracle, and against the GEMM pair (same operands, another summation order)."""
    w = _small(f"wide_fused_m{m}", B=2, H=3, n_q=n_q, n=n, d=64, m=m, dtype="bf16", iters=iters, seed=7 + m, lam=0.01)
    Q, K, V = gen.make_qkv(w)
    Phi = gen.make_workload_phi(w)
    mu = _mu(Phi)
    ref = orc.forward(Q, K, V, Phi, w.lam, mu, iters)
    p = DeviceProblem(w, Q, K, V, Phi)
    Cg, _, Xg = p.forward(w.lam, mu, iters)
    assert csat.csat_profile_decoder_kernel() == -1          # few rows: the GEMM pair
    options("decoder", 2)
    options("fused_thin", groups128)
    for state in (1, 2, 2 + 4):                              # dense, sparse, sparse with streamed accesses
        options("state", state)
        C, _, X = p.forward(w.lam, mu, iters)
        assert csat.csat_decoder_status(p.ws) == 0
        assert csat.csat_profile_decoder_kernel() == (2 if not groups128 else (0 if state == 1 else 1))
        assert_close("X", to_np(X), ref["X"], TOL["bf16"])
        assert_close("C", to_np(C), ref["C"], TOL["bf16"])
        assert_close("X (GEMM pair)", to_np(Xg), to_np(X), 2 * TOL["bf16"])


SCHEDULE_CASES = [      # (n, m, iterations): even and odd chunk counts, the shortest row the two-chunk schedule takes,
    (1600, 392, 3),     # the headline row length; partially sparse iterates from the second iteration on
    (704, 200, 2),
    (1600, 75, 3),      # three residual tiles: the narrowest instantiation on this schedule
    (448, 392, 3),
    (180, 100, 4),      # six chunks, the last ragged: the shortest row sent to this schedule (three steps)
    (700, 150, 3),      # 22 chunks with a ragged last one
    (660, 392, 2),      # odd count (21 chunks, the last ragged) padded by a zero chunk
    (704, 200, 1),      # a single iteration: only the last-iteration form of the step runs
    (512, 416, 2),      # the widest instantiation (13 tiles of m, all of them full), sixteen chunks
]


@pytest.mark.parametrize("n,m,iters", SCHEDULE_CASES)
def test_fused_decoder_schedules_are_bit_identical(n, m, iters, options):
    """The 128-row fused decoder has two schedules of the same arithmetic (one column chunk per step, or two);
    both sum every product in the same order, so the iterate must agree bit for bit, with dense and with
    sparse state and however the iterations are cut into segments.  The one-chunk result is checked against
    the oracle, so the agreement pins the other one to it too."""
    w = _small("schedules_bf16", B=2, H=3, n_q=150, n=n, d=64, m=m, dtype="bf16", iters=iters)
    Q, K, V = gen.make_qkv(w)
    Phi = gen.make_workload_phi(w)
    mu = _mu(Phi)
    p = DeviceProblem(w, Q, K, V, Phi)
    options("fused_thin", 1)                              # 128-row workgroups, as large launches get
    options("fused_schedule", 1)                          # one chunk per step
    options("state", 1)
    C1, _, X1 = p.forward(w.lam, mu, iters)
    ref = orc.forward(Q, K, V, Phi, w.lam, mu, iters)
    assert_close("X", to_np(X1), ref["X"], TOL[w.dtype])
    nonzero = float((X1 != 0).float().mean())
    print(f"n={n} m={m} iterations={iters}: non-zero share of the iterate {nonzero:.3f}")
    assert csat.csat_profile_decoder_kernel() == 0        # one chunk per step, dense state
    options("fused_schedule", 0)                          # the library's choice: two chunks per step for these rows
    for state in (1, 2):
        for segments in (1, 2, 3):
            options("state", state)
            options("fused_segments", segments)
            C2, _, X2 = p.forward(w.lam, mu, iters)
            assert csat.csat_decoder_status(p.ws) == 0
            assert csat.csat_profile_decoder_kernel() == 2 + state         # the two-chunk kernels really ran
            assert torch.equal(X2, X1), (state, segments, float((X2 != X1).float().mean()))
            assert torch.equal(C2, C1), (state, segments)
    # the other work distribution of the two-chunk kernel (what large launches get): the 8 groups x iterations of
    # this launch in 3, 5 and 8 equal shares, a share running the beginning of its last group first and the end of
    # its first group last
    options("state", 0)
    for shares in (3, 5, 8):
        options("fused_segments", -shares)
        C3, _, X3 = p.forward(w.lam, mu, iters)
        assert csat.csat_decoder_status(p.ws) == 0
        assert csat.csat_profile_decoder_kernel() >= 3
        assert torch.equal(X3, X1) and torch.equal(C3, C1), shares


def test_large_tile_orders_are_bit_identical(options):
    """The large-tile GEMM walks its tiles in an order that depends on the shape (16 column tiles here: every XCD owns
    an eighth of them and walks them in groups); the order must not change a single bit of the decoder's result.
    Against the oracle, and the column-fastest order and the other group sizes against the default; so must not the
    cache hint that large row operands are loaded with (16: forced on here, with and without a group size)."""
    w = _small("tile_order_bf16", B=1, H=2, n_q=300, n=4096, d=64, m=448, dtype="bf16", iters=3, lam=0.004, seed=97)
    Q, K, V = gen.make_qkv(w)
    Phi = gen.make_workload_phi(w)
    mu = _mu(Phi)
    ref = orc.forward(Q, K, V, Phi, w.lam, mu, w.iters)
    p = DeviceProblem(w, Q, K, V, Phi)
    C0, _, X0 = p.forward(w.lam, mu, w.iters)
    assert csat.csat_profile_decoder_kernel() == -1          # the GEMM pair (m > 416 and few rows)
    assert_close("X", to_np(X0), ref["X"], TOL["bf16"])
    assert_close("C", to_np(C0), ref["C"], TOL["bf16"])
    for order in (1, 2, 3, 5, 16, 16 + 3):
        options("raster", order)
        C1, _, X1 = p.forward(w.lam, mu, w.iters)
        assert torch.equal(X1, X0) and torch.equal(C1, C0), order


DIRECT_SYNTHESIS_CASES = [w for w in SMALL if w.dtype == "bf16" and w.d in (64, 128) and w.iters > 0]


@pytest.mark.parametrize("w", DIRECT_SYNTHESIS_CASES, ids=lambda w: w.name)
def test_synthesis_straight_from_v(w, options):
    """bf16 with d = 64 or 128: the product kernel behind the decoder reads V as the caller holds it (no transposed
    copy); the small bf16 cases (ragged n and n_q, one to fifteen tiles of m, both decoders) against the oracle and
    against the GEMM over the transposed copy, which sums in another order; csat_recover takes the same kernel."""
    Q, K, V = gen.make_qkv(w)
    Phi = gen.make_workload_phi(w)
    mu = _mu(Phi)
    ref = orc.forward(Q, K, V, Phi, w.lam, mu, w.iters)
    p = DeviceProblem(w, Q, K, V, Phi)
    options("synthesis", 1)                                   # (not inside the decoder, where that would apply)
    C1, _, X1 = p.forward(w.lam, mu, w.iters)
    Kc, Vc = p.measure()
    Y, _ = p.attention(Kc, Vc)
    _, C1r = p.recover(Y, w.lam, mu, w.iters, want_x=False)
    options("synthesis", 2)
    C2, _, X2 = p.forward(w.lam, mu, w.iters)
    _, C2r = p.recover(Y, w.lam, mu, w.iters, want_x=False)
    assert torch.equal(X1, X2)
    assert_close_iterate("C", to_np(C1), ref["C"], ref["U"], TOL["bf16"], scale_by_ratio_of=(ref["X"], ref["U"]))
    assert_close("C (GEMM over V^T)", to_np(C2), to_np(C1), TOL["bf16"])
    assert_close("C (csat_recover)", to_np(C2r), to_np(C1r), TOL["bf16"])


SYNTHESIS_CASES = [(160, 704, 200, 3), (96, 1600, 392, 2), (320, 448, 100, 4), (32, 660, 392, 1), (160, 512, 416, 3)]


@pytest.mark.parametrize("n_q,n,m,iters", SYNTHESIS_CASES)
def test_synthesis_in_the_decoder(n_q, n, m, iters, options):
    """bf16 with d = 64 and whole 32-row tiles per head: the two-chunk fused decoder forms C = X V itself in its
    last iteration (from V as MFMA fragments; no bf16 copy of the iterate, no product kernel).  Against the oracle
    and against the product kernel kept behind an option; 128-row groups that straddle heads (n_q = 160, 96, 32),
    a padded last group, an odd chunk count padded by a zero chunk, a single iteration."""
    w = _small(f"synthesis_nq{n_q}_n{n}", B=2, H=3, n_q=n_q, n=n, d=64, m=m, dtype="bf16", iters=iters, seed=90 + n_q,
               lam=0.05 if m < 300 else 0.01)
    Q, K, V = gen.make_qkv(w)
    Phi = gen.make_workload_phi(w)
    mu = _mu(Phi)
    ref = orc.forward(Q, K, V, Phi, w.lam, mu, iters)
    tol = TOL["bf16"]
    p = DeviceProblem(w, Q, K, V, Phi)
    options("fused_thin", 1)                              # 128-row workgroups, as large launches get
    C, Z, X = p.forward(w.lam, mu, iters)
    assert csat.csat_decoder_status(p.ws) == 0
    assert csat.csat_profile_decoder_kernel() >= 3        # the two-chunk kernel ran
    assert_close("X", to_np(X), ref["X"], tol)
    assert_close("C", to_np(C), ref["C"], tol)
    Cn, _, _ = p.forward(w.lam, mu, iters, want_z=False, want_x=False)
    assert torch.equal(Cn, C)
    for shares in (3, 5):                                 # ... and however the work is cut
        options("fused_segments", -shares)
        Cs, _, Xs = p.forward(w.lam, mu, iters)
        assert torch.equal(Cs, C) and torch.equal(Xs, X), shares
    options("fused_segments", 0)
    # A~ goes from the attention kernel to this decoder in accumulator tiles; row-major must give the same bits
    options("y_layout", 1)
    Cr, Zr, Xr = p.forward(w.lam, mu, iters)
    assert torch.equal(Cr, C) and torch.equal(Xr, X) and torch.equal(Zr, Z)
    Cr, _, _ = p.forward(w.lam, mu, iters, want_z=False, want_x=False)
    assert torch.equal(Cr, C)
    options("y_layout", 0)
    options("synthesis", 1)
    Cg, _, Xg = p.forward(w.lam, mu, iters)
    assert torch.equal(Xg, X)
    assert_close("C, in the decoder vs product kernel", to_np(C), to_np(Cg), 2 * tol)
    assert_close("C (product kernel)", to_np(Cg), ref["C"], tol)


HADAMARD_SMALL = [
    _small("hadamard_f32", B=2, H=2, n_q=150, n=203, d=64, m=75, dtype="f32", iters=7),
    _small("hadamard_bf16", B=2, H=2, n_q=150, n=203, d=64, m=75, dtype="bf16", iters=7),
    _small("hadamard_pow2", B=1, H=2, n_q=70, n=2048, d=64, m=392, dtype="bf16", iters=6, lam=0.02),   # n = N, four passes
    _small("hadamard_tiny", n_q=3, n=40, d=8, m=8, dtype="f32", iters=3),                             # N = 64 < 256 threads
    _small("hadamard_long", B=1, H=1, n_q=5, n=9000, d=64, m=700, dtype="f32", iters=4, lam=0.02),      # N = 16384
    # every transform length of the register-resident kernel: N = 512, 1024 (2048 and 16384 above), 4096, 8192
    _small("hadamard_512_f32", B=1, H=2, n_q=33, n=300, d=64, m=120, dtype="f32", iters=6),
    _small("hadamard_1024_bf16", B=1, H=2, n_q=21, n=700, d=64, m=250, dtype="bf16", iters=5, lam=0.03),
    # nine column groups per head in the measurement kernel (d = 72), three heads
    _small("hadamard_d72_bf16", B=1, H=3, n_q=40, n=600, d=72, m=200, dtype="bf16", iters=4, lam=0.03),
    _small("hadamard_4096_bf16", B=1, H=2, n_q=9, n=3000, d=64, m=500, dtype="bf16", iters=5, lam=0.02),
    _small("hadamard_8192_f32", B=1, H=1, n_q=7, n=5000, d=64, m=333, dtype="f32", iters=3, lam=0.02),
]


@pytest.mark.parametrize("w", HADAMARD_SMALL, ids=lambda w: w.name)
def test_hadamard_decoder_small(w):
    """Structured Phi applied by Walsh-Hadamard transforms: the whole path with the explicit matrix in
    the measurement and attention stages and the transform-based decoder, against the oracle's ISTA
    with the same explicit matrix."""
    Q, K, V = gen.make_qkv(w)
    Phi64, rows_of_h, signs = gen.make_hadamard_phi(w.m, w.n, seed=9)
    Phi = gen.quantize(Phi64, w.dtype)
    mu = _mu(Phi)
    tol = TOL[w.dtype]
    ref = orc.forward(Q, K, V, Phi, w.lam, mu, w.iters)
    density = float((ref["X"] != 0).mean())
    assert 0.001 < density < 0.95, f"degenerate case, density {density}"
    p = DeviceProblem(w, Q, K, V, Phi)
    # the measurement by transforms (no stored matrix) against the oracle's product with the explicit matrix
    Kh, Vh = p.measure_hadamard(rows_of_h, signs)
    assert_close("Kc (transforms)", to_np(Kh), ref["Kc"], tol)
    assert_close("Vc (transforms)", to_np(Vh), ref["Vc"], tol)
    A, _ = p.attention(Kh, Vh)
    assert_close("A", to_np(A), ref["A"], tol)
    Xo, _, Uo = orc.ista_trace(to_np(A).reshape(-1, w.m), Phi, w.lam, mu, w.iters)     # from the GPU's own A
    Xg, Cg = p.recover_hadamard(A, rows_of_h, signs, w.lam, mu, w.iters)
    assert_close("X", to_np(Xg).reshape(-1, w.n)[None], Xo[None], 1e-4)                # fp32 transforms in both modes
    Vq = gen.quantize(V, w.dtype).astype(np.float64)
    assert_close("C", to_np(Cg), Xo.reshape(p.BH, w.n_q, w.n) @ Vq, tol)
    theta = mu * w.lam
    ambiguous = np.abs(np.abs(Uo) - theta) <= 1e-5 * theta
    mismatch = (to_np(Xg).reshape(-1, w.n) != 0) != (Xo != 0)
    print(f"{w.name}: {int(ambiguous.sum())} coordinates in the tie band, {int((mismatch & ambiguous).sum())} of them differ in support")
    assert not (mismatch & ~ambiguous).any(), "support mismatch outside the tie band"
    # the same problem through the stored-matrix decoder
    Xs, _ = p.recover(A, w.lam, mu, w.iters, want_c=False)
    assert_close("X (stored Phi)", to_np(Xs).reshape(-1, w.n)[None], Xo[None], 2 * tol)
    X0, C0 = p.recover_hadamard(A, rows_of_h, signs, w.lam, mu, 0)
    assert not X0.any() and not C0.any()


@pytest.mark.parametrize("w", HADAMARD_SMALL, ids=lambda w: w.name)
def test_forward_hadamard_small(w):
    """The whole block with the structured matrix in one call (no stored Phi on the GPU side) against the
    oracle's forward with the explicit matrix."""
    Q, K, V = gen.make_qkv(w)
    Phi64, rows_of_h, signs = gen.make_hadamard_phi(w.m, w.n, seed=9)
    Phi = gen.quantize(Phi64, w.dtype)
    mu = _mu(Phi)
    tol = TOL[w.dtype]
    ref = orc.forward(Q, K, V, Phi, w.lam, mu, w.iters)
    p = DeviceProblem(w, Q, K, V, Phi)
    C, Z, X = p.forward_hadamard(rows_of_h, signs, w.lam, mu, w.iters)
    assert_close("Z", to_np(Z), ref["Z"], tol)
    assert_close("X", to_np(X), ref["X"], tol)
    assert_close("C", to_np(C), ref["C"], tol)
    if w.dtype == "f32":
        flipped, band = _support_check(w.name, to_np(X), ref, mu * w.lam)
        print(f"{w.name}: {flipped} of {band} tie-band coordinates differ in support")
    C2, _, _ = p.forward_hadamard(rows_of_h, signs, w.lam, mu, w.iters, want_z=False, want_x=False)
    assert torch.equal(C2, C)
    C0, Z0, _ = p.forward_hadamard(rows_of_h, signs, w.lam, mu, 0, want_x=False)
    assert torch.equal(C0, Z0)
    assert_close("Z (no decoder)", to_np(Z0), ref["Z"], tol)


@pytest.mark.parametrize("w", RD_SMALL + [
    _small("rd_hadamard_4096_bf16", B=1, H=2, n_q=2500, n=2500, d=16, m=400, dtype="bf16", iters=4, lam=0.3)], ids=lambda w: w.name)
def test_column_wise_forward_hadamard_small(w):
    """The column-wise reading with the structured matrix (measurement, Y = Phi Z and decoder by transforms)
    against the oracle's column-wise forward with the explicit matrix."""
    Q, K, V = gen.make_qkv(w)
    Phi64, rows_of_h, signs = gen.make_hadamard_phi(w.m, w.n, seed=9)
    Phi = gen.quantize(Phi64, w.dtype)
    mu = _mu(Phi)
    tol = TOL[w.dtype]
    ref = orc.forward_rd(Q, K, V, Phi, w.lam, mu, w.iters)
    density = float((ref["X"] != 0).mean())
    assert 0.01 < density < 0.99, f"degenerate test case, density {density}"
    p = DeviceProblem(w, Q, K, V, Phi)
    C, Z = p.forward_rd_hadamard(rows_of_h, signs, w.lam, mu, w.iters)
    assert_close("Z", to_np(Z), ref["Z"], tol)
    assert_close("C", to_np(C), ref["C"], tol)
    C2, _ = p.forward_rd_hadamard(rows_of_h, signs, w.lam, mu, w.iters, want_z=False)
    assert torch.equal(C2, C)
    C0, Z0 = p.forward_rd_hadamard(rows_of_h, signs, w.lam, mu, 0)
    assert torch.equal(C0, Z0)
    assert_close("Z (no decoder)", to_np(Z0), ref["Z"], tol)


def test_identity_phi_is_exact_attention_on_gpu():
    """Phi = I (m = n), lambda = 0: compressed attention and the whole block give softmax(QK^T/sqrt d)V."""
    w = _small("identity", B=1, H=2, n_q=96, n=96, d=64, m=96, dtype="f32", iters=3, lam=0.0)
    Q, K, V = gen.make_qkv(w)
    Phi = gen.quantize(gen.make_phi("identity", w.n, w.n), "f32")
    want = orc.attention_exact(Q, K, V)
    p = DeviceProblem(w, Q, K, V, Phi)
    Kc, Vc = p.measure()
    assert torch.equal(Kc, p.K) and torch.equal(Vc, p.V)
    _, Z = p.attention(Kc, Vc)
    assert_close("Z", to_np(Z), want, 1e-4)
    C, _, X = p.forward(0.0, 1.0, 3)
    assert_close("C", to_np(C), want, 1e-4)


def test_forward_identities_on_gpu():
    w = _small("ident2", B=1, H=2, n_q=70, n=160, d=64, m=48, dtype="f32")
    Q, K, V = gen.make_qkv(w)
    Phi = gen.make_workload_phi(w)
    mu = _mu(Phi)
    p = DeviceProblem(w, Q, K, V, Phi)
    # no decoder iterations: C = Z
    C0, Z0, _ = p.forward(0.1, mu, 0, want_x=False)
    assert torch.equal(C0, Z0)
    ref = orc.forward(Q, K, V, Phi, 0.1, mu, 0)
    assert_close("Z", to_np(Z0), ref["Z"], 1e-4)
    # lambda = 0, one iteration: C = mu Z
    C1, Z1, _ = p.forward(0.0, mu, 1, want_x=False)
    assert_close("C vs mu Z", to_np(C1), mu * ref["Z"], 1e-4)
    # recover with zero iterations returns zeros
    A, _ = p.attention(*p.measure())
    X, C = p.recover(A, 0.1, mu, 0)
    assert not X.any() and not C.any()
    # lambda >= ||Phi^T y||_inf: every iterate is zero
    big = float(np.abs(to_np(A).reshape(-1, w.m) @ Phi.astype(np.float64)).max() * 1.01)
    X, _ = p.recover(A, big, mu, 4)
    assert not X.any()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_planted_sparse_recovery_on_gpu(dtype):
    """csat_recover as a generic batched ISTA: planted k-sparse rows, noise-free; the recovered
    support is the planted one (and the oracle's) bit for bit."""
    m, n, k, rows = 64, 128, 4, 96
    Phi64, Xs, sups = gen.planted_sparse(21, m, n, k, rows=rows)
    Phi = gen.quantize(Phi64, dtype)
    Y = (Xs @ Phi.astype(np.float64).T).astype(np.float32)
    mu = _mu(Phi)
    lam, iters = 0.05, 300
    ref_X, _, ref_U = orc.ista_trace(Y, Phi, lam, mu, iters)
    dims = csat.make_dims(1, 1, rows, n, 8, m, dtype)
    ws = csat.alloc_workspace(dims, iters)
    X = torch.empty(rows, n, device=DEV)
    csat.csat_recover(dims, torch.from_numpy(Y).to(DEV), to_dev(Phi, dtype), lam, mu, iters, X, None, None, ws)
    Xg = to_np(X)
    assert_close("X", Xg[None], ref_X[None], TOL[dtype])
    planted = np.zeros((rows, n), dtype=bool)
    np.put_along_axis(planted, sups, True, axis=1)
    big = np.abs(ref_X) > 1e-3
    assert (big & planted).sum() == planted.sum()         # every planted coordinate is recovered ...
    assert (big != planted).sum() <= 0.002 * planted.size  # ... with next to no spurious ones
    np.testing.assert_array_equal(np.abs(Xg) > 1e-3, big)
    if dtype == "f32":
        _support_check("planted", Xg, {"X": ref_X, "U": ref_U}, mu * lam)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_planted_sparse_omp_on_gpu(dtype):
    """Matching pursuit on planted k-sparse rows, noise-free: the picked set is the planted one for
    (nearly) every row, equal to the oracle's picks as a set, and the coefficients are exact."""
    m, n, k, rows = 64, 128, 4, 200
    Phi64, Xs, sups = gen.planted_sparse(23, m, n, k, rows=rows)
    Phi = gen.quantize(Phi64, dtype)
    Y = (Xs @ Phi.astype(np.float64).T).astype(np.float32)
    Xo, picks_o, margins = orc.omp(Y, Phi, k)
    dims = csat.make_dims(1, 1, rows, n, 8, m, dtype)
    ws = torch.empty(csat.csat_omp_workspace_bytes(dims, k), dtype=torch.uint8, device=DEV)
    X = torch.empty(rows, n, device=DEV)
    P = torch.empty(rows, k, dtype=torch.int32, device=DEV)
    csat.csat_recover_omp(dims, torch.from_numpy(Y).to(DEV), to_dev(Phi, dtype), k, X, P, None, None, ws)
    Xg, Pg = to_np(X), P.cpu().numpy().astype(np.int64)
    recovered = np.array([sorted(picks_o[i]) == list(sups[i]) for i in range(rows)])
    assert recovered.mean() > 0.95                       # greedy recovery holds for almost every draw
    same = np.array([sorted(Pg[i]) == sorted(picks_o[i]) for i in range(rows)])
    assert same[recovered].all()                         # integer result: the same set of columns
    clear = margins.min(axis=1) > (1e-3 if dtype == "f32" else 1e-2)
    np.testing.assert_array_equal(Pg[clear], picks_o[clear])      # and the same order where no call was close
    assert_close("X", Xg[recovered][None], Xs[recovered][None], 1e-4 if dtype == "f32" else 2e-2)


def test_full_short_video_omp_sampled():
    """Matching pursuit at the headline workload's size, k = 8: sampled rows against the oracle."""
    w = gen.WORKLOADS["short_video"]
    k = 8
    Q, K, V = gen.make_qkv(w)
    Phi = gen.make_workload_phi(w)
    p = DeviceProblem(w, Q, K, V, Phi)
    A, _ = p.attention(*p.measure())
    X, P, C = p.recover_omp(A, k)
    rng = np.random.default_rng(98)
    Vq = gen.quantize(V, w.dtype).astype(np.float64)
    Phi64 = Phi.astype(np.float64)
    checked = 0
    for h in np.sort(rng.choice(p.BH, size=3, replace=False)):
        rows = np.sort(rng.choice(w.n_q, size=48, replace=False))
        ridx = torch.from_numpy(rows).to(DEV)
        Y = to_np(A[h][ridx]).astype(np.float64)
        Xo, picks_o, margins = orc.omp(Y, Phi, k)
        Xg, Pg = to_np(X[h][ridx]), P[h][ridx].cpu().numpy().astype(np.int64)
        unclear = margins <= 1e-2
        prefix = np.where(unclear.any(axis=1), unclear.argmax(axis=1), k)
        for i in range(len(rows)):
            assert list(Pg[i, :prefix[i]]) == list(picks_o[i, :prefix[i]])
            r = Y[i] - Phi64 @ Xg[i]
            assert len(set(Pg[i])) == k and np.abs(Phi64[:, Pg[i]].T @ r).max() <= 5e-3 * np.abs(Phi64.T @ Y[i]).max()
        clear = prefix == k
        checked += int(clear.sum())
        if clear.any():
            assert_close(f"X[{h}]", Xg[clear][None], Xo[clear][None], TOL[w.dtype])
            assert_close(f"C[{h}]", to_np(C[h][ridx])[clear][None], (Xo @ Vq[h])[clear][None], TOL[w.dtype])
    print(f"short_video, matching pursuit: {checked} sampled rows with only clear picks")
    assert checked >= 8


FULL = ["image_text", "short_video", "cross_modal", "long_video"]


@pytest.mark.parametrize("name", FULL)
def test_full_workloads_sampled(name):
    """Full-size workloads in the launch configuration the benchmark times.  Stages 1-3 are
    compared in full on a subset of heads; decoder and synthesis on sampled query rows (rows are
    independent problems, so the oracle computes exactly those)."""
    w = gen.WORKLOADS[name]
    BH = w.B * w.H
    Q, K, V = gen.make_qkv(w)
    Phi = gen.make_workload_phi(w)
    mu = _mu(Phi)
    tol = TOL[w.dtype]
    p = DeviceProblem(w, Q, K, V, Phi)
    rng = np.random.default_rng(1234)
    heads = np.sort(rng.choice(BH, size=min(BH, 4), replace=False))
    nrows = {"image_text": 48, "short_video": 32, "cross_modal": 24, "long_video": 12}[name]
    Kc, Vc = p.measure()
    A, Z = p.attention(Kc, Vc)
    C, Z2, X = p.forward(w.lam, mu, w.iters)
    assert_close("Z forward vs stage", to_np(Z2), to_np(Z), tol)
    for h in heads:
        rows = np.sort(rng.choice(w.n_q, size=min(nrows, w.n_q), replace=False))
        ref = orc.forward(Q[h:h + 1], K[h:h + 1], V[h:h + 1], Phi, w.lam, mu, w.iters, rows=rows)
        assert_close(f"Kc[{h}]", to_np(Kc[h:h + 1]), ref["Kc"], tol)
        assert_close(f"Vc[{h}]", to_np(Vc[h:h + 1]), ref["Vc"], tol)
        assert_close(f"A[{h}]", to_np(A[h:h + 1]), ref["A"], tol)
        assert_close(f"Z[{h}]", to_np(Z[h:h + 1]), ref["Z"], tol)
        ridx = torch.from_numpy(rows).to(DEV)
        assert_close(f"X[{h}]", to_np(X[h][ridx])[None], ref["X"], tol)
        assert_close(f"C[{h}]", to_np(C[h][ridx])[None], ref["C"], tol)
    # properties that hold at any size
    Ag = A.view(-1, w.m)
    assert torch.allclose(Ag.sum(-1), torch.ones(Ag.shape[0], device=DEV), atol=1e-5)
    nz = float((X != 0).float().mean())
    print(f"{name}: density of X = {nz:.4f}")
    assert 0.0 < nz < 0.7


@pytest.mark.parametrize("name", ["image_text", "short_video", "cross_modal"])
def test_full_workloads_every_row(name):
    """Full-size workloads 2-4 in the launch configuration the benchmark times, every stage, every head and
    every query row against the oracle (a head at a time), and a second call that must repeat the first bit
    for bit (at this size the fused decoder runs its default work distribution: hundreds of row groups whose
    iterations are cut into segments handed from workgroup to workgroup)."""
    w = gen.WORKLOADS[name]
    BH = w.B * w.H
    Q, K, V = gen.make_qkv(w)
    Phi = gen.make_workload_phi(w)
    mu = _mu(Phi)
    tol = TOL[w.dtype]
    p = DeviceProblem(w, Q, K, V, Phi)
    Kc, Vc = p.measure()
    A, Z = p.attention(Kc, Vc)
    C, Z2, X = p.forward(w.lam, mu, w.iters)
    assert csat.csat_decoder_status(p.ws) == 0
    worst = {}
    for h in range(BH):
        ref = orc.forward(Q[h:h + 1], K[h:h + 1], V[h:h + 1], Phi, w.lam, mu, w.iters)
        for key, got in (("Kc", Kc), ("Vc", Vc), ("A", A), ("Z", Z), ("Z (forward)", Z2), ("X", X), ("C", C)):
            err = assert_close(f"{key}[{h}]", to_np(got[h:h + 1]), ref[key.split(" ")[0]], tol)
            worst[key] = max(worst.get(key, 0.0), err)
    print(f"{name}: worst relative error over {BH} heads x {w.n_q} rows: " + ", ".join(f"{k} {v:.2e}" for k, v in worst.items()))
    C2, _, X2 = p.forward(w.lam, mu, w.iters)
    assert torch.equal(C2, C) and torch.equal(X2, X), "a repeated call differs"


def test_sweep_shape_compressed_block():
    """The compressed block (measurement + compressed attention) at the shape of the sequence sweep the
    benchmark times (batch 4, 12 heads, d = 64, m = 256 fixed, n = 8192): two heads in full against the oracle,
    and every row of A~ sums to one."""
    w = _small("sweep_n8192", B=4, H=12, n_q=8192, n=8192, d=64, m=256, dtype="bf16", iters=0, seed=8192)
    Q, K, V = gen.make_qkv(w)
    Phi = gen.make_workload_phi(w)
    p = DeviceProblem(w, Q, K, V, Phi)
    Kc, Vc = p.measure()
    A, Z = p.attention(Kc, Vc)
    for h in (0, 29):
        ref = orc.forward(Q[h:h + 1], K[h:h + 1], V[h:h + 1], Phi, 0.0, 1.0, 0)
        for key, got in (("Kc", Kc), ("Vc", Vc), ("A", A), ("Z", Z)):
            assert_close(f"{key}[{h}]", to_np(got[h:h + 1]), ref[key], TOL[w.dtype])
    Ag = A.view(-1, w.m)
    assert torch.allclose(Ag.sum(-1), torch.ones(Ag.shape[0], device=DEV), atol=1e-5)


@pytest.mark.parametrize("name", ["image_text", "short_video", "long_video"])
def test_full_workloads_column_wise_sampled(name):
    """The column-wise reading at full size: compressed output in full on a subset of heads,
    decoded output on sampled feature columns (columns are independent problems)."""
    w = gen.WORKLOADS[name]
    BH = w.B * w.H
    Q, K, V = gen.make_qkv(w)
    Phi = gen.make_workload_phi(w)
    mu = _mu(Phi)
    tol = TOL[w.dtype]
    p = DeviceProblem(w, Q, K, V, Phi)
    rng = np.random.default_rng(4321)
    heads = np.sort(rng.choice(BH, size=min(BH, 3), replace=False))
    C, Z = p.forward_rd(w.lam, mu, w.iters)
    for h in heads:
        cols = np.sort(rng.choice(w.d, size=8, replace=False))
        ref = orc.forward_rd(Q[h:h + 1], K[h:h + 1], V[h:h + 1], Phi, w.lam, mu, w.iters, cols=cols)
        assert_close(f"Z[{h}]", to_np(Z[h:h + 1]), ref["Z"], tol)
        cidx = torch.from_numpy(cols).to(DEV)
        assert_close(f"C[{h}]", to_np(C[h][:, cidx])[None], ref["C"], tol)
    nz = float((C != 0).float().mean())
    print(f"{name}: density of the column-wise output = {nz:.4f}")
    assert 0.0 < nz < 0.99


@pytest.mark.parametrize("name", ["image_text", "short_video", "long_video"])
def test_full_workloads_column_wise_hadamard_sampled(name):
    """The column-wise reading with the structured matrix at full size: sampled feature columns against the
    oracle's column-wise forward with the explicit matrix."""
    w = gen.WORKLOADS[name]
    BH = w.B * w.H
    Q, K, V = gen.make_qkv(w)
    Phi64, rows_of_h, signs = gen.make_hadamard_phi(w.m, w.n, seed=9)
    Phi = gen.quantize(Phi64, w.dtype)
    mu = _mu(Phi)
    tol = TOL[w.dtype]
    p = DeviceProblem(w, Q, K, V, Phi)
    rng = np.random.default_rng(987)
    C, Z = p.forward_rd_hadamard(rows_of_h, signs, w.lam, mu, w.iters)
    for h in np.sort(rng.choice(BH, size=min(BH, 2), replace=False)):
        cols = np.sort(rng.choice(w.d, size=6, replace=False))
        ref = orc.forward_rd(Q[h:h + 1], K[h:h + 1], V[h:h + 1], Phi, w.lam, mu, w.iters, cols=cols)
        assert_close(f"Z[{h}]", to_np(Z[h:h + 1]), ref["Z"], tol)
        cidx = torch.from_numpy(cols).to(DEV)
        assert_close(f"C[{h}]", to_np(C[h][:, cidx])[None], ref["C"], tol)
    nz = float((C != 0).float().mean())
    print(f"{name}: density of the column-wise output = {nz:.4f}")
    assert 0.0 < nz < 0.995


def test_full_short_video_lista_sampled():
    """The unrolled decoder at the headline workload's size (analytic weights rounded to bf16):
    sampled rows against the oracle (rows are independent problems)."""
    w = gen.WORKLOADS["short_video"]
    Q, K, V = gen.make_qkv(w)
    Phi = gen.make_workload_phi(w)
    mu = _mu(Phi)
    tol = TOL[w.dtype]
    p = DeviceProblem(w, Q, K, V, Phi)
    A, _ = p.attention(*p.measure())
    Phi64 = Phi.astype(np.float64)
    S = gen.quantize((np.eye(w.n) - mu * Phi64.T @ Phi64).astype(np.float32), w.dtype)
    Bw = gen.quantize((mu * Phi64.T).astype(np.float32), w.dtype)
    thetas = [float(np.float32(mu * w.lam))] * w.iters
    X, C = p.recover_lista(A, S, Bw, thetas)
    rng = np.random.default_rng(99)
    Vq = gen.quantize(V, w.dtype).astype(np.float64)
    for h in np.sort(rng.choice(p.BH, size=3, replace=False)):
        rows = np.sort(rng.choice(w.n_q, size=24, replace=False))
        ridx = torch.from_numpy(rows).to(DEV)
        Xo, _ = orc.lista(to_np(A[h][ridx]), S, Bw, thetas)
        assert_close(f"X[{h}]", to_np(X[h][ridx])[None], Xo[None], tol)
        assert_close(f"C[{h}]", to_np(C[h][ridx])[None], (Xo @ Vq[h])[None], tol)
    nz = float((X != 0).float().mean())
    print(f"short_video, unrolled decoder: density of X = {nz:.4f}")
    assert 0.0 < nz < 0.7


def _random_case(seed):
    rng = np.random.default_rng(1000 + seed)
    dtype = ["f32", "bf16"][seed % 2]
    n = int(rng.integers(8, 600))
    m = int(rng.integers(1, min(n, 460) + 1))
    return _small(f"random{seed}", B=int(rng.integers(1, 4)), H=int(rng.integers(1, 4)), n_q=int(rng.integers(1, 300)),
                  n=n, m=m, d=int(rng.choice([8, 16, 64, 72, 128])), dtype=dtype, iters=int(rng.integers(1, 7)),
                  phi_kind=["gaussian", "rademacher"][int(rng.integers(0, 2))], seed=50 + seed)


@pytest.mark.parametrize("seed", range(24))
def test_random_shapes(seed):
    """Seeded random shapes (ragged everything, m from 1 to n, both element types): every stage against the
    oracle; the decoder is fed the GPU's own compressed attention so that only its own error is compared,
    with lambda set from the data so that the iterate is neither empty nor full; then the whole block in one
    call against the oracle's whole block."""
    w = _random_case(seed)
    Q, K, V = gen.make_qkv(w)
    Phi = gen.make_workload_phi(w)
    mu = _mu(Phi)
    tol = TOL[w.dtype]
    p = DeviceProblem(w, Q, K, V, Phi)
    ref = orc.forward(Q, K, V, Phi, 0.0, mu, 0)
    Kc, Vc = p.measure()
    assert_close("Kc", to_np(Kc), ref["Kc"], tol)
    assert_close("Vc", to_np(Vc), ref["Vc"], tol)
    A, Z = p.attention(Kc, Vc)
    assert_close("A", to_np(A), ref["A"], tol)
    assert_close("Z", to_np(Z), ref["Z"], tol)
    Y = to_np(A).reshape(-1, w.m)
    # 15 % of the first iterate survives the threshold, in both element types
    lam = float(np.quantile(np.abs(Y @ Phi.astype(np.float64)), 0.85))
    Xo, _, Uo = orc.ista_trace(Y, Phi, lam, mu, w.iters)
    X, C = p.recover(A, lam, mu, w.iters)
    Xg = to_np(X).reshape(-1, w.n)
    Vq = gen.quantize(V, w.dtype).astype(np.float64)
    assert_close_iterate(f"{w.name} X", Xg[None], Xo[None], Uo[None], tol)
    assert_close_iterate(f"{w.name} C", to_np(C).reshape(1, -1, w.d), (Xo.reshape(p.BH, w.n_q, w.n) @ Vq).reshape(1, -1, w.d),
                         Uo[None], tol, scale_by_ratio_of=(Xo[None], Uo[None]))
    if w.dtype == "f32":
        theta = mu * lam
        ambiguous = np.abs(np.abs(Uo) - theta) <= 1e-5 * theta
        assert not (((Xg != 0) != (Xo != 0)) & ~ambiguous).any(), "support mismatch outside the tie band"
    # the whole block in one call against the oracle's whole block (its own compressed attention)
    ref = orc.forward(Q, K, V, Phi, lam, mu, w.iters)
    Cf, Zf, Xf = p.forward(lam, mu, w.iters)
    assert_close("Z (forward)", to_np(Zf), ref["Z"], tol)
    U_all = ref["U"].reshape(1, -1, w.n)
    assert_close_iterate(f"{w.name} X (forward)", to_np(Xf).reshape(1, -1, w.n), ref["X"].reshape(1, -1, w.n), U_all, tol)
    assert_close_iterate(f"{w.name} C (forward)", to_np(Cf).reshape(1, -1, w.d), ref["C"].reshape(1, -1, w.d), U_all, tol,
                         scale_by_ratio_of=(ref["X"].reshape(1, -1, w.n), U_all))


def test_reference_kernels_of_the_benchmark():
    """The streaming copy copies (ragged tail included); the MFMA loop reports its operation count."""
    g = torch.Generator(device="cpu").manual_seed(3)
    src = torch.randint(0, 255, ((1 << 22) + 16 * 37,), dtype=torch.uint8, generator=g).to(DEV)
    dst = torch.zeros_like(src)
    assert csat.csat_peak_copy(src, dst) == 2 * src.numel()
    torch.cuda.synchronize()
    assert torch.equal(src, dst)
    out = torch.empty(1 << 18, dtype=torch.float32, device=DEV)
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    assert csat.csat_peak_mfma(out, 3) == cus * 2 * 4 * 3 * 16 * 2.0 * 32 * 32 * 16
    torch.cuda.synchronize()
    assert torch.isfinite(out[: cus * 2 * 256]).all()
    # one wavefront per SIMD with other instructions behind each MFMA: every supported mix runs and counts its flops
    for kv, kl in ((0, 0), (3, 0), (6, 0), (9, 0), (12, 0), (0, 1), (3, 1), (6, 1), (0, 2)):
        out.fill_(float("nan"))
        assert csat.csat_peak_mfma_issue(out, 2, kv, kl) == cus * 4 * 2 * 8 * 2.0 * 32 * 32 * 16
        torch.cuda.synchronize()
        assert torch.isfinite(out[: cus * 256]).all()
    with pytest.raises(csat.CsatError) as e:
        csat.csat_peak_mfma_issue(out, 2, 5, 0)
    assert e.value.status == -6


@pytest.mark.parametrize("name", ["tiny", "ragged_bf16", "wide_m_bf16"])
def test_forward_on_a_side_stream_and_in_a_captured_graph(name):
    """The whole forward is stream-ordered kernel launches (buffers are cleared by fill kernels, the fused
    decoder's counters included), so it runs on any stream and can be captured; every replay, with eager
    work and synchronisations between the replays, must reproduce the eager result bit for bit."""
    w = next(x for x in SMALL if x.name == name)
    Q, K, V = gen.make_qkv(w)
    Phi = gen.make_workload_phi(w)
    mu = _mu(Phi)
    p = DeviceProblem(w, Q, K, V, Phi)
    C0, Z0, X0 = p.forward(w.lam, mu, w.iters)
    C, Z, X = torch.zeros_like(C0), torch.zeros_like(Z0), torch.zeros_like(X0)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        csat.csat_forward(p.dims, p.Q, p.K, p.V, p.Phi, w.lam, mu, w.iters, C, Z, X, p.ws)
    side.synchronize()
    assert torch.equal(C, C0) and torch.equal(Z, Z0) and torch.equal(X, X0)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        csat.csat_forward(p.dims, p.Q, p.K, p.V, p.Phi, w.lam, mu, w.iters, C, Z, X, p.ws)
    for replay in range(3):
        C.zero_(), Z.zero_(), X.zero_()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(C, C0) and torch.equal(Z, Z0) and torch.equal(X, X0), f"replay {replay}"
        Ce, _, _ = p.forward(w.lam, mu, max(w.iters - 1, 1))      # eager work on the same workspace in between
        assert torch.isfinite(Ce.float()).all()


@pytest.mark.parametrize("name", ["short_video", "cross_modal", "long_video"])
def test_full_workloads_hadamard_sampled(name):
    """The transform-based decoder at full size, in the launch configuration the benchmark times
    (N = 2048, 4096, 16384): the iterate of sampled rows against the oracle's ISTA with the explicit
    subsampled-Hadamard matrix, fed the GPU's own measurements (rows are independent problems)."""
    w = gen.WORKLOADS[name]
    Q, K, V = gen.make_qkv(w)
    Phi64, rows_of_h, signs = gen.make_hadamard_phi(w.m, w.n, seed=9)
    Phi = gen.quantize(Phi64, w.dtype)
    mu = _mu(Phi)
    p = DeviceProblem(w, Q, K, V, Phi)
    Kh, Vh = p.measure_hadamard(rows_of_h, signs)
    Ks, Vs = p.measure()                                    # the same product with the stored matrix
    assert_close("Kc transforms vs stored", to_np(Kh), to_np(Ks), TOL[w.dtype])
    assert_close("Vc transforms vs stored", to_np(Vh), to_np(Vs), TOL[w.dtype])
    A, _ = p.attention(Kh, Vh)
    Xg, Cg = p.recover_hadamard(A, rows_of_h, signs, w.lam, mu, w.iters)
    rng = np.random.default_rng(4321)
    theta = mu * w.lam
    Vq = gen.quantize(V, w.dtype).astype(np.float64)
    for h in np.sort(rng.choice(p.BH, size=min(p.BH, 3), replace=False)):
        rows = np.sort(rng.choice(w.n_q, size=min(10, w.n_q), replace=False))
        ridx = torch.from_numpy(rows).to(DEV)
        Xo, _, Uo = orc.ista_trace(to_np(A[h][ridx]), Phi, w.lam, mu, w.iters)
        got = to_np(Xg[h][ridx])
        assert_close(f"X[{h}]", got[None], Xo[None], 1e-4)                       # fp32 transforms in both modes
        assert_close(f"C[{h}]", to_np(Cg[h][ridx])[None], (Xo @ Vq[h])[None], TOL[w.dtype])
        ambiguous = np.abs(np.abs(Uo) - theta) <= 1e-5 * theta
        mismatch = (got != 0) != (Xo != 0)
        print(f"{name}[{h}]: {int(ambiguous.sum())} coordinates in the tie band, {int((mismatch & ambiguous).sum())} of them differ in support")
        assert not (mismatch & ~ambiguous).any(), "support mismatch outside the tie band"
    nz = float((Xg != 0).float().mean())
    print(f"{name}: density of X = {nz:.4f}")
    assert 0.0 < nz < 0.9
    # the same block in one call, against the oracle's whole forward on sampled rows of one head
    del Xg, Cg
    Cf, Zf, Xf = p.forward_hadamard(rows_of_h, signs, w.lam, mu, w.iters)
    h = int(rng.integers(p.BH))
    rows = np.sort(rng.choice(w.n_q, size=min(8, w.n_q), replace=False))
    ridx = torch.from_numpy(rows).to(DEV)
    ref = orc.forward(Q[h:h + 1], K[h:h + 1], V[h:h + 1], Phi, w.lam, mu, w.iters, rows=rows)
    assert_close("Z (one call)", to_np(Zf[h:h + 1]), ref["Z"], TOL[w.dtype])
    assert_close("X (one call)", to_np(Xf[h][ridx])[None], ref["X"], TOL[w.dtype])
    assert_close("C (one call)", to_np(Cf[h][ridx])[None], ref["C"], TOL[w.dtype])
