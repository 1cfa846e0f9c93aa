"""fp64 CPU oracle for the CSAT forward pass.  TEST INFRASTRUCTURE ONLY.

This file is the yardstick the HIP kernels are compared with.  It is written
from the paper's equations, step by step, in float64 numpy, with no blocking,
fusion or reordering, and it shares no code with the GPU path.  Only tests,
the smoke check and the benchmark's `cpu_baseline` leg may import it; the
product path must never route through it.

What each function follows (paper: "CS-VLM: Compressed Sensing Attention",
section 3 "Mathematical Framework"):

  attention_exact        eq. Attn(Q,K,V) = softmax(Q K^T / sqrt(d_k)) V
  measure                eq. K~ = Phi_K K, V~ = Phi_V V            (one shared Phi, or the two given)
  compressed_attention   eq. A~ = softmax(Q K~^T / sqrt(d_k)),  Z = A~ V~
  ista / ista_trace      the ISTA decoder named in section 3 for the l1 problem
                         min ||alpha||_1 s.t. measurements = Phi alpha, solved in
                         its LASSO form  min 1/2 ||y - Phi x||^2 + lambda ||x||_1
  lista_form             eq. alpha^(t+1) = eta_theta(S alpha^(t) + B y) with the
                         analytic weights S = I - mu Phi^T Phi, B = mu Phi^T,
                         theta = mu lambda
  lista                  the same equation with caller-supplied ("learned") S, B and
                         one threshold per layer
  omp                    orthogonal matching pursuit, the greedy decoder the paper names
                         next to ISTA (introduction and limitations); the paper gives no
                         details, so this is the standard algorithm: pick the column most
                         correlated with the residual (largest |phi_j^T r|, lowest index on a
                         tie, never a column twice), refit all picked coefficients by least
                         squares, update the residual; exactly k picks
  phi_fill               the measurement ensembles section 3 names (random Gaussian, Rademacher), drawn from
                         a counter-based generator so that any element can be produced on its own: word k
                         of seed s is output k of SplitMix64 (Steele, Lea, Flood 2014) started at s; element
                         i = r n + c takes words 2 i and 2 i + 1; Gaussian by Box-Muller from
                         u1 = ((w1 >> 11) + 1) 2^-53, u2 = (w2 >> 11) 2^-53, scaled by 1/sqrt(m);
                         Rademacher +-1/sqrt(m) by the top bit of w1.  (The scaling and the generator are this
                         build's choice: the paper names the ensembles only.)
  synthesize / forward   eq. C^_i = Psi alpha^_i, applied row-wise
  forward_rd             second reading of the recovery passage (column-wise, see below)

Readings of passages the paper leaves open or states inconsistently
(the recovery equation Z_i = Phi Psi alpha_i does not type-check as printed:
Z_i has d_k entries, Phi has n columns, Psi is d_k x d_k):

  * the signal recovered per query i is its length-n attention row over the
    original keys; its length-m measurement is the compressed attention row
    y_i = A~[i, :]; the synthesis operator "Psi" of C^_i = Psi alpha^_i is V^T,
    so C^_i = sum_j x_ij V[j, :] is literally the attention definition;
  * step size mu and l1 weight lambda are inputs; threshold is theta = mu*lambda;
  * x^0 = 0, exactly T iterations, no early exit;
  * |u| == theta maps to 0 (strict inequality defines the support);
  * two-sided soft threshold (no sign constraint);
  * one Phi shared by keys, values, all batches and all heads; where the caller gives the two
    matrices of K~ = Phi_K K, V~ = Phi_V V separately, Phi_K is used for K~ only and Phi_V is the
    decoder's matrix (the recovery passage names Phi_V as the one reused for decoding; with it the
    identity "lambda = 0, one iteration => C^ = mu Z" holds whatever Phi_K is);
  * softmax over the m compressed keys, scale 1/sqrt(d_k), no mask.

Second reading (forward_rd, self-attention only, n_q = n): the paper motivates
the recovery by redundancy of the context matrix along the token axis and
claims a cost linear in n.  Read that way, each of the d_k feature columns of
the context matrix is a length-n signal, its measurement is the same column of
Y = Phi Z (Z = A~ V~, the compressed block's output, measured with the shared
Phi), the ISTA decoder above recovers it, and the recovered columns are the
output: d_k problems per head instead of n_q.

Pins (tests/test_oracle_*.py): Phi = I reduces to exact attention (checked
against torch's fp64 scaled_dot_product_attention); planted k-sparse recovery
matches exhaustive support search; ISTA converges to the exhaustive KKT LASSO
solution and to scikit-learn's coordinate-descent Lasso; closed forms for
orthogonal Phi; objective monotone; hand-worked fixtures in tests/golden/.
Full-size workloads 2-5 have no printed reference values in the paper:
"parity unpinned" beyond these identities.
"""
from __future__ import annotations

import numpy as np

__all__ = [
    "phi_opnorm_sq", "attention_exact", "measure", "compressed_scores_counted",
    "compressed_attention", "soft_threshold", "ista", "ista_trace", "lista_form",
    "lasso_objective", "synthesize", "forward", "forward_rd", "support", "lista", "omp",
    "splitmix64_words", "phi_fill",
]


def _f64(a):
    return np.asarray(a, dtype=np.float64)


def phi_opnorm_sq(Phi) -> float:
    """L = ||Phi||_2^2, the largest eigenvalue of Phi Phi^T (ISTA's Lipschitz constant)."""
    Phi = _f64(Phi)
    return float(np.linalg.eigvalsh(Phi @ Phi.T)[-1])


def splitmix64_words(seed: int, first: int, count: int) -> np.ndarray:
    """Outputs first .. first+count-1 of SplitMix64 started at `seed` (output k mixes seed + (k + 1) gamma)."""
    with np.errstate(over="ignore"):
        k = np.arange(first + 1, first + count + 1, dtype=np.uint64)
        z = np.uint64(seed & 0xFFFFFFFFFFFFFFFF) + k * np.uint64(0x9E3779B97F4A7C15)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        return z ^ (z >> np.uint64(31))


def phi_fill(kind: str, seed: int, m: int, n: int) -> np.ndarray:
    """Phi [m, n] in float32: kind "gaussian" (entries N(0, 1/m)) or "rademacher" (entries +-1/sqrt(m))."""
    w = splitmix64_words(seed, 0, 2 * m * n).reshape(m * n, 2)
    if kind == "rademacher":
        sign = np.where(w[:, 0] >> np.uint64(63), -1.0, 1.0)
        return (sign / np.sqrt(float(m))).astype(np.float32).reshape(m, n)
    if kind != "gaussian":
        raise ValueError(kind)
    u1 = ((w[:, 0] >> np.uint64(11)).astype(np.float64) + 1.0) * 2.0 ** -53      # (0, 1]
    u2 = (w[:, 1] >> np.uint64(11)).astype(np.float64) * 2.0 ** -53              # [0, 1)
    g = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
    return (g / np.sqrt(float(m))).astype(np.float32).reshape(m, n)


def _softmax_rows(S):
    S = S - S.max(axis=-1, keepdims=True)
    E = np.exp(S)
    return E / E.sum(axis=-1, keepdims=True)


def attention_exact(Q, K, V):
    """softmax(Q K^T / sqrt(d_k)) V for Q [..., n_q, d], K, V [..., n, d]."""
    Q, K, V = _f64(Q), _f64(K), _f64(V)
    d = Q.shape[-1]
    A = _softmax_rows(Q @ np.swapaxes(K, -1, -2) / np.sqrt(d))
    return A @ V


def measure(Phi, K, V, Phi_K=None):
    """K~ = Phi_K K and V~ = Phi_V V: matrices [m, n], K, V [..., n, d] -> [..., m, d].
    Phi is Phi_V; Phi_K defaults to the same matrix (the shared-Phi case)."""
    Phi, K, V = _f64(Phi), _f64(K), _f64(V)
    Phi_K = Phi if Phi_K is None else _f64(Phi_K)
    return Phi_K @ K, Phi @ V


def compressed_scores_counted(Q, Kc):
    """Scores S = Q K~^T / sqrt(d_k) for one head with explicit loops, returning
    (S [n_q, m], number of multiply-accumulates).  Small inputs only."""
    Q, Kc = _f64(Q), _f64(Kc)
    n_q, d = Q.shape
    m = Kc.shape[0]
    S = np.zeros((n_q, m))
    macs = 0
    for i in range(n_q):
        for l in range(m):
            acc = 0.0
            for c in range(d):
                acc += Q[i, c] * Kc[l, c]
                macs += 1
            S[i, l] = acc / np.sqrt(d)
    return S, macs


def compressed_attention(Q, Kc, Vc):
    """A~ = softmax(Q K~^T / sqrt(d_k)) [..., n_q, m] and Z = A~ V~ [..., n_q, d]."""
    Q, Kc, Vc = _f64(Q), _f64(Kc), _f64(Vc)
    d = Q.shape[-1]
    A = _softmax_rows(Q @ np.swapaxes(Kc, -1, -2) / np.sqrt(d))
    return A, A @ Vc


def soft_threshold(u, theta):
    """eta_theta(u) = sign(u) * max(|u| - theta, 0)."""
    u = _f64(u)
    return np.sign(u) * np.maximum(np.abs(u) - theta, 0.0)


def ista_trace(Y, Phi, lam, mu, iters):
    """ISTA on independent rows.  Y [rows, m], Phi [m, n].
    Returns (X [rows, n], list of iterates X^1..X^T, last pre-threshold U [rows, n])."""
    Y, Phi = _f64(Y), _f64(Phi)
    X = np.zeros((Y.shape[0], Phi.shape[1]))
    theta = mu * lam
    trace, U = [], np.zeros_like(X)
    for _ in range(int(iters)):
        R = Y - X @ Phi.T            # residual y - Phi x
        U = X + mu * (R @ Phi)       # gradient step  x + mu Phi^T r
        X = soft_threshold(U, theta)
        trace.append(X)
    return X, trace, U


def ista(Y, Phi, lam, mu, iters):
    """X after exactly `iters` ISTA iterations from X^0 = 0."""
    return ista_trace(Y, Phi, lam, mu, iters)[0]


def lista_form(Y, Phi, lam, mu, iters):
    """The unrolled-network form alpha <- eta_theta(S alpha + B y) with analytic weights."""
    Y, Phi = _f64(Y), _f64(Phi)
    n = Phi.shape[1]
    S = np.eye(n) - mu * (Phi.T @ Phi)
    Bm = mu * Phi.T                                  # [n, m]
    X = np.zeros((Y.shape[0], n))
    for _ in range(int(iters)):
        X = soft_threshold(X @ S.T + Y @ Bm.T, mu * lam)
    return X


def lista(Y, S, Bm, thetas):
    """The unrolled decoder alpha^(t+1) = eta_theta_t(S alpha^(t) + B y) from alpha^(0) = 0 with
    given weights: Y [rows, m], S [n, n], Bm [n, m], thetas one threshold per layer.
    Returns (X [rows, n], last pre-threshold values U [rows, n])."""
    Y, S, Bm = _f64(Y), _f64(S), _f64(Bm)
    X = np.zeros((Y.shape[0], S.shape[0]))
    U = np.zeros_like(X)
    for theta in thetas:
        U = X @ S.T + Y @ Bm.T
        X = soft_threshold(U, float(theta))
    return X, U


def omp(Y, Phi, k):
    """Orthogonal matching pursuit on independent rows.  Y [rows, m], Phi [m, n], k picks per row.
    Returns (X [rows, n] with k non-zeros per row, picks [rows, k] column indices in the order
    they were chosen, margins [rows, k]: how far ahead the chosen correlation was of the runner-up,
    relative to the chosen one)."""
    Y, Phi = _f64(Y), _f64(Phi)
    rows, n = Y.shape[0], Phi.shape[1]
    X = np.zeros((rows, n))
    picks = np.zeros((rows, int(k)), dtype=np.int64)
    margins = np.zeros((rows, int(k)))
    for i in range(rows):
        y = Y[i]
        r = y.copy()
        sel = []
        coef = np.zeros(0)
        for t in range(int(k)):
            c = np.abs(Phi.T @ r)
            c[sel] = -1.0                       # a column is picked at most once
            j = int(np.argmax(c))               # first index attaining the maximum
            runner = np.partition(c, -2)[-2] if n > 1 else 0.0
            margins[i, t] = (c[j] - max(runner, 0.0)) / c[j] if c[j] > 0 else 0.0
            sel.append(j)
            coef, *_ = np.linalg.lstsq(Phi[:, sel], y, rcond=None)
            r = y - Phi[:, sel] @ coef
        X[i, sel] = coef
        picks[i] = sel
    return X, picks, margins


def lasso_objective(Y, Phi, X, lam):
    """1/2 ||y - Phi x||_2^2 + lambda ||x||_1 per row."""
    Y, Phi, X = _f64(Y), _f64(Phi), _f64(X)
    R = Y - X @ Phi.T
    return 0.5 * (R * R).sum(axis=-1) + lam * np.abs(X).sum(axis=-1)


def support(X):
    """Boolean mask of the non-zero coordinates."""
    return np.asarray(X) != 0


def synthesize(X, V):
    """C^ = X V: X [..., n_q, n] codes over the keys, V [..., n, d]."""
    return _f64(X) @ _f64(V)


def forward(Q, K, V, Phi, lam, mu, iters, rows=None, Phi_K=None):
    """The whole CSAT block for Q [BH, n_q, d], K, V [BH, n, d], Phi [m, n].

    Phi_K: optional separate key matrix [m, n] (module header); Phi then is Phi_V and the decoder's matrix.

    rows: optional index array of query rows; when given, the decoder and the
    synthesis run on those rows only (rows are independent problems) and X, U, C
    have len(rows) rows per head.  iters == 0 skips the decoder: C = Z.
    Returns dict with Kc, Vc, A, Z, X, U (last pre-threshold values) and C.
    """
    Q, K, V, Phi = _f64(Q), _f64(K), _f64(V), _f64(Phi)
    Kc, Vc = measure(Phi, K, V, Phi_K)
    A, Z = compressed_attention(Q, Kc, Vc)
    out = {"Kc": Kc, "Vc": Vc, "A": A, "Z": Z}
    if iters == 0:
        out["C"] = Z if rows is None else Z[:, rows]
        return out
    BH = Q.shape[0]
    sel = np.arange(Q.shape[1]) if rows is None else np.asarray(rows)
    Xs, Us, Cs = [], [], []
    for h in range(BH):
        X, _, U = ista_trace(A[h][sel], Phi, lam, mu, iters)
        Xs.append(X)
        Us.append(U)
        Cs.append(synthesize(X, V[h]))
    out["X"], out["U"], out["C"] = np.stack(Xs), np.stack(Us), np.stack(Cs)
    return out


def forward_rd(Q, K, V, Phi, lam, mu, iters, cols=None, Phi_K=None):
    """Column-wise reading of the block (module header): Q, K, V [BH, n, d], Phi [m, n].
    Phi_K: optional separate key matrix; Phi then is Phi_V, which also forms Y and decodes it.

    Y = Phi Z per head; every feature column k of Y is decoded by ISTA into the column
    C[:, k] of the output.  cols: optional index array of feature columns to decode
    (columns are independent problems).  iters == 0 skips the decoder: C = Z.
    Returns dict with Kc, Vc, A, Z, Y [BH, m, d], X [BH, len(cols), n] (one decoded
    column per row), U (last pre-threshold values, same shape) and C [BH, n, len(cols)].
    """
    Q, K, V, Phi = _f64(Q), _f64(K), _f64(V), _f64(Phi)
    if Q.shape[1] != K.shape[1]:
        raise ValueError("the column-wise reading needs n_q == n")
    Kc, Vc = measure(Phi, K, V, Phi_K)
    A, Z = compressed_attention(Q, Kc, Vc)
    sel = np.arange(Q.shape[2]) if cols is None else np.asarray(cols)
    out = {"Kc": Kc, "Vc": Vc, "A": A, "Z": Z, "Y": Phi @ Z}
    if iters == 0:
        out["C"] = Z[:, :, sel]
        return out
    Xs, Us = [], []
    for h in range(Q.shape[0]):
        X, _, U = ista_trace(out["Y"][h][:, sel].T, Phi, lam, mu, iters)     # rows = feature columns
        Xs.append(X)
        Us.append(U)
    out["X"], out["U"] = np.stack(Xs), np.stack(Us)
    out["C"] = np.swapaxes(out["X"], 1, 2)
    return out
