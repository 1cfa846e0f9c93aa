"""Helpers for the GPU parity tests: move seeded inputs to the device, call the HIP path through
the C ABI binding, and compare with the fp64 oracle under the stated tolerances."""
import numpy as np
import torch

import csat_inputs as gen
import paper_2507_02957_amd as csat

DEV = "cuda:0"
TOL = {"f32": 1e-4, "bf16": 2e-2}   # relative tolerances of the HIP path vs the fp64 oracle


def to_dev(a: np.ndarray, dtype: str):
    """float32 numpy (already rounded to `dtype`) -> device tensor of that element type."""
    if dtype == "bf16":
        return torch.from_numpy(gen.bf16_bits(a)).view(torch.bfloat16).to(DEV)
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(DEV)


def to_np(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def tdtype(dtype: str):
    return torch.bfloat16 if dtype == "bf16" else torch.float32


def assert_close(name, got, want, tol, slices_axis0=True):
    """Per leading-axis slice: ||G-O||_F <= tol ||O||_F and max|G-O| <= tol max|O|."""
    got, want = np.asarray(got, dtype=np.float64), np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, f"{name}: shape {got.shape} vs {want.shape}"
    assert np.isfinite(got).all(), f"{name}: non-finite values"
    G = got.reshape(got.shape[0], -1) if slices_axis0 else got.reshape(1, -1)
    O = want.reshape(G.shape)
    fro = np.linalg.norm(G - O, axis=1) / np.maximum(np.linalg.norm(O, axis=1), 1e-300)
    mx = np.abs(G - O).max(axis=1) / np.maximum(np.abs(O).max(axis=1), 1e-300)
    worst = max(fro.max(), mx.max())
    assert worst <= tol, f"{name}: rel fro {fro.max():.3e}, rel max {mx.max():.3e} > {tol}"
    return worst


# Above this ratio ||U||_F / ||X||_F of the last pre-threshold values to the iterate, the iterate is what is left
# of a cancellation (x = u - theta with nearly all of u's energy below the threshold) and its relative error says
# little about the arithmetic that produced u.
ILL_CONDITIONED_RATIO = 10.0


def assert_close_iterate(name, got, want, U, tol, scale_by_ratio_of=None):
    """Tolerance for a thresholded iterate X = eta(U) (or for C = X V, given scale_by_ratio_of=(X, U)).

    The stated tolerance is applied as for every other tensor (one slice).  Only a case that misses it AND that
    the oracle itself shows to be ill-conditioned, ||U||_F > ILL_CONDITIONED_RATIO * ||X||_F, gets the second check.  The soft threshold is 1-Lipschitz, so an
    error in U (what the products compute) passes to X unamplified in absolute terms; when the threshold then
    removes nearly all of U's energy, the same absolute error is a large relative one.  Such a case is held to
    the tolerance on U's scale instead: ||G - O||_F <= tol ||U||_F and max|G - O| <= tol max|U| (for C, the
    allowance tol is scaled by ||U||_F / ||X||_F), and the departure from the plain norm is printed."""
    got, want, U = (np.asarray(a, dtype=np.float64) for a in (got, want, U))
    assert got.shape == want.shape, f"{name}: shape {got.shape} vs {want.shape}"
    assert np.isfinite(got).all(), f"{name}: non-finite values"
    Xref = want if scale_by_ratio_of is None else np.asarray(scale_by_ratio_of[0], dtype=np.float64)
    fro_plain = np.linalg.norm(got - want) / max(np.linalg.norm(want), 1e-300)
    max_plain = np.abs(got - want).max() / max(np.abs(want).max(), 1e-300)
    if max(fro_plain, max_plain) <= tol:
        return max(fro_plain, max_plain)
    ratio = np.linalg.norm(U) / max(np.linalg.norm(Xref), 1e-300)
    assert np.linalg.norm(Xref) > 0 and ratio > ILL_CONDITIONED_RATIO, \
        f"{name}: rel fro {fro_plain:.3e}, rel max {max_plain:.3e} > {tol} (||U||/||X|| = {ratio:.1f}: well-conditioned)"
    if scale_by_ratio_of is None:
        fro = np.linalg.norm(got - want) / np.linalg.norm(U)
        mx = np.abs(got - want).max() / np.abs(U).max()
    else:
        fro, mx = fro_plain / ratio, max_plain / ratio
    print(f"{name}: ill-conditioned case (||U||/||X|| = {ratio:.1f}): plain norm rel fro {fro_plain:.3e}, rel max "
          f"{max_plain:.3e}; on U's scale rel fro {fro:.3e}, rel max {mx:.3e} (tolerance {tol})")
    assert max(fro, mx) <= tol, f"{name}: on U's scale rel fro {fro:.3e}, rel max {mx:.3e} > {tol}"
    return max(fro, mx)


class DeviceProblem:
    """Inputs of one workload on the device plus a workspace sized by the library."""

    def __init__(self, w: gen.Workload, Q, K, V, Phi):
        self.w = w
        BH = Q.shape[0]
        self.BH = BH
        # the flattened batch*head axis is passed as B = BH, H = 1 when the arrays hold a head subset
        self.dims = csat.make_dims(BH, 1, w.n_q, w.n, w.d, w.m, w.dtype)
        self.Q, self.K, self.V, self.Phi = (to_dev(a, w.dtype) for a in (Q, K, V, Phi))
        self.ws = csat.alloc_workspace(self.dims, w.iters)
        self.t = tdtype(w.dtype)

    def empty(self, *shape, dtype=None):
        return torch.empty(*shape, dtype=dtype or self.t, device=DEV)

    def measure(self):
        w = self.w
        Kc, Vc = self.empty(self.BH, w.m, w.d), self.empty(self.BH, w.m, w.d)
        csat.csat_measure(self.dims, self.Phi, self.K, self.V, Kc, Vc, self.ws)
        return Kc, Vc

    def attention(self, Kc, Vc):
        w = self.w
        A = self.empty(self.BH, w.n_q, w.m, dtype=torch.float32)
        Z = self.empty(self.BH, w.n_q, w.d)
        csat.csat_compressed_attention(self.dims, self.Q, Kc, Vc, A, Z, self.ws)
        return A, Z

    def recover(self, Y, lam, mu, iters, want_x=True, want_c=True):
        w = self.w
        X = self.empty(self.BH, w.n_q, w.n, dtype=torch.float32) if want_x else None
        C = self.empty(self.BH, w.n_q, w.d) if want_c else None
        csat.csat_recover(self.dims, Y, self.Phi, lam, mu, iters, X, self.V if want_c else None, C, self.ws)
        return X, C

    def forward(self, lam, mu, iters, want_z=True, want_x=True):
        w = self.w
        C = self.empty(self.BH, w.n_q, w.d)
        Z = self.empty(self.BH, w.n_q, w.d) if want_z else None
        X = self.empty(self.BH, w.n_q, w.n, dtype=torch.float32) if want_x else None
        csat.csat_forward(self.dims, self.Q, self.K, self.V, self.Phi, lam, mu, iters, C, Z, X, self.ws)
        torch.cuda.synchronize()
        return C, Z, X

    def forward_rd(self, lam, mu, iters, want_z=True):
        w = self.w
        C = self.empty(self.BH, w.n, w.d)
        Z = self.empty(self.BH, w.n, w.d) if want_z else None
        csat.csat_forward_rd(self.dims, self.Q, self.K, self.V, self.Phi, lam, mu, iters, C, Z, self.ws)
        torch.cuda.synchronize()
        return C, Z

    def recover_lista(self, Y, S, Bw, thetas, want_x=True, want_c=True):
        """S, Bw: numpy arrays (already rounded to the workload's dtype)."""
        w = self.w
        ws = torch.empty(csat.csat_lista_workspace_bytes(self.dims, len(thetas)), dtype=torch.uint8, device=DEV)
        X = self.empty(self.BH, w.n_q, w.n, dtype=torch.float32) if want_x else None
        C = self.empty(self.BH, w.n_q, w.d) if want_c else None
        csat.csat_recover_lista(self.dims, Y, to_dev(S, w.dtype), to_dev(Bw, w.dtype), thetas, X,
                                self.V if want_c else None, C, ws)
        torch.cuda.synchronize()
        return X, C

    def recover_omp(self, Y, k, want_x=True, want_picks=True, want_c=True):
        w = self.w
        ws = torch.empty(csat.csat_omp_workspace_bytes(self.dims, k), dtype=torch.uint8, device=DEV)
        X = self.empty(self.BH, w.n_q, w.n, dtype=torch.float32) if want_x else None
        P = self.empty(self.BH, w.n_q, max(k, 1), dtype=torch.int32) if want_picks else None
        C = self.empty(self.BH, w.n_q, w.d) if want_c else None
        csat.csat_recover_omp(self.dims, Y, self.Phi, k, X, P, self.V if want_c else None, C, ws)
        torch.cuda.synchronize()
        return X, P, C

    def measure_hadamard(self, rows_of_h, signs):
        w = self.w
        Kc, Vc = self.empty(self.BH, w.m, w.d), self.empty(self.BH, w.m, w.d)
        csat.csat_measure_hadamard(self.dims, torch.from_numpy(rows_of_h).to(DEV), torch.from_numpy(signs).to(DEV),
                                   self.K, self.V, Kc, Vc)
        torch.cuda.synchronize()
        return Kc, Vc

    def forward_hadamard(self, rows_of_h, signs, lam, mu, iters, want_z=True, want_x=True):
        w = self.w
        C = self.empty(self.BH, w.n_q, w.d)
        Z = self.empty(self.BH, w.n_q, w.d) if want_z else None
        X = self.empty(self.BH, w.n_q, w.n, dtype=torch.float32) if want_x else None
        csat.csat_forward_hadamard(self.dims, self.Q, self.K, self.V, torch.from_numpy(rows_of_h).to(DEV),
                                   torch.from_numpy(signs).to(DEV), lam, mu, iters, C, Z, X, self.ws)
        torch.cuda.synchronize()
        return C, Z, X

    def forward_rd_hadamard(self, rows_of_h, signs, lam, mu, iters, want_z=True):
        w = self.w
        C = self.empty(self.BH, w.n, w.d)
        Z = self.empty(self.BH, w.n, w.d) if want_z else None
        csat.csat_forward_rd_hadamard(self.dims, self.Q, self.K, self.V, torch.from_numpy(rows_of_h).to(DEV),
                                      torch.from_numpy(signs).to(DEV), lam, mu, iters, C, Z, self.ws)
        torch.cuda.synchronize()
        return C, Z

    def recover_hadamard(self, Y, rows_of_h, signs, lam, mu, iters, want_x=True, want_c=True):
        w = self.w
        X = self.empty(self.BH, w.n_q, w.n, dtype=torch.float32) if want_x else None
        C = self.empty(self.BH, w.n_q, w.d) if want_c else None
        csat.csat_recover_hadamard(self.dims, Y, torch.from_numpy(rows_of_h).to(DEV), torch.from_numpy(signs).to(DEV),
                                   lam, mu, iters, X, self.V if want_c else None, C, self.ws)
        torch.cuda.synchronize()
        return X, C
