"""csat_forward_static, the entry point that allocates nothing (the workspace is a static array in the
library's own device memory): same outputs as csat_forward with a caller-allocated workspace, bit for bit
(same kernels, same carving), on two calls in a row, the second with a smaller input."""
import numpy as np
import pytest
import torch

import csat_inputs as gen
import paper_2507_02957_amd as csat
from oracle import csat_oracle as orc
from tests.gpu_harness import DEV, TOL, DeviceProblem, assert_close, to_np

pytestmark = pytest.mark.gpu


def _case(name, **kw):
    base = dict(name=name, B=1, H=1, n_q=64, n=64, d=64, m=32, dtype="f32", phi_kind="gaussian", iters=5,
                lam=0.05, structure="iid", seed=31)
    base.update(kw)
    return gen.Workload(**base)


def _both(w):
    """One problem through csat_forward (caller's workspace) and through csat_forward_static."""
    Q, K, V = gen.make_qkv(w)
    Phi = gen.make_workload_phi(w)
    mu = float(np.float32(1.0 / orc.phi_opnorm_sq(Phi)))
    p = DeviceProblem(w, Q, K, V, Phi)
    C0, Z0, X0 = p.forward(w.lam, mu, w.iters)
    assert csat.csat_decoder_status(p.ws) == 0
    C, Z = torch.full_like(C0, float("nan")), torch.full_like(Z0, float("nan"))
    X = torch.full_like(X0, float("nan"))
    csat.csat_forward_static(p.dims, p.Q, p.K, p.V, p.Phi, w.lam, mu, w.iters, C, Z, X)
    torch.cuda.synchronize()
    assert csat.csat_decoder_status(None) == 0
    ref = orc.forward(Q, K, V, Phi, w.lam, mu, w.iters)
    return (C0, Z0, X0), (C, Z, X), ref, p, mu


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_static_scratch_forward_matches_workspace_forward(dtype):
    first = _case("static_a_" + dtype, B=2, H=3, n_q=150, n=203, d=64, m=75, dtype=dtype, iters=7)
    second = _case("static_b_" + dtype, B=1, H=2, n_q=40, n=65, d=64, m=33, dtype=dtype, iters=4, seed=32)   # smaller
    for w in (first, second):
        (C0, Z0, X0), (C, Z, X), ref, p, mu = _both(w)
        assert torch.equal(C, C0) and torch.equal(Z, Z0) and torch.equal(X, X0), w.name
        tol = TOL[w.dtype]
        assert_close("Z", to_np(Z), ref["Z"], tol)
        assert_close("X", to_np(X), ref["X"], tol)
        assert_close("C", to_np(C), ref["C"], tol)
    # optional outputs left out, and no decoder iterations (C = Z)
    w = second
    (C0, _, _), _, _, p, mu = _both(w)
    C1 = torch.empty_like(C0)
    csat.csat_forward_static(p.dims, p.Q, p.K, p.V, p.Phi, w.lam, mu, w.iters, C1, None, None)
    torch.cuda.synchronize()
    assert torch.equal(C1, C0)
    Cz, Zz = torch.empty_like(C0), torch.empty_like(C0)
    csat.csat_forward_static(p.dims, p.Q, p.K, p.V, p.Phi, w.lam, mu, 0, Cz, Zz, None)
    torch.cuda.synchronize()
    assert torch.equal(Cz, Zz)


def test_static_scratch_limit_and_arguments():
    """A problem whose carving exceeds the static array is refused before anything is launched."""
    limit = csat.csat_static_workspace_bytes()
    assert limit == 48 << 20
    w = gen.WORKLOADS["short_video"]
    dims = csat.make_dims(w.B, w.H, w.n_q, w.n, w.d, w.m, w.dtype)
    assert csat.csat_workspace_bytes(dims, w.iters) > limit
    t = torch.zeros(16, device=DEV)
    with pytest.raises(csat.CsatError) as e:
        csat.csat_forward_static(dims, t, t, t, t, 0.1, 0.5, 3, t, None, None)
    assert e.value.status == -5
    small = csat.make_dims(1, 1, 8, 16, 8, 4, "f32")
    with pytest.raises(csat.CsatError) as e:
        csat.csat_forward_static(small, t, t, t, t, 0.1, 0.0, 3, t, None, None)
    assert e.value.status == -6
    with pytest.raises(csat.CsatError) as e:
        csat.csat_forward_static(small, t, None, t, t, 0.1, 0.5, 3, t, None, None)
    assert e.value.status == -1
