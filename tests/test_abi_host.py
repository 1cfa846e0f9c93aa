"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2507_02957_amd as csat
from oracle import csat_oracle as orc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(csat.LIB_PATH):
        from paper_2507_02957_amd import build
        build.build()
    return csat.load_library()


def _declared():
    text = open(os.path.join(ROOT, "include", "csat.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(csat_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = _declared()
    assert set(names) == set(csat.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_status_strings(lib):
    for code in range(0, -9, -1):
        s = lib.csat_status_string(code)
        assert s and s != b"unknown status"
    assert lib.csat_status_string(-99) == b"unknown status"


def test_workspace_query_and_dim_checks(lib):
    d = csat.make_dims(4, 12, 1600, 1600, 64, 392, "bf16")
    nbytes = csat.csat_workspace_bytes(d, 20)
    rows = 4 * 12 * 1600
    assert nbytes >= rows * 1600 * 6                     # fp32 state + bf16 operand copy at least
    assert csat.csat_workspace_bytes(csat.make_dims(4, 12, 1600, 1600, 64, 392, "f32"), 20) < nbytes + rows * 1600 * 4
    bad = [
        (csat.make_dims(0, 1, 8, 8, 8, 4, "f32"), -2),
        (csat.make_dims(1, 1, 8, 8, 8, 9, "f32"), -2),     # m > n
        (csat.make_dims(1, 1, 8, 8, 12, 4, "f32"), -2),    # d not a multiple of 8
        (csat.csat_dims(1, 1, 8, 8, 8, 4, 7), -3),         # unknown dtype
    ]
    for dims, code in bad:
        with pytest.raises(csat.CsatError) as e:
            csat.csat_workspace_bytes(dims, 1)
        assert e.value.status == code
    with pytest.raises(csat.CsatError) as e:
        csat.csat_workspace_bytes(d, -1)
    assert e.value.status == -6
    assert csat.csat_workspace_bytes(csat.make_dims(1, 1, 8, 8, 8, 8, "f32"), 0) > 0     # m == n is legal


def test_argument_validation_without_device(lib):
    """Bad arguments are refused on the host; the fake pointers below are never dereferenced."""
    ctx = csat.context()
    d = csat.make_dims(1, 1, 16, 32, 8, 8, "f32")
    need = csat.csat_workspace_bytes(d, 3)
    P = ctypes.c_void_p(0x1000)            # aligned, non-NULL, never touched
    odd = ctypes.c_void_p(0x1004)
    rd = ctypes.byref(d)
    f = lib.csat_forward
    assert f(None, rd, P, P, P, P, 0.1, 0.5, 3, P, None, None, P, need, None) == -1
    assert f(ctx, None, P, P, P, P, 0.1, 0.5, 3, P, None, None, P, need, None) == -1
    assert f(ctx, rd, None, P, P, P, 0.1, 0.5, 3, P, None, None, P, need, None) == -1
    assert f(ctx, rd, P, P, P, P, 0.1, 0.5, 3, None, None, None, P, need, None) == -1
    assert f(ctx, rd, P, P, P, P, -0.1, 0.5, 3, P, None, None, P, need, None) == -6
    assert f(ctx, rd, P, P, P, P, 0.1, 0.0, 3, P, None, None, P, need, None) == -6
    assert f(ctx, rd, P, P, P, P, 0.1, float("nan"), 3, P, None, None, P, need, None) == -6
    assert f(ctx, rd, P, P, P, P, 0.1, 0.5, -1, P, None, None, P, need, None) == -6
    assert f(ctx, rd, odd, P, P, P, 0.1, 0.5, 3, P, None, None, P, need, None) == -4
    assert f(ctx, rd, P, P, P, P, 0.1, 0.5, 3, P, None, None, None, need, None) == -5
    assert f(ctx, rd, P, P, P, P, 0.1, 0.5, 3, P, None, None, P, need - 1, None) == -5
    r = lib.csat_recover
    assert r(ctx, rd, P, P, 0.1, 0.5, 3, None, None, None, P, need, None) == -1          # nothing requested
    assert r(ctx, rd, P, P, 0.1, 0.5, 3, None, P, None, P, need, None) == -1             # V without C
    assert r(ctx, rd, None, P, 0.1, 0.5, 3, P, None, None, P, need, None) == -1
    assert r(ctx, rd, P, P, 0.1, -1.0, 3, P, None, None, P, need, None) == -6
    m_ = lib.csat_measure
    assert m_(ctx, rd, P, P, None, P, P, P, need, None) == -1
    assert m_(ctx, rd, P, P, P, P, P, P, 16, None) == -5
    a = lib.csat_compressed_attention
    assert a(ctx, rd, P, P, P, None, None, P, need, None) == -1                          # Z is required
    assert a(ctx, rd, P, odd, P, None, P, P, need, None) == -4
    bad = csat.make_dims(1, 1, 16, 32, 8, 64, "f32")
    assert f(ctx, ctypes.byref(bad), P, P, P, P, 0.1, 0.5, 3, P, None, None, P, need, None) == -2
    # the unrolled decoder: host-side threshold array, own workspace query
    need_l = csat.csat_lista_workspace_bytes(d, 3)
    assert need_l > need
    th = (ctypes.c_float * 3)(0.1, 0.1, 0.1)
    bad_th = (ctypes.c_float * 3)(0.1, -0.1, 0.1)
    nan_th = (ctypes.c_float * 3)(0.1, float("nan"), 0.1)
    l = lib.csat_recover_lista
    assert l(ctx, rd, None, P, P, th, 3, P, None, None, P, need_l, None) == -1
    assert l(ctx, rd, P, None, P, th, 3, P, None, None, P, need_l, None) == -1
    assert l(ctx, rd, P, P, P, None, 3, P, None, None, P, need_l, None) == -1
    assert l(ctx, rd, P, P, P, th, 3, None, None, None, P, need_l, None) == -1           # nothing requested
    assert l(ctx, rd, P, P, P, bad_th, 3, P, None, None, P, need_l, None) == -6
    assert l(ctx, rd, P, P, P, nan_th, 3, P, None, None, P, need_l, None) == -6
    assert l(ctx, rd, P, P, P, th, -1, P, None, None, P, need_l, None) == -6
    assert l(ctx, rd, P, odd, P, th, 3, P, None, None, P, need_l, None) == -4
    assert l(ctx, rd, P, P, P, th, 3, P, None, None, P, need, None) == -5                # the ISTA workspace is too small
    # matching pursuit: number of picks 0 .. min(32, m), m <= 1024
    need_o = csat.csat_omp_workspace_bytes(d, 4)
    assert need_o > need
    o = lib.csat_recover_omp
    assert o(ctx, rd, None, P, 4, P, None, None, None, P, need_o, None) == -1
    assert o(ctx, rd, P, P, 4, None, None, None, None, P, need_o, None) == -1            # nothing requested
    assert o(ctx, rd, P, P, -1, P, None, None, None, P, need_o, None) == -6
    assert o(ctx, rd, P, P, 9, P, None, None, None, P, need_o, None) == -6               # more picks than measurements
    assert o(ctx, rd, P, P, 4, P, odd, None, None, P, need_o, None) == -4
    assert o(ctx, rd, P, P, 4, P, None, None, None, P, need, None) == -5
    with pytest.raises(csat.CsatError) as e:
        csat.csat_omp_workspace_bytes(csat.make_dims(1, 1, 8, 64, 8, 40, "f32"), 33)
    assert e.value.status == -6
    with pytest.raises(csat.CsatError) as e:
        csat.csat_omp_workspace_bytes(csat.make_dims(1, 1, 8, 2048, 8, 1032, "f32"), 4)
    assert e.value.status == -2
    # transform-based decoder
    hd = lib.csat_recover_hadamard
    assert hd(ctx, rd, P, None, P, 0.1, 0.5, 3, P, None, None, P, need, None) == -1
    assert hd(ctx, rd, P, P, None, 0.1, 0.5, 3, P, None, None, P, need, None) == -1
    assert hd(ctx, rd, P, P, P, 0.1, 0.5, 3, None, None, None, P, need, None) == -1
    assert hd(ctx, rd, P, P, P, 0.1, 0.0, 3, P, None, None, P, need, None) == -6
    assert hd(ctx, rd, P, P, P, 0.1, 0.5, 3, P, None, None, P, need - 1, None) == -5
    wide_m = csat.make_dims(1, 1, 8, 16384, 8, 13000, "f32")       # measurements of a row would not fit LDS
    assert hd(ctx, ctypes.byref(wide_m), P, P, P, 0.1, 0.5, 3, P, None, None, P, 1 << 44, None) == -2
    long_n = csat.make_dims(1, 1, 8, 20000, 8, 8, "f32")
    assert hd(ctx, ctypes.byref(long_n), P, P, P, 0.1, 0.5, 3, P, None, None, P, 1 << 40, None) == -2
    fh = lib.csat_forward_hadamard
    assert fh(ctx, rd, P, P, P, None, P, 0.1, 0.5, 3, P, None, None, P, need, None) == -1
    assert fh(ctx, rd, P, P, P, P, P, 0.1, 0.5, 3, None, None, None, P, need, None) == -1
    assert fh(ctx, rd, P, P, P, P, P, 0.1, 0.0, 3, P, None, None, P, need, None) == -6
    assert fh(ctx, rd, P, P, odd, P, P, 0.1, 0.5, 3, P, None, None, P, need, None) == -4
    assert fh(ctx, rd, P, P, P, P, P, 0.1, 0.5, 3, P, None, None, P, need - 1, None) == -5
    assert fh(ctx, ctypes.byref(long_n), P, P, P, P, P, 0.1, 0.5, 3, P, None, None, P, 1 << 44, None) == -2
    # a row's buffers would not fit LDS: refused by the entry point, before the measurement could write anything
    assert fh(ctx, ctypes.byref(wide_m), P, P, P, P, P, 0.1, 0.5, 3, P, None, None, P, 1 << 44, None) == -2
    wide_sq = csat.make_dims(1, 1, 16384, 16384, 8, 13000, "f32")
    assert lib.csat_forward_rd_hadamard(ctx, ctypes.byref(wide_sq), P, P, P, P, P, 0.1, 0.5, 3, P, None, P, 1 << 46, None) == -2
    mh = lib.csat_measure_hadamard
    assert mh(ctx, rd, None, P, P, P, P, P, None) == -1
    assert mh(ctx, rd, P, P, P, P, None, P, None) == -1
    assert mh(ctx, rd, P, P, odd, P, P, P, None) == -4
    assert mh(ctx, ctypes.byref(long_n), P, P, P, P, P, P, None) == -2
    many_heads = csat.make_dims(300, 300, 8, 64, 8, 8, "f32")
    assert mh(ctx, ctypes.byref(many_heads), P, P, P, P, P, P, None) == -2
    # the column-wise forward: self-attention shapes only, and its workspace is the larger one
    frd = lib.csat_forward_rd
    assert frd(ctx, rd, P, P, P, P, 0.1, 0.5, 3, P, None, P, need, None) == -2            # n_q != n
    ds = csat.make_dims(1, 1, 32, 32, 8, 8, "f32")
    need_s = csat.csat_workspace_bytes(ds, 3)
    assert need_s > csat.csat_workspace_bytes(csat.make_dims(1, 1, 31, 32, 8, 8, "f32"), 3)
    rs = ctypes.byref(ds)
    assert frd(ctx, rs, P, P, P, P, 0.1, 0.5, 3, None, None, P, need_s, None) == -1
    assert frd(ctx, rs, P, P, P, P, 0.1, -0.5, 3, P, None, P, need_s, None) == -6
    assert frd(ctx, rs, P, P, P, odd, 0.1, 0.5, 3, P, None, P, need_s, None) == -4
    assert frd(ctx, rs, P, P, P, P, 0.1, 0.5, 3, P, None, P, need_s - 1, None) == -5
    assert frd(ctx, rs, P, P, P, P, 0.1, 0.5, 3, P, None, None, need_s, None) == -5
    rh = lib.csat_forward_rd_hadamard
    assert rh(ctx, rd, P, P, P, P, P, 0.1, 0.5, 3, P, None, P, need, None) == -2             # n_q != n
    assert rh(ctx, rs, P, P, P, None, P, 0.1, 0.5, 3, P, None, P, need_s, None) == -1
    assert rh(ctx, rs, P, P, P, P, P, 0.1, 0.5, -1, P, None, P, need_s, None) == -6
    assert rh(ctx, rs, P, P, P, P, P, 0.1, 0.5, 3, P, None, P, need_s - 1, None) == -5
    # the calls with the key and the value matrix given separately
    mk, fk, rk = lib.csat_measure_kv, lib.csat_forward_kv, lib.csat_forward_rd_kv
    assert mk(ctx, rs, None, P, P, P, P, P, P, need_s, None) == -1
    assert mk(ctx, rs, P, None, P, P, P, P, P, need_s, None) == -1
    assert mk(ctx, rs, odd, P, P, P, P, P, P, need_s, None) == -4
    assert mk(ctx, rs, P, P, P, P, P, P, P, 256, None) == -5
    assert fk(ctx, rs, P, P, P, None, P, 0.1, 0.5, 3, P, None, None, P, need_s, None) == -1
    assert fk(ctx, rs, P, P, P, P, None, 0.1, 0.5, 3, P, None, None, P, need_s, None) == -1
    assert fk(ctx, rs, P, P, P, odd, P, 0.1, 0.5, 3, P, None, None, P, need_s, None) == -4
    assert fk(ctx, rs, P, P, P, P, P, -0.1, 0.5, 3, P, None, None, P, need_s, None) == -6
    assert fk(ctx, rs, P, P, P, P, P, 0.1, 0.5, 3, P, None, None, P, 256, None) == -5
    assert rk(ctx, rd, P, P, P, P, P, 0.1, 0.5, 3, P, None, P, need, None) == -2
    assert rk(ctx, rs, P, P, P, None, P, 0.1, 0.5, 3, P, None, P, need_s, None) == -1
    assert rk(ctx, rs, P, P, P, odd, P, 0.1, 0.5, 3, P, None, P, need_s, None) == -4
    assert rk(ctx, rs, P, P, P, P, P, 0.1, 0.5, 3, P, None, P, need_s - 1, None) == -5
    # reference kernels of the benchmark
    fl = ctypes.c_double()
    assert lib.csat_peak_copy(ctx, None, P, 4096, None) == -1
    assert lib.csat_peak_copy(ctx, P, P, 0, None) == -2
    assert lib.csat_peak_copy(ctx, P, P, 4100, None) == -2
    assert lib.csat_peak_copy(ctx, odd, P, 4096, None) == -4
    assert lib.csat_peak_mfma(ctx, None, 1 << 20, 10, ctypes.byref(fl), None) == -1
    assert lib.csat_peak_mfma(ctx, P, 1 << 20, 10, None, None) == -1
    assert lib.csat_peak_mfma(ctx, P, 1 << 20, 0, ctypes.byref(fl), None) == -6
    assert lib.csat_peak_mfma_issue(ctx, None, 1 << 20, 10, 3, 0, ctypes.byref(fl), None) == -1
    assert lib.csat_peak_mfma_issue(ctx, P, 1 << 20, 10, 3, 0, None, None) == -1
    assert lib.csat_peak_mfma_issue(ctx, P, 1 << 20, 0, 3, 0, ctypes.byref(fl), None) == -6
    assert lib.csat_peak_mfma_issue(ctx, ctypes.c_void_p(0x1004), 1 << 20, 10, 3, 0, ctypes.byref(fl), None) == -4


def test_context_lifecycle(lib):
    c = ctypes.c_void_p()
    assert lib.csat_create(ctypes.byref(c)) == 0 and c.value
    assert lib.csat_destroy(c) == 0
    assert lib.csat_create(None) == -1
    assert lib.csat_destroy(None) == -1


def test_opnorm_helper_matches_oracle(lib):
    """The library's own power iteration (host, double) against the oracle's eigenvalue routine."""
    import csat_inputs as gen
    for kind, m, n in (("gaussian", 64, 256), ("rademacher", 48, 300), ("gaussian", 96, 274)):
        Phi = gen.quantize(gen.make_phi(kind, m, n), "f32")
        got = csat.csat_phi_opnorm2(Phi)
        assert got == pytest.approx(orc.phi_opnorm_sq(Phi), rel=1e-9)
    assert csat.csat_phi_opnorm2(np.eye(5, dtype=np.float32)) == pytest.approx(1.0, rel=1e-12)
    # the largest workload's shape (m = 1024, n = 16384): the Gram matrix is formed on several host threads
    import time
    Phi = gen.quantize(gen.make_phi("gaussian", 1024, 16384), "bf16")
    t0 = time.perf_counter()
    got = csat.csat_phi_opnorm2(Phi)
    dt = time.perf_counter() - t0
    assert got == pytest.approx(orc.phi_opnorm_sq(Phi), rel=1e-9)
    print(f"csat_phi_opnorm2 at 1024 x 16384: {dt:.1f} s")


def test_options_and_decoder_status_arguments(lib):
    ctx = csat.context()
    assert lib.csat_set_option(None, 0, 1) == -1
    assert lib.csat_set_option(ctx, -1, 1) == -6
    assert lib.csat_set_option(ctx, len(csat.OPTIONS), 1) == -6          # one past the last key
    for key in csat.OPTIONS.values():
        assert lib.csat_set_option(ctx, key, 0) == 0
    # the workspace size does not depend on the options
    d = csat.make_dims(2, 3, 150, 203, 64, 75, "bf16")
    base = csat.csat_workspace_bytes(d, 5)
    for key, value in (("decoder", 1), ("gemm", 1), ("state", 2), ("fused_thin", 1)):
        csat.csat_set_option(key, value)
        assert csat.csat_workspace_bytes(d, 5) == base
        csat.csat_set_option(key, 0)
    assert lib.csat_decoder_status(None, ctypes.c_void_p(0x1000), None) == -1
    assert lib.csat_decoder_status(ctx, ctypes.c_void_p(0x1004), None) == -4
    k = ctypes.c_int(7)
    assert lib.csat_profile_decoder_kernel(None, ctypes.byref(k)) == -1
    assert lib.csat_profile_decoder_kernel(ctx, None) == -1
    assert lib.csat_profile_decoder_kernel(ctx, ctypes.byref(k)) == 0 and -1 <= k.value <= 4
    n = ctypes.c_size_t()
    assert lib.csat_static_workspace_bytes(None) == -1
    assert lib.csat_static_workspace_bytes(ctypes.byref(n)) == 0 and n.value == 48 << 20
    s = lib.csat_forward_static
    P = ctypes.c_void_p(0x1000)
    small = csat.make_dims(1, 1, 16, 32, 8, 8, "f32")
    rs = ctypes.byref(small)
    assert s(None, rs, P, P, P, P, 0.1, 0.5, 3, P, None, None, None) == -1
    assert s(ctx, rs, P, P, P, None, 0.1, 0.5, 3, P, None, None, None) == -1
    assert s(ctx, rs, P, P, P, P, 0.1, 0.5, -1, P, None, None, None) == -6
    assert s(ctx, rs, P, P, ctypes.c_void_p(0x1004), P, 0.1, 0.5, 3, P, None, None, None) == -4
    big = csat.make_dims(4, 12, 1600, 1600, 64, 392, "bf16")
    assert s(ctx, ctypes.byref(big), P, P, P, P, 0.1, 0.5, 3, P, None, None, None) == -5     # beyond the static array


def test_phi_fill_matches_the_oracles_generator(lib):
    """csat_phi_fill (host helper) against the oracle's own implementation of the same counter-based draw: the
    Rademacher matrix bit for bit, the Gaussian one to the last bits of the host's log and cosine; error codes."""
    for seed, m, n in ((0, 5, 7), (11, 64, 300), (2 ** 63 + 5, 3, 1000)):
        R = csat.csat_phi_fill("rademacher", seed, m, n)
        np.testing.assert_array_equal(R, orc.phi_fill("rademacher", seed, m, n))
        G, want = csat.csat_phi_fill("gaussian", seed, m, n), orc.phi_fill("gaussian", seed, m, n)
        assert G.dtype == np.float32 and G.shape == (m, n)
        assert np.abs(G.astype(np.float64) - want).max() <= 1e-6 * np.abs(want).max()
        assert (G == want).mean() > 0.99          # (a rare last-bit difference of log or cos may flip the float rounding)
    out = np.zeros((2, 2), dtype=np.float32)
    assert lib.csat_phi_fill(7, 0, 2, 2, out.ctypes.data) == -6 and not out.any()        # CSAT_ERR_PARAM
    assert lib.csat_phi_fill(0, 0, 0, 2, out.ctypes.data) == -2                          # CSAT_ERR_SHAPE
    assert lib.csat_phi_fill(0, 0, 2, 2, None) == -1                                       # CSAT_ERR_NULL
