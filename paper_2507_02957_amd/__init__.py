"""Python binding of libcsat: the CSAT forward pass as hand-written HIP kernels for MI355X.

Argument marshalling only: every function takes torch tensors that already live on the GPU
(torch is used for device memory and streams, nothing else), checks nothing the C library
does not check itself, and forwards raw device pointers through ctypes.  Function names and
argument order are those of include/csat.h.  There is no CPU fallback: if the shared library
is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libcsat.so")

CSAT_F32, CSAT_BF16 = 0, 1

EXPORTS = (
    "csat_create", "csat_destroy", "csat_status_string", "csat_workspace_bytes", "csat_phi_opnorm2", "csat_phi_fill",
    "csat_measure", "csat_compressed_attention", "csat_recover", "csat_forward", "csat_forward_rd",
    "csat_lista_workspace_bytes", "csat_recover_lista", "csat_omp_workspace_bytes", "csat_recover_omp",
    "csat_recover_hadamard", "csat_measure_hadamard", "csat_forward_hadamard", "csat_forward_rd_hadamard", "csat_measure_kv", "csat_forward_kv", "csat_forward_rd_kv",
    "csat_peak_copy", "csat_peak_mfma", "csat_peak_mfma_issue", "csat_profile_enable", "csat_profile_read", "csat_profile_decoder_kernel",
    "csat_set_option", "csat_decoder_status", "csat_static_workspace_bytes", "csat_forward_static",
)
# keys of csat_set_option (include/csat.h, csat_option)
OPTIONS = {"decoder": 0, "gemm": 1, "raster": 2, "state": 3, "fused_segments": 4, "fused_thin": 5, "lista": 6,
           "hadamard": 7, "fused_spin_limit": 8, "inject_decoder_error": 9, "attention": 10, "fused_schedule": 11,
           "measure": 12, "synthesis": 13, "y_layout": 14}
CSAT_ERR_TIMEOUT = -8
KERNEL_IDS = {"layout": 0, "measure": 1, "scores": 2, "softmax": 3, "output": 4, "residual": 5, "update": 6,
              "synthesis": 7}


class csat_dims(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int), ("H", ctypes.c_int), ("n_q", ctypes.c_int), ("n", ctypes.c_int),
                ("d", ctypes.c_int), ("m", ctypes.c_int), ("dtype", ctypes.c_int)]


class CsatError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"csat status {status}: {message}")
        self.status = status


_lib = None
_ctx = None


def load_library() -> ctypes.CDLL:
    """Loads libcsat.so (built beforehand by paper_2507_02957_amd.build); raises if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} not found: build it first (python -m paper_2507_02957_amd.build); there is no fallback path")
    lib = ctypes.CDLL(LIB_PATH)
    vp, sz, fl, it = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_float, ctypes.c_int
    dp = ctypes.POINTER(csat_dims)
    lib.csat_create.argtypes = [ctypes.POINTER(vp)]
    lib.csat_destroy.argtypes = [vp]
    lib.csat_status_string.argtypes = [it]
    lib.csat_status_string.restype = ctypes.c_char_p
    lib.csat_workspace_bytes.argtypes = [dp, it, ctypes.POINTER(sz)]
    lib.csat_phi_opnorm2.argtypes = [vp, it, it, ctypes.POINTER(ctypes.c_double)]
    lib.csat_phi_fill.argtypes = [it, ctypes.c_ulonglong, it, it, vp]
    lib.csat_measure.argtypes = [vp, dp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.csat_compressed_attention.argtypes = [vp, dp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.csat_recover.argtypes = [vp, dp, vp, vp, fl, fl, it, vp, vp, vp, vp, sz, vp]
    lib.csat_forward.argtypes = [vp, dp, vp, vp, vp, vp, fl, fl, it, vp, vp, vp, vp, sz, vp]
    lib.csat_forward_rd.argtypes = [vp, dp, vp, vp, vp, vp, fl, fl, it, vp, vp, vp, sz, vp]
    lib.csat_measure_kv.argtypes = [vp, dp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.csat_forward_kv.argtypes = [vp, dp, vp, vp, vp, vp, vp, fl, fl, it, vp, vp, vp, vp, sz, vp]
    lib.csat_forward_rd_kv.argtypes = [vp, dp, vp, vp, vp, vp, vp, fl, fl, it, vp, vp, vp, sz, vp]
    lib.csat_lista_workspace_bytes.argtypes = [dp, it, ctypes.POINTER(sz)]
    lib.csat_recover_lista.argtypes = [vp, dp, vp, vp, vp, ctypes.POINTER(fl), it, vp, vp, vp, vp, sz, vp]
    lib.csat_omp_workspace_bytes.argtypes = [dp, it, ctypes.POINTER(sz)]
    lib.csat_recover_omp.argtypes = [vp, dp, vp, vp, it, vp, vp, vp, vp, vp, sz, vp]
    lib.csat_recover_hadamard.argtypes = [vp, dp, vp, vp, vp, fl, fl, it, vp, vp, vp, vp, sz, vp]
    lib.csat_peak_copy.argtypes = [vp, vp, vp, sz, vp]
    lib.csat_peak_mfma.argtypes = [vp, vp, sz, it, ctypes.POINTER(ctypes.c_double), vp]
    lib.csat_peak_mfma_issue.argtypes = [vp, vp, sz, it, it, it, ctypes.POINTER(ctypes.c_double), vp]
    lib.csat_measure_hadamard.argtypes = [vp, dp, vp, vp, vp, vp, vp, vp, vp]
    lib.csat_forward_rd_hadamard.argtypes = [vp, dp, vp, vp, vp, vp, vp, fl, fl, it, vp, vp, vp, sz, vp]
    lib.csat_forward_hadamard.argtypes = [vp, dp, vp, vp, vp, vp, vp, fl, fl, it, vp, vp, vp, vp, sz, vp]
    lib.csat_set_option.argtypes = [vp, it, it]
    lib.csat_decoder_status.argtypes = [vp, vp, vp]
    lib.csat_static_workspace_bytes.argtypes = [ctypes.POINTER(sz)]
    lib.csat_forward_static.argtypes = [vp, dp, vp, vp, vp, vp, fl, fl, it, vp, vp, vp, vp]
    lib.csat_profile_enable.argtypes = [vp, it]
    lib.csat_profile_read.argtypes = [vp, it, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(it)]
    lib.csat_profile_decoder_kernel.argtypes = [vp, ctypes.POINTER(it)]
    for name in EXPORTS:
        if name != "csat_status_string":
            getattr(lib, name).restype = it
    _lib = lib
    return lib


def _check(status: int):
    if status != 0:
        raise CsatError(status, load_library().csat_status_string(status).decode())


def context() -> ctypes.c_void_p:
    global _ctx
    if _ctx is None:
        c = ctypes.c_void_p()
        _check(load_library().csat_create(ctypes.byref(c)))
        _ctx = c
    return _ctx


def make_dims(B, H, n_q, n, d, m, dtype) -> csat_dims:
    """dtype: CSAT_F32 / CSAT_BF16, "f32" / "bf16", or a torch dtype."""
    code = {"f32": CSAT_F32, "bf16": CSAT_BF16, CSAT_F32: CSAT_F32, CSAT_BF16: CSAT_BF16}.get(dtype)
    if code is None:
        import torch
        code = {torch.float32: CSAT_F32, torch.bfloat16: CSAT_BF16}[dtype]
    return csat_dims(B, H, n_q, n, d, m, code)


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def csat_workspace_bytes(dims: csat_dims, iters: int) -> int:
    out = ctypes.c_size_t()
    _check(load_library().csat_workspace_bytes(ctypes.byref(dims), iters, ctypes.byref(out)))
    return out.value


def csat_phi_opnorm2(phi_host) -> float:
    """phi_host: contiguous float32 CPU tensor or numpy array [m, n].  Returns ||Phi||_2^2."""
    if hasattr(phi_host, "data_ptr"):
        m, n = phi_host.shape
        ptr = phi_host.data_ptr()
    else:
        m, n = phi_host.shape
        ptr = phi_host.ctypes.data
    out = ctypes.c_double()
    _check(load_library().csat_phi_opnorm2(ctypes.c_void_p(ptr), m, n, ctypes.byref(out)))
    return out.value


def csat_phi_fill(kind: str, seed: int, m: int, n: int):
    """Measurement matrix [m, n] (numpy float32, host) of the "gaussian" or "rademacher" ensemble from `seed`."""
    import numpy as np
    out = np.empty((m, n), dtype=np.float32)
    code = {"gaussian": 0, "rademacher": 1}[kind]
    _check(load_library().csat_phi_fill(code, ctypes.c_ulonglong(seed & 0xFFFFFFFFFFFFFFFF), m, n,
                                        ctypes.c_void_p(out.ctypes.data)))
    return out


def alloc_workspace(dims: csat_dims, iters: int, device="cuda:0"):
    import torch
    return torch.empty(csat_workspace_bytes(dims, iters), dtype=torch.uint8, device=device)


def csat_measure(dims, Phi, K, V, Kc, Vc, workspace, stream=None):
    _check(load_library().csat_measure(context(), ctypes.byref(dims), _ptr(Phi), _ptr(K), _ptr(V), _ptr(Kc), _ptr(Vc),
                                       _ptr(workspace), workspace.numel(), _stream(stream)))


def csat_compressed_attention(dims, Q, Kc, Vc, A, Z, workspace, stream=None):
    _check(load_library().csat_compressed_attention(context(), ctypes.byref(dims), _ptr(Q), _ptr(Kc), _ptr(Vc),
                                                    _ptr(A), _ptr(Z), _ptr(workspace), workspace.numel(),
                                                    _stream(stream)))


def csat_recover(dims, Y, Phi, lam, step, iters, X, V, C, workspace, stream=None):
    _check(load_library().csat_recover(context(), ctypes.byref(dims), _ptr(Y), _ptr(Phi), lam, step, iters,
                                       _ptr(X), _ptr(V), _ptr(C), _ptr(workspace), workspace.numel(),
                                       _stream(stream)))


def csat_forward(dims, Q, K, V, Phi, lam, step, iters, C, Z, X, workspace, stream=None):
    _check(load_library().csat_forward(context(), ctypes.byref(dims), _ptr(Q), _ptr(K), _ptr(V), _ptr(Phi),
                                       lam, step, iters, _ptr(C), _ptr(Z), _ptr(X), _ptr(workspace),
                                       workspace.numel(), _stream(stream)))


def csat_forward_rd(dims, Q, K, V, Phi, lam, step, iters, C, Z, workspace, stream=None):
    _check(load_library().csat_forward_rd(context(), ctypes.byref(dims), _ptr(Q), _ptr(K), _ptr(V), _ptr(Phi),
                                          lam, step, iters, _ptr(C), _ptr(Z), _ptr(workspace),
                                          workspace.numel(), _stream(stream)))


def csat_measure_kv(dims, PhiK, PhiV, K, V, Kc, Vc, workspace, stream=None):
    _check(load_library().csat_measure_kv(context(), ctypes.byref(dims), _ptr(PhiK), _ptr(PhiV), _ptr(K), _ptr(V),
                                          _ptr(Kc), _ptr(Vc), _ptr(workspace), workspace.numel(), _stream(stream)))


def csat_forward_kv(dims, Q, K, V, PhiK, PhiV, lam, step, iters, C, Z, X, workspace, stream=None):
    _check(load_library().csat_forward_kv(context(), ctypes.byref(dims), _ptr(Q), _ptr(K), _ptr(V), _ptr(PhiK),
                                          _ptr(PhiV), lam, step, iters, _ptr(C), _ptr(Z), _ptr(X), _ptr(workspace),
                                          workspace.numel(), _stream(stream)))


def csat_forward_rd_kv(dims, Q, K, V, PhiK, PhiV, lam, step, iters, C, Z, workspace, stream=None):
    _check(load_library().csat_forward_rd_kv(context(), ctypes.byref(dims), _ptr(Q), _ptr(K), _ptr(V), _ptr(PhiK),
                                             _ptr(PhiV), lam, step, iters, _ptr(C), _ptr(Z), _ptr(workspace),
                                             workspace.numel(), _stream(stream)))


def csat_peak_copy(src, dst, stream=None):
    """One streaming copy src -> dst (same-size device tensors); returns the bytes moved through HBM."""
    nbytes = src.numel() * src.element_size()
    _check(load_library().csat_peak_copy(context(), _ptr(src), _ptr(dst), nbytes, _stream(stream)))
    return 2 * nbytes


def csat_peak_mfma(out, iters, stream=None) -> float:
    """Launches the register-resident MFMA loop; returns the launch's floating-point operation count."""
    flops = ctypes.c_double()
    _check(load_library().csat_peak_mfma(context(), _ptr(out), out.numel() * out.element_size(), iters,
                                         ctypes.byref(flops), _stream(stream)))
    return flops.value


def csat_peak_mfma_issue(out, iters, valu_per_mfma, lds_reads_per_mfma, stream=None) -> float:
    """Launches the one-wavefront-per-SIMD loop of MFMA + other instructions; returns its floating-point operation count."""
    flops = ctypes.c_double()
    _check(load_library().csat_peak_mfma_issue(context(), _ptr(out), out.numel() * out.element_size(), iters,
                                               valu_per_mfma, lds_reads_per_mfma, ctypes.byref(flops), _stream(stream)))
    return flops.value


def csat_measure_hadamard(dims, rows_of_h, signs, K, V, Kc, Vc, stream=None):
    _check(load_library().csat_measure_hadamard(context(), ctypes.byref(dims), _ptr(rows_of_h), _ptr(signs), _ptr(K),
                                                _ptr(V), _ptr(Kc), _ptr(Vc), _stream(stream)))


def csat_forward_hadamard(dims, Q, K, V, rows_of_h, signs, lam, step, iters, C, Z, X, workspace, stream=None):
    _check(load_library().csat_forward_hadamard(context(), ctypes.byref(dims), _ptr(Q), _ptr(K), _ptr(V), _ptr(rows_of_h),
                                                _ptr(signs), lam, step, iters, _ptr(C), _ptr(Z), _ptr(X), _ptr(workspace),
                                                workspace.numel(), _stream(stream)))


def csat_forward_rd_hadamard(dims, Q, K, V, rows_of_h, signs, lam, step, iters, C, Z, workspace, stream=None):
    _check(load_library().csat_forward_rd_hadamard(context(), ctypes.byref(dims), _ptr(Q), _ptr(K), _ptr(V),
                                                   _ptr(rows_of_h), _ptr(signs), lam, step, iters, _ptr(C), _ptr(Z),
                                                   _ptr(workspace), workspace.numel(), _stream(stream)))


def csat_lista_workspace_bytes(dims: csat_dims, iters: int) -> int:
    out = ctypes.c_size_t()
    _check(load_library().csat_lista_workspace_bytes(ctypes.byref(dims), iters, ctypes.byref(out)))
    return out.value


def csat_recover_lista(dims, Y, S, Bw, thetas, X, V, C, workspace, stream=None):
    """thetas: a sequence of per-layer thresholds (host floats); its length is the number of layers."""
    th = (ctypes.c_float * max(len(thetas), 1))(*[float(t) for t in thetas])
    _check(load_library().csat_recover_lista(context(), ctypes.byref(dims), _ptr(Y), _ptr(S), _ptr(Bw), th, len(thetas),
                                             _ptr(X), _ptr(V), _ptr(C), _ptr(workspace), workspace.numel(),
                                             _stream(stream)))


def csat_omp_workspace_bytes(dims: csat_dims, k: int) -> int:
    out = ctypes.c_size_t()
    _check(load_library().csat_omp_workspace_bytes(ctypes.byref(dims), k, ctypes.byref(out)))
    return out.value


def csat_recover_omp(dims, Y, Phi, k, X, picks, V, C, workspace, stream=None):
    _check(load_library().csat_recover_omp(context(), ctypes.byref(dims), _ptr(Y), _ptr(Phi), k, _ptr(X), _ptr(picks),
                                           _ptr(V), _ptr(C), _ptr(workspace), workspace.numel(), _stream(stream)))


def csat_recover_hadamard(dims, Y, rows_of_h, signs, lam, step, iters, X, V, C, workspace, stream=None):
    """rows_of_h: int32 device tensor [m]; signs: int8 device tensor [N] of +-1."""
    _check(load_library().csat_recover_hadamard(context(), ctypes.byref(dims), _ptr(Y), _ptr(rows_of_h), _ptr(signs),
                                                lam, step, iters, _ptr(X), _ptr(V), _ptr(C), _ptr(workspace),
                                                workspace.numel(), _stream(stream)))


def csat_set_option(key, value: int):
    """key: a name from OPTIONS or the integer key; value 0 restores the library's own choice."""
    _check(load_library().csat_set_option(context(), OPTIONS.get(key, key), int(value)))


def csat_decoder_status(workspace, stream=None) -> int:
    """Waits for the stream; 0 if the ISTA decoder of the last call on `workspace` ran to the end, CSAT_ERR_TIMEOUT
    (-8) if it gave up (then that call's X and C hold NaN).  workspace None: the scratch of csat_forward_static."""
    st = load_library().csat_decoder_status(context(), _ptr(workspace), _stream(stream))
    if st not in (0, CSAT_ERR_TIMEOUT):
        _check(st)
    return st


def csat_static_workspace_bytes() -> int:
    out = ctypes.c_size_t()
    _check(load_library().csat_static_workspace_bytes(ctypes.byref(out)))
    return out.value


def csat_forward_static(dims, Q, K, V, Phi, lam, step, iters, C, Z, X, stream=None):
    """csat_forward on the library's static scratch (no workspace argument, nothing allocated)."""
    _check(load_library().csat_forward_static(context(), ctypes.byref(dims), _ptr(Q), _ptr(K), _ptr(V), _ptr(Phi),
                                              lam, step, iters, _ptr(C), _ptr(Z), _ptr(X), _stream(stream)))


def csat_profile_enable(on: bool):
    _check(load_library().csat_profile_enable(context(), int(bool(on))))


def csat_profile_decoder_kernel() -> int:
    """Which kernel the last ISTA decoder call launched (include/csat.h: -1 not the fused decoder, 0-2 one chunk per
    step, 3-4 two chunks per step)."""
    k = ctypes.c_int()
    _check(load_library().csat_profile_decoder_kernel(context(), ctypes.byref(k)))
    return k.value


def csat_profile_read(kernel: str):
    """(total milliseconds, launches) recorded for one step since profiling was enabled."""
    ms, cnt = ctypes.c_double(), ctypes.c_int()
    _check(load_library().csat_profile_read(context(), KERNEL_IDS[kernel], ctypes.byref(ms), ctypes.byref(cnt)))
    return ms.value, cnt.value
