"""Seeded synthetic inputs for the CSAT forward path.

This module only *draws numbers*: it holds none of the method's arithmetic
(no projection, no softmax, no thresholding, no step size), so both the CPU
oracle's tests and the HIP path's tests/benchmark may feed from it without
sharing any computation.  Every tensor comes from a counter-based Philox
stream keyed by (master seed, tensor id), so a tensor's values do not depend
on the order in which tensors are requested.

The five workloads are synthetic stand-ins for the *shapes* of the
vision-language workloads the paper evaluates on (ViT-B/16 patch tokens plus
text tokens, short and long video token streams, text-to-video
cross-attention); none of the paper's datasets is reproduced.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

# tensor ids used to key the Philox streams
_TID_Q, _TID_K, _TID_V, _TID_PHI, _TID_PLANTED, _TID_HADAMARD = 1, 2, 3, 4, 5, 6


@dataclass(frozen=True)
class Workload:
    """One benchmark configuration (shapes, measurement ensemble, decoder settings)."""

    name: str
    B: int
    H: int
    n_q: int
    n: int
    d: int
    m: int
    dtype: str          # "f32" or "bf16": element type of Q, K, V, Phi
    phi_kind: str       # "gaussian" (N(0, 1/m)) or "rademacher" (+-1/sqrt(m))
    iters: int          # ISTA iterations T
    lam: float          # l1 weight lambda
    structure: str      # "iid" | "lowrank_image_text" | "frame_drift" | "cross_frame_drift"
    frames: int = 0     # number of video frames (frame_drift structures)
    patches: int = 0    # patch tokens per frame / image rows
    seed: int = 0       # master seed for Q, K, V (Phi always uses seed 0)


WORKLOADS = {
    "tiny": Workload("tiny", 1, 1, 256, 256, 64, 64, "f32", "gaussian", 10, 0.1, "iid", seed=1),
    "image_text": Workload("image_text", 8, 12, 274, 274, 64, 96, "bf16", "gaussian", 20, 0.05,
                           "lowrank_image_text", patches=197, seed=2),
    "short_video": Workload("short_video", 4, 12, 1600, 1600, 64, 392, "bf16", "gaussian", 20, 0.05,
                            "frame_drift", frames=8, patches=196, seed=3),
    "cross_modal": Workload("cross_modal", 16, 16, 77, 4096, 64, 512, "bf16", "rademacher", 30, 0.02,
                            "cross_frame_drift", frames=16, patches=256, seed=4),
    "long_video": Workload("long_video", 1, 16, 16384, 16384, 128, 1024, "bf16", "gaussian", 50, 0.02,
                           "frame_drift", frames=64, patches=256, seed=5),
}


def _rng(seed: int, tensor_id: int, sub: int = 0) -> np.random.Generator:
    """Philox generator whose 128-bit key is (seed, tensor id, sub-stream)."""
    key = (int(seed) & 0xFFFFFFFF) | ((int(tensor_id) & 0xFFFF) << 32) | ((int(sub) & 0xFFFF) << 48)
    return np.random.Generator(np.random.Philox(key=key))


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float values to the nearest bfloat16 (ties to even); result is float32
    holding exactly representable bf16 values."""
    a = np.ascontiguousarray(x, dtype=np.float32)
    bits = a.view(np.uint32).astype(np.uint64)
    lsb = (bits >> 16) & 1
    rounded = ((bits + 0x7FFF + lsb) >> 16) << 16
    return rounded.astype(np.uint32).view(np.float32).reshape(a.shape)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """Upper 16 bits (as int16) of float32 values that are already bf16-representable."""
    a = np.ascontiguousarray(x, dtype=np.float32)
    return (a.view(np.uint32) >> 16).astype(np.uint16).view(np.int16).reshape(a.shape)


def quantize(x: np.ndarray, dtype: str) -> np.ndarray:
    """Values as the device will see them: float32 (for "f32") or bf16-rounded float32."""
    if dtype == "f32":
        return np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "bf16":
        return round_to_bf16(x)
    raise ValueError(f"unknown dtype {dtype!r}")


def make_phi(kind: str, m: int, n: int, seed: int = 0) -> np.ndarray:
    """Measurement matrix draw, float64 [m, n].

    gaussian:   i.i.d. N(0, 1/m) entries.
    rademacher: i.i.d. +-1/sqrt(m) entries with equal probability.
    identity:   eye(n) (requires m == n); the degenerate case with no compression.
    """
    g = _rng(seed, _TID_PHI)
    if kind == "gaussian":
        return g.standard_normal((m, n)) / np.sqrt(m)
    if kind == "rademacher":
        signs = g.integers(0, 2, size=(m, n), dtype=np.int8).astype(np.float64) * 2.0 - 1.0
        return signs / np.sqrt(m)
    if kind == "identity":
        if m != n:
            raise ValueError("identity measurement needs m == n")
        return np.eye(n)
    raise ValueError(f"unknown measurement ensemble {kind!r}")


def make_hadamard_phi(m: int, n: int, seed: int = 0):
    """Structured measurement ensemble: m rows of the Walsh-Hadamard matrix of order N (the smallest
    power of two >= n, natural ordering: H[i, j] = (-1)^popcount(i & j)), columns flipped by random
    signs, the first n columns kept, scaled by 1/sqrt(m).
    Returns (Phi float64 [m, n], rows int32 [m] sorted ascending, signs int8 [N] of +-1)."""
    g = _rng(seed, _TID_HADAMARD)
    N = 1
    while N < n:
        N *= 2
    rows = np.sort(g.choice(N, size=m, replace=False)).astype(np.int32)
    signs = (g.integers(0, 2, size=N, dtype=np.int8) * 2 - 1).astype(np.int8)
    i = rows[:, None].astype(np.int64)
    j = np.arange(n, dtype=np.int64)[None, :]
    parity = np.zeros((m, n), dtype=np.int64)
    v = i & j
    while v.any():
        parity ^= v & 1
        v >>= 1
    H = 1.0 - 2.0 * parity
    return H * signs[None, :n].astype(np.float64) / np.sqrt(m), rows, signs


def _iid(g: np.random.Generator, BH: int, rows: int, d: int) -> np.ndarray:
    return g.standard_normal((BH, rows, d), dtype=np.float32)


def _lowrank_image_text(g, BH, n, d, patches, rank=16, noise=0.1):
    """First `patches` rows: rank-`rank` factor model U W + noise*E; remaining rows i.i.d. N(0,1)."""
    out = np.empty((BH, n, d), dtype=np.float32)
    U = g.standard_normal((BH, patches, rank), dtype=np.float32)
    W = g.standard_normal((BH, rank, d), dtype=np.float32) / np.float32(np.sqrt(rank))
    E = g.standard_normal((BH, patches, d), dtype=np.float32)
    out[:, :patches] = np.matmul(U, W) + np.float32(noise) * E
    out[:, patches:] = g.standard_normal((BH, n - patches, d), dtype=np.float32)
    return out


def _frame_drift(g, BH, n, d, frames, patches, drift=0.05):
    """`frames` copies of one base frame, each with its own N(0, drift^2) perturbation
    (independent per frame, not a random walk); trailing rows are i.i.d. N(0,1) text tokens."""
    out = np.empty((BH, n, d), dtype=np.float32)
    base = g.standard_normal((BH, 1, patches, d), dtype=np.float32)
    vid = frames * patches
    for f in range(frames):
        out[:, f * patches:(f + 1) * patches] = (
            base[:, 0] + np.float32(drift) * g.standard_normal((BH, patches, d), dtype=np.float32))
    if n > vid:
        out[:, vid:] = g.standard_normal((BH, n - vid, d), dtype=np.float32)
    return out


def make_qkv(w: Workload, heads: slice | None = None):
    """Q [BH, n_q, d], K [BH, n, d], V [BH, n, d] as float32 arrays already rounded to the
    workload's element type.  `heads` (a slice over the flattened batch*head axis) returns
    only those slices, with the same values they have in the full tensors."""
    BH = w.B * w.H
    outs = []
    for tid, rows in ((_TID_Q, w.n_q), (_TID_K, w.n), (_TID_V, w.n)):
        g = _rng(w.seed, tid)
        if w.structure == "iid":
            t = _iid(g, BH, rows, w.d)
        elif w.structure == "lowrank_image_text":
            t = _lowrank_image_text(g, BH, rows, w.d, w.patches)
        elif w.structure == "frame_drift":
            t = _frame_drift(g, BH, rows, w.d, w.frames, w.patches)
        elif w.structure == "cross_frame_drift":
            t = _iid(g, BH, rows, w.d) if tid == _TID_Q else _frame_drift(g, BH, rows, w.d, w.frames, w.patches)
        else:
            raise ValueError(w.structure)
        t = quantize(t, w.dtype)
        outs.append(t if heads is None else np.ascontiguousarray(t[heads]))
    return tuple(outs)


def make_workload_phi(w: Workload) -> np.ndarray:
    """The workload's measurement matrix, float32 [m, n], rounded to the workload's element type."""
    return quantize(make_phi(w.phi_kind, w.m, w.n, seed=0), w.dtype)


def scaled(w: Workload, **kw) -> Workload:
    """Copy of a workload with some fields replaced (e.g. fewer batches for a CPU-sized case)."""
    from dataclasses import replace
    return replace(w, **kw)


def planted_sparse(seed: int, m: int, n: int, k: int, rows: int = 1, min_mag: float = 1.0,
                   kind: str = "gaussian"):
    """Noise-free planted problems: Phi [m, n]; X* [rows, n] with exactly k non-zeros per row,
    magnitudes in [min_mag, 2*min_mag] and random signs; supports [rows, k] sorted.
    (The measurements Phi X*^T are left to the caller: that product is the method's, not ours.)"""
    g = _rng(seed, _TID_PLANTED)
    if kind == "gaussian":
        Phi = g.standard_normal((m, n)) / np.sqrt(m)
    else:
        Phi = (g.integers(0, 2, size=(m, n)).astype(np.float64) * 2.0 - 1.0) / np.sqrt(m)
    X = np.zeros((rows, n))
    supports = np.empty((rows, k), dtype=np.int64)
    for r in range(rows):
        sup = np.sort(g.choice(n, size=k, replace=False))
        mags = min_mag * (1.0 + g.random(k))
        sgn = g.integers(0, 2, size=k) * 2.0 - 1.0
        X[r, sup] = mags * sgn
        supports[r] = sup
    return Phi, X, supports
