#!/usr/bin/env python3
"""Benchmark of the CSAT forward pass (csat_forward through the C ABI) on one MI355X.

A step is one whole forward pass (measurement, compressed attention, ISTA recovery, synthesis)
over one batch of seeded synthetic inputs that are already resident in HBM.  Prints ONE JSON
line: nominal TFLOP/s (value), tokens/s, the roofline figures of the dominant kernel measured
with HIP events on the launch stream, and the fp64 CPU oracle timed on a bounded sample of the
same workload on this machine's host cores.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_PEAK_TFLOPS = {"bf16": 2500.0, "f32": 157.3}


def nominal_flops(w, mode="rows", picks=8):
    """Dense count of what the method as defined computes (first ISTA iteration has x = 0)."""
    import numpy as np
    BH = w.B * w.H
    front = 4.0 * w.m * w.n * w.d * BH + 4.0 * w.n_q * w.m * w.d * BH
    if mode == "columns":      # Y = Phi Z, then one decoder problem per feature column; no synthesis product
        return front + 2.0 * w.m * w.n * w.d * BH + (4.0 * w.iters - 2.0) * w.m * w.n * w.d * BH
    if mode == "columns_hadamard":      # the column-wise reading by transforms: B*H*d decoder problems, Y = Phi Z by d transforms per head
        N = 1
        while N < w.n:
            N *= 2
        return front + 2.0 * w.iters * N * np.log2(N) * w.d * BH
    if mode == "hadamard":     # two transforms of length N per row and iteration (one in the first), N log2 N additions each
        N = 1
        while N < w.n:
            N *= 2
        return front + (2.0 * w.iters - 1.0) * N * np.log2(N) * w.n_q * BH + 2.0 * w.n_q * w.n * w.d * BH
    if mode == "omp":          # one correlation product per pick (the per-row refits are lower order) and a sparse synthesis
        return front + picks * 2.0 * w.m * w.n * w.n_q * BH + 2.0 * picks * w.d * w.n_q * BH
    if mode == "lista":        # W = B y once, then (S - I) alpha per layer
        return front + (2.0 * w.m * w.n + 2.0 * w.iters * w.n * w.n) * w.n_q * BH + 2.0 * w.n_q * w.n * w.d * BH
    return front + (4.0 * w.iters - 2.0) * w.m * w.n * w.n_q * BH + 2.0 * w.n_q * w.n * w.d * BH


def cpu_baseline_columns(w, Q, K, V, Phi, mu, budget_s=20.0):
    """The fp64 oracle of the column-wise reading on a bounded sample of heads."""
    from oracle import csat_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    BH = w.B * w.H
    t0 = time.perf_counter()
    orc.forward_rd(Q[:1], K[:1], V[:1], Phi, w.lam, mu, w.iters)
    per_head = time.perf_counter() - t0
    heads = int(max(1, min(BH, budget_s / max(per_head, 1e-9))))
    t0 = time.perf_counter()
    orc.forward_rd(Q[:heads], K[:heads], V[:heads], Phi, w.lam, mu, w.iters)
    dt = time.perf_counter() - t0
    return {"value": heads * w.n_q / w.H / dt, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"{heads} of {BH} heads, all stages, all {w.d} feature columns, fp64 numpy, {dt:.1f} s",
            "tflops": nominal_flops(w, "columns") * heads / BH / dt / 1e12}


def cpu_baseline(w, Q, K, V, Phi, mu, budget_s=20.0):
    """The fp64 oracle, as it stands, on a bounded sample of heads of the same workload."""
    import numpy as np
    from oracle import csat_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    BH = w.B * w.H
    rows_all = np.arange(w.n_q)
    # calibrate on a slice of one head, then size the sample to the budget
    cal = rows_all[: max(1, min(w.n_q, 64))]
    t0 = time.perf_counter()
    orc.forward(Q[:1], K[:1], V[:1], Phi, w.lam, mu, w.iters, rows=cal)
    t_cal = time.perf_counter() - t0
    per_row = t_cal / len(cal)
    nrows = int(max(len(cal), min(w.n_q * BH, budget_s / max(per_row, 1e-9))))
    heads = max(1, min(BH, nrows // w.n_q)) if nrows >= w.n_q else 1
    rows = rows_all if nrows >= w.n_q else rows_all[:nrows]
    t0 = time.perf_counter()
    orc.forward(Q[:heads], K[:heads], V[:heads], Phi, w.lam, mu, w.iters, rows=rows)
    dt = time.perf_counter() - t0
    tokens = heads * len(rows) / w.H            # query tokens of one batch element span H heads
    return {"value": tokens / dt, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"{heads} of {BH} heads x {len(rows)} of {w.n_q} query rows, all stages, fp64 numpy, {dt:.1f} s",
            "tflops": nominal_flops(w) * (heads * len(rows)) / (BH * w.n_q) / dt / 1e12}


def cpu_baseline_other_decoder(w, Q, K, V, Phi, mu, mode, picks, budget_s=15.0):
    """The fp64 oracle of the unrolled decoder (analytic weights) or of matching pursuit on a bounded sample of
    query rows of the first head: measurement and compressed attention of that head, then the decoder and the
    synthesis on the sampled rows."""
    import numpy as np
    from oracle import csat_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    Phi64 = Phi.astype(np.float64)
    if mode == "lista":
        S, Bm = np.eye(w.n) - mu * Phi64.T @ Phi64, mu * Phi64.T
        thetas = [mu * w.lam] * w.iters

    def run(nrows):
        t0 = time.perf_counter()
        Kc, Vc = orc.measure(Phi, K[:1], V[:1])
        A, _ = orc.compressed_attention(Q[:1], Kc, Vc)
        Y = A[0][:nrows]
        X = orc.lista(Y, S, Bm, thetas)[0] if mode == "lista" else orc.omp(Y, Phi, picks)[0]
        orc.synthesize(X, V[0])
        return time.perf_counter() - t0

    cal = max(1, min(w.n_q, 8))
    t_cal = run(cal)
    nrows = int(max(cal, min(w.n_q, cal * budget_s / max(t_cal, 1e-9))))
    dt = run(nrows)
    return {"value": nrows / w.H / dt, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"1 of {w.B * w.H} heads x {nrows} of {w.n_q} query rows, all stages, fp64 numpy, {dt:.1f} s",
            "tflops": nominal_flops(w, mode, picks) * nrows / (w.B * w.H * w.n_q) / dt / 1e12}


def sweep(args):
    """The paper's scaling claim for the compressed block (stages measure + compressed attention): time
    against sequence length n at fixed m, and the same two stages with m = n (Phi square: nothing saved)."""
    import numpy as np
    import torch

    import csat_inputs as gen
    import paper_2507_02957_amd as csat
    dev = torch.device("cuda:0")
    B, H, d, m = 4, 12, 64, 256

    def run(n, mm):
        g = torch.Generator(device="cpu").manual_seed(n)
        t = lambda *shape: torch.randn(*shape, generator=g).to(torch.bfloat16).to(dev)
        Q, K, V = t(B, H, n, d), t(B, H, n, d), t(B, H, n, d)
        Phi = (torch.randn(mm, n, generator=g) / mm ** 0.5).to(torch.bfloat16).to(dev)
        dims = csat.make_dims(B, H, n, n, d, mm, "bf16")
        ws = csat.alloc_workspace(dims, 0)
        Kc = torch.empty(B, H, mm, d, dtype=torch.bfloat16, device=dev)
        Vc = torch.empty_like(Kc)
        Z = torch.empty(B, H, n, d, dtype=torch.bfloat16, device=dev)

        def step():
            csat.csat_measure(dims, Phi, K, V, Kc, Vc, ws)
            csat.csat_compressed_attention(dims, Q, Kc, Vc, None, Z, ws)
        for _ in range(args.warmup):
            step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / args.steps * 1e3

    rows = []
    for n in (512, 1024, 2048, 4096, 8192):
        ms = run(n, m)
        ms_full = run(n, n) if n <= 4096 else None
        rows.append({"n": n, "m": m, "ms": ms, "us_per_token": ms * 1e3 / (B * n), "ms_m_equals_n": ms_full})
    last = rows[-1]
    print(json.dumps({"metric": "compressed_block_tokens_per_s", "value": B * last["n"] / (last["ms"] / 1e3), "unit": "tokens/s",
                      "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": last["ms"],
                      "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
                      "config": {"workload": "sweep", "B": B, "H": H, "d": d, "m": m, "n": [r["n"] for r in rows]},
                      "sweep": rows}))


def measure_peaks(reps=10):
    """What this device delivers for the two roofs: a streaming copy (GB/s through HBM, reads + writes) and a
    register-resident bf16 MFMA loop with full-entropy operands (TFLOP/s)."""
    import torch

    import paper_2507_02957_amd as csat
    dev = torch.device("cuda:0")
    src = torch.zeros(1 << 31, dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    out = torch.empty(1 << 18, dtype=torch.float32, device=dev)

    def timed(fn):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            work = fn()
        e1.record()
        torch.cuda.synchronize()
        return work, e0.elapsed_time(e1) / reps

    moved, ms_copy = timed(lambda: csat.csat_peak_copy(src, dst))
    flops, ms_mfma = timed(lambda: csat.csat_peak_mfma(out, 20000))
    del src, dst, out
    return {"stream_copy_GBps": moved / ms_copy / 1e6, "stream_copy_ms": ms_copy,
            "mfma_loop_TFLOPps": flops / ms_mfma / 1e9, "mfma_loop_ms": ms_mfma}


ISSUE_CASES = ((0, 0), (3, 0), (6, 0), (9, 0), (12, 0), (0, 1), (3, 1), (6, 1), (0, 2))


def measure_issue(reps=5):
    """One wavefront per SIMD (the fused decoder's occupancy): nanoseconds per 32x32x16 bf16 MFMA with a number of
    independent fp32 fmas and 16-byte LDS reads issued behind each.  Shows how much else fits under an MFMA."""
    import torch

    import paper_2507_02957_amd as csat
    out = torch.empty(1 << 18, dtype=torch.float32, device=torch.device("cuda:0"))
    rows = []
    for kv, kl in ISSUE_CASES:
        csat.csat_peak_mfma_issue(out, 200, kv, kl)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            flops = csat.csat_peak_mfma_issue(out, 20000, kv, kl)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        rows.append({"valu_per_mfma": kv, "lds_reads_per_mfma": kl, "ns_per_mfma": ms * 1e6 / (20000 * 8),
                     "TFLOPps": flops / ms / 1e9})
    return rows


def peaks(args):
    pk = measure_peaks(max(args.steps, 1))
    pk["one_wavefront_per_simd_issue"] = measure_issue()
    print(json.dumps({"metric": "achievable_peaks", "value": pk["mfma_loop_TFLOPps"], "unit": "TFLOP/s", "n_gpus": 1,
                      "steps": args.steps, "warmup": 1, "ms_per_step": pk["mfma_loop_ms"], "higher_is_better": True,
                      "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
                      "config": {"workload": "peaks"}, "achievable": pk,
                      "frac_of_published": {"hbm_8TBps": pk["stream_copy_GBps"] / 8000.0,
                                            "bf16_mfma_2.5PFLOPps": pk["mfma_loop_TFLOPps"] / 2500.0}}))


def measure(args, workload, steps, warmup, with_peaks, with_cpu):
    """One workload, one decode mode: `warmup` untimed steps, `steps` timed ones, up to three more with every launch
    bracketed by HIP events (the dominant kernel's roofline figures), and the oracle leg when asked for."""
    import numpy as np
    import torch

    import csat_inputs as gen
    import paper_2507_02957_amd as csat
    w = gen.WORKLOADS[workload]
    if args.mode in ("columns", "columns_hadamard") and w.n_q != w.n:
        sys.exit("bench.py: --mode columns needs a self-attention workload (n_q == n)")
    dev = torch.device("cuda:0")
    Q, K, V = gen.make_qkv(w)
    if args.mode in ("hadamard", "columns_hadamard"):
        Phi64, h_rows, h_signs = gen.make_hadamard_phi(w.m, w.n, seed=0)
        Phi = gen.quantize(Phi64, w.dtype)
    else:
        Phi = gen.make_workload_phi(w)
    mu = float(np.float32(1.0 / csat.csat_phi_opnorm2(Phi)))     # the library's own step-size helper

    def dv(a):
        if w.dtype == "bf16":
            return torch.from_numpy(gen.bf16_bits(a)).view(torch.bfloat16).to(dev)
        return torch.from_numpy(a).to(dev)

    tQ, tK, tV, tPhi = dv(Q), dv(K), dv(V), dv(Phi)
    dims = csat.make_dims(w.B, w.H, w.n_q, w.n, w.d, w.m, w.dtype)
    ws = csat.alloc_workspace(dims, w.iters)
    C = torch.empty(w.B, w.H, w.n_q, w.d, dtype=tQ.dtype, device=dev)
    Zout = torch.empty_like(C)      # the compressed output Z = A~ V~ is requested too: a step runs every stage of the path

    if args.mode == "lista":
        Phi64 = gen.quantize(Phi, w.dtype).astype(np.float64)
        tS = dv((np.eye(w.n) - mu * Phi64.T @ Phi64).astype(np.float32))
        tB = dv((mu * Phi64.T).astype(np.float32))
        thetas = [mu * w.lam] * w.iters
        ws = torch.empty(csat.csat_lista_workspace_bytes(dims, w.iters), dtype=torch.uint8, device=dev)
        Kc = torch.empty(w.B, w.H, w.m, w.d, dtype=tQ.dtype, device=dev)
        Vc = torch.empty_like(Kc)
        A = torch.empty(w.B, w.H, w.n_q, w.m, dtype=torch.float32, device=dev)
        Zt = torch.empty(w.B, w.H, w.n_q, w.d, dtype=tQ.dtype, device=dev)

    if args.mode in ("hadamard", "columns_hadamard"):
        t_rows, t_signs = torch.from_numpy(h_rows).to(dev), torch.from_numpy(h_signs).to(dev)
        Kc = torch.empty(w.B, w.H, w.m, w.d, dtype=tQ.dtype, device=dev)
        Vc = torch.empty_like(Kc)
        A = torch.empty(w.B, w.H, w.n_q, w.m, dtype=torch.float32, device=dev)
        Zt = torch.empty(w.B, w.H, w.n_q, w.d, dtype=tQ.dtype, device=dev)
    if args.mode == "omp":
        ws = torch.empty(csat.csat_omp_workspace_bytes(dims, args.picks), dtype=torch.uint8, device=dev)
        Kc = torch.empty(w.B, w.H, w.m, w.d, dtype=tQ.dtype, device=dev)
        Vc = torch.empty_like(Kc)
        A = torch.empty(w.B, w.H, w.n_q, w.m, dtype=torch.float32, device=dev)
        Zt = torch.empty(w.B, w.H, w.n_q, w.d, dtype=tQ.dtype, device=dev)
        Pk = torch.empty(w.B, w.H, w.n_q, args.picks, dtype=torch.int32, device=dev)

    def step():
        if args.mode == "columns_hadamard":
            csat.csat_forward_rd_hadamard(dims, tQ, tK, tV, t_rows, t_signs, w.lam, mu, w.iters, C, None, ws)
        elif args.mode == "hadamard":
            csat.csat_forward_hadamard(dims, tQ, tK, tV, t_rows, t_signs, w.lam, mu, w.iters, C, Zout, None, ws)
        elif args.mode == "omp":
            csat.csat_measure(dims, tPhi, tK, tV, Kc, Vc, ws)
            csat.csat_compressed_attention(dims, tQ, Kc, Vc, A, Zt, ws)
            csat.csat_recover_omp(dims, A, tPhi, args.picks, None, Pk, tV, C, ws)
        elif args.mode == "lista":
            csat.csat_measure(dims, tPhi, tK, tV, Kc, Vc, ws)
            csat.csat_compressed_attention(dims, tQ, Kc, Vc, A, Zt, ws)
            csat.csat_recover_lista(dims, A, tS, tB, thetas, None, tV, C, ws)
        elif args.mode == "columns":
            csat.csat_forward_rd(dims, tQ, tK, tV, tPhi, w.lam, mu, w.iters, C, None, ws)
        else:
            csat.csat_forward(dims, tQ, tK, tV, tPhi, w.lam, mu, w.iters, C, Zout, None, ws)

    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    timed_step = step
    if args.graph:      # the step is stream-ordered launches only, so a replay is the same work
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step()
        graph.replay()
        torch.cuda.synchronize()
        timed_step = graph.replay
    t0 = time.perf_counter()
    for _ in range(steps):
        timed_step()
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / steps

    # per-kernel durations from HIP events on the launch stream (extra steps, same launches).  Two unbracketed steps
    # go in front, without a synchronisation in between, so that the bracketed ones run on a busy device like the
    # timed ones do: the first launch on an idle device takes about 8 % longer than the ones behind it.
    for _ in range(min(steps, 2)):
        step()
    csat.csat_profile_enable(True)
    prof_steps = min(steps, 5)
    for _ in range(prof_steps):
        step()
    torch.cuda.synchronize()
    prof = {k: csat.csat_profile_read(k) for k in csat.KERNEL_IDS}
    csat.csat_profile_enable(False)
    stage_ms = {k: v[0] / prof_steps for k, v in prof.items()}

    rows = w.B * w.H * (w.d if args.mode in ("columns", "columns_hadamard") else w.n_q)      # decoder problems
    T = w.iters
    fused = prof["residual"][1] == 0 and args.mode in ("rows", "columns")          # one launch runs every ISTA iteration
    hadamard = args.mode in ("hadamard", "columns_hadamard")
    if hadamard:
        dom, kname = "update", "ista_hadamard_kernel"
        N = 1
        while N < w.n:
            N *= 2
        flops_dom = (2.0 * T - 1.0) * N * np.log2(N) * rows
        bytes_dom = rows * (4.0 * w.m + 2.0 * w.n)       # y in, the bf16 iterate out: nothing else leaves the chip
    elif fused:
        dom, kname = "update", ("ista_fused2_kernel" if csat.csat_profile_decoder_kernel() >= 3 else "ista_fused_kernel")
        # per launch: all T iterations.  Algorithmic bytes: the fp32 iterate is written T-1 times and
        # read T-1 times (8n bytes per row and iteration), y is read once per iteration.
        flops_dom = (4.0 * T - 2.0) * w.m * w.n * rows
        bytes_dom = rows * ((T - 1) * 8.0 * w.n + T * 4.0 * w.m)
        if args.mode == "rows" and prof["synthesis"][1] == 0:      # the kernel also formed C = X V (no product kernel ran)
            flops_dom += 2.0 * rows * w.n * w.d
            bytes_dom += rows * 2.0 * w.d
    else:
        dom = max(("update", "residual"), key=lambda k: prof[k][0])
        big = w.dtype == "bf16" and rows >= 256      # the large-tile kernel takes the decoder's bf16 GEMM pair
        kname = (("gemm_nt_bf16_big_kernel<EpiIstaUpdateTiled>" if dom == "update" else "gemm_nt_bf16_big_kernel<EpiResidualTiled>")
                 if big else ("gemm_nt_kernel<EpiIstaUpdate>" if dom == "update" else "gemm_nt_kernel<EpiResidual>"))
        esz = 2.0 if w.dtype == "bf16" else 0.0      # bf16 operand copy next to the fp32 state
        if args.mode == "omp":                         # correlations R Phi: reads bf16 r, writes fp32 correlations
            dom = "update"
            kname = "gemm_nt_bf16_big_kernel<EpiStore<float>>" if big else "gemm_nt_kernel<EpiStore<float>>"
        if args.mode == "lista":                       # one layer: (S - I) alpha, K = n
            dom = "update"
            kname = "gemm_nt_bf16_big_kernel<EpiListaUpdateTiled>" if big else "gemm_nt_kernel<EpiListaUpdate>"
        flops_dom = 2.0 * rows * w.n * (w.n if args.mode == "lista" else w.m)
        bytes_dom = {"update": rows * ((4.0 * w.n + max(esz, 4.0) * w.m) if args.mode == "omp" else
                                       ((8.0 + esz) * w.n + (max(esz, 4.0) * w.m if args.mode != "lista" else (4.0 + esz) * w.n))),
                     "residual": rows * (max(esz, 4.0) * w.n + (4.0 + max(esz, 4.0)) * w.m)}[dom]
    ms_dom, n_dom = prof[dom]
    avg_s = ms_dom / max(n_dom, 1) / 1e3
    # HBM bytes per launch measured with rocprofv3 (FETCH_SIZE + WRITE_SIZE), if on record for this kernel
    traffic, traffic_src = None, None
    try:
        rec = json.load(open(os.path.join(ROOT, "profiles", "hbm_traffic.json"))).get(w.name)
        if rec and rec["kernel"] == kname and args.mode == "rows":
            traffic, traffic_src = rec["fetch_bytes"] + rec["write_bytes"], rec["summary"]
    except (OSError, ValueError, KeyError):
        pass
    # Which roof: the arithmetic intensity against the ridge, taken with the bytes the kernel really
    # moves when they are on record (the fused decoder with a sparse iterate moves far fewer than the
    # algorithmic figure, which assumes a dense iterate streamed every iteration), else the algorithmic ones.
    ai = flops_dom / bytes_dom
    ai_roof = flops_dom / traffic if traffic else ai
    ridge = MFMA_PEAK_TFLOPS[w.dtype] * 1e12 / (HBM_PEAK_GBS * 1e9)
    if hadamard:      # plain fp32 additions on the vector units: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz x 2 (fma peak) = 157.3 TFLOP/s
        roof = {"bound": "alu", "achieved": flops_dom / avg_s / 1e12, "peak": 157.3, "unit": "TFLOP/s",
                # butterflies are single additions (no fused multiply-add) and packed fp32 is compiled out on the test machines:
                # 256 CUs x 64 lanes x 2.4 GHz additions per second is what the vector units can do with them
                "addition_peak": 39.3, "frac_of_addition_peak": flops_dom / avg_s / 1e12 / 39.3}
    elif ai_roof < ridge:
        roof = {"bound": "hbm", "achieved": bytes_dom / avg_s / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s"}
    else:
        roof = {"bound": "mfma", "achieved": flops_dom / avg_s / 1e12, "peak": MFMA_PEAK_TFLOPS[w.dtype],
                "unit": "TFLOP/s"}
    roof["frac"] = roof["achieved"] / roof["peak"]
    roof["traffic"] = traffic
    if traffic_src:
        roof["traffic_source"] = traffic_src
    roof["algorithmic_bytes"] = bytes_dom
    roof["kernel"] = kname
    roof["avg_launch_us"] = avg_s * 1e6
    roof["launches_per_step"] = n_dom / prof_steps
    roof["arithmetic_intensity_flop_per_byte"] = ai
    roof["arithmetic_intensity_measured_traffic"] = ai_roof if traffic else None
    # Flops the dominant kernel executes per launch, padding included (nothing is skipped: the decoder is dense);
    # `achieved` counts only the algorithmic ones.  Fused decoder: every 32-row tile runs 2*MT MFMAs (32x32x16) per
    # chunk and product; large-tile GEMM: whole 256x256 tiles over K padded to 64.
    executed = None
    if fused and not hadamard:
        mt, nct = -(-w.m // 32), -(-w.n // 32)
        executed = (-(-rows // 128) * 4) * nct * (2.0 * T - 1.0) * (2 * mt) * 2.0 * 32 * 32 * 16
    elif kname.startswith("gemm_nt_bf16_big_kernel"):
        up = lambda v, q: -(-v // q) * q
        n_out, k_in = ((w.n, w.n) if args.mode == "lista" else (w.n, w.m)) if dom == "update" else (w.m, w.n)
        executed = 2.0 * up(rows, 256) * up(up(n_out, 64), 256) * up(k_in, 64)
    roof["executed_flops"] = executed
    roof["executed_over_algorithmic"] = executed / flops_dom if executed else None
    roof["mfma_tflops"] = flops_dom / avg_s / 1e12
    roof["mfma_frac"] = flops_dom / avg_s / 1e12 / MFMA_PEAK_TFLOPS[w.dtype]
    roof["hbm_algorithmic_gbs"] = bytes_dom / avg_s / 1e9
    roof["hbm_algorithmic_frac"] = bytes_dom / avg_s / 1e9 / HBM_PEAK_GBS
    # the same figures against what this device delivers on the two reference kernels (context; `frac` stays
    # against the published peaks)
    if with_peaks:
        pk = measure_peaks(5)
        roof["achievable"] = pk
        if w.dtype == "bf16":
            roof["mfma_frac_of_achievable"] = roof["mfma_tflops"] / pk["mfma_loop_TFLOPps"]
        roof["hbm_algorithmic_frac_of_achievable"] = roof["hbm_algorithmic_gbs"] / pk["stream_copy_GBps"]

    flops = nominal_flops(w, args.mode, args.picks)
    out = {
        "metric": {"rows": "csat_forward_tflops", "columns": "csat_forward_columnwise_tflops",
                   "lista": "csat_forward_lista_tflops", "omp": "csat_forward_omp_tflops",
                   "hadamard": "csat_forward_hadamard_tflops",
                   "columns_hadamard": "csat_forward_columnwise_hadamard_tflops"}[args.mode], "value": flops / dt / 1e12, "unit": "TFLOP/s",
        "tokens_per_s": w.B * w.n_q / dt,
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": dt * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "H": w.H, "n_q": w.n_q, "n": w.n, "d": w.d, "m": w.m,
                   "iters": w.iters, "lambda": w.lam, "phi": w.phi_kind, "decode": args.mode,
                   "launch": "hip graph replay" if args.graph else "eager",
                   **({"picks": args.picks} if args.mode == "omp" else {})},
        "nominal_flops": flops,
        "stage_ms": stage_ms,
        "roofline": roof,
    }
    if with_cpu:
        if args.mode in ("lista", "omp"):
            out["cpu_baseline"] = cpu_baseline_other_decoder(w, Q, K, V, Phi, mu, args.mode, args.picks)
        else:       # the structured matrix is an explicit Phi to the oracle
            columns = args.mode in ("columns", "columns_hadamard")
            out["cpu_baseline"] = (cpu_baseline_columns if columns else cpu_baseline)(w, Q, K, V, Phi, mu)
    del tQ, tK, tV, tPhi, ws, C
    torch.cuda.empty_cache()
    return out


def summary(o):
    """The figures of one workload that go into the headline line's `all_workloads` array."""
    r = o["roofline"]
    return {"workload": o["config"]["workload"], "dtype": o["dtype"], "steps": o["steps"], "warmup": o["warmup"],
            "ms_per_step": o["ms_per_step"], "tflops": o["value"], "tokens_per_s": o["tokens_per_s"],
            "stage_ms": o["stage_ms"],
            "roofline": {k: r.get(k) for k in ("bound", "achieved", "peak", "unit", "frac", "kernel", "avg_launch_us",
                                                "launches_per_step", "traffic", "algorithmic_bytes", "mfma_frac",
                                                "hbm_algorithmic_frac")}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="short_video")
    ap.add_argument("--picks", type=int, default=8, help="picks per row for --mode omp")
    ap.add_argument("--mode", choices=("rows", "columns", "lista", "omp", "hadamard", "columns_hadamard", "sweep", "peaks"), default="rows",
                    help="rows: one decoder problem per query row (csat_forward, the headline); "
                         "columns: one per feature column of the context matrix (csat_forward_rd, self-attention workloads); "
                         "lista: the row-wise path with the unrolled decoder (csat_measure + csat_compressed_attention + "
                         "csat_recover_lista, analytic weights); omp: the same with matching pursuit (csat_recover_omp); "
                         "hadamard: the block with a subsampled-Hadamard Phi, measurement and decoder by fast transforms (csat_forward_hadamard); "
                         "sweep: the compressed block alone (measurement + compressed attention) over sequence lengths "
                         "512..8192 at fixed m = 256, next to m = n (no compression)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step into a HIP graph and time replays (for the launch-bound small workloads)")
    ap.add_argument("--no-peaks", action="store_true",
                    help="skip the two reference kernels (streaming copy, MFMA loop) behind roofline.achievable")
    ap.add_argument("--option", action="append", default=[], metavar="KEY=VALUE",
                    help="kernel-selection override passed to csat_set_option (A/B measurements), e.g. fused_schedule=1")
    ap.add_argument("--headline-only", action="store_true",
                    help="time the named workload only (the default run adds the other four workloads as `all_workloads`)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy (reference dispatch for rocprofv3 FETCH_SIZE/WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1")

    import numpy as np
    import torch

    import csat_inputs as gen
    import paper_2507_02957_amd as csat

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the HIP path has no CPU fallback")
    for kv in args.option:
        key, _, value = kv.partition("=")
        csat.csat_set_option(key, int(value))
    if args.mode == "sweep":
        return sweep(args)
    if args.mode == "peaks":
        return peaks(args)
    out = measure(args, args.workload, args.steps, args.warmup, not args.no_peaks, not args.no_cpu_baseline)
    if args.mode == "rows" and args.workload == "short_video" and not args.headline_only and not args.graph:
        # the other four workloads, in the same line: few steps each (long_video takes 0.9 s per forward)
        others = []
        for name, st, wu in (("tiny", 20, 5), ("image_text", 20, 5), ("cross_modal", 10, 3), ("long_video", 2, 1)):
            o = measure(args, name, st, wu, False, False)
            others.append(summary(o))
        out["all_workloads"] = [summary(out)] + others
    print(json.dumps(out))


if __name__ == "__main__":
    main()
