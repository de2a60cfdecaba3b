#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input: one fg_gemm call
computing D = A.B + C at M = N = K = 8192 (FP16 A and B, column-major; FP32 C and D; FP32
accumulation; alpha = beta = 1) with the inputs already resident in HBM.  The line printed at
the end is the contract with the build driver:

    value      whole-job TFLOP/s (2 M N K flops per step)
    roofline   the GEMM kernel against the dense FP16 MFMA peak of the chip; `achieved` uses the
               kernel's average launch duration measured with HIP events on the launch stream
               over the timed region
    cpu_baseline  the FP64 CPU oracle as it stands, timed on this machine's host cores on a bounded
               sample of output entries of the same problem (each a full K-long dot product)
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "TFLOP/s and % of FP16 MFMA peak, mixed-precision GEMM N=8192 and GETT"
MFMA_FP16_PEAK_TFLOPS = 2500.0     # MI355X dense FP16 MFMA, published (2.5 PFLOP/s)
# Bytes per launch of the 8192^3 kernel that crossed the L2 <-> memory-side boundary.  NOT measured
# by this program: a constant from two rocprofv3 --pmc runs of this command (FETCH_SIZE, WRITE_SIZE),
# each scaled by what the same counter reads for a plain copy kernel of known size (factors 2.0 and
# 1.0), recorded in the file named below.  It is reported only when the kernel that is timed is the
# one that was profiled (same plan name), and the JSON line names the source.
PROFILED_TRAFFIC = {"kernel": "gemm_nn_256x256x64_k32", "bytes": 2.168e9, "source": "profiles/gemm_nn_8192_pmc.md"}


def cpu_baseline(M, N, K, A, lda, B, ldb, C, ldc, budget_s=12.0):
    """The oracle as it stands, timed on this machine's host cores.  `value` comes from a bounded sample
    of output entries of the timed workload itself (each a full K-long FP64 dot product) and is
    what the full problem would run at: `projected_seconds_full_problem` is a projection from it,
    not a measurement.  `legs` are problems the oracle computes in full: config 1 (256^3), the
    1024^3 point of config 2 and contraction 5a."""
    import numpy as np
    from oracle import cpu_oracle as O
    threads = O.default_threads()
    rng = np.random.default_rng(1)

    def run(count):
        I = rng.integers(0, M, count); J = rng.integers(0, N, count)
        t0 = time.perf_counter()
        O.gemm(M, N, K, 1.0, O.Operand(A, O.COL, lda), O.Operand(B, O.COL, ldb), 1.0, C, None, O.COL, ldc,
               at=(I, J), threads=threads)
        return time.perf_counter() - t0

    probe = 20000
    t = run(probe)
    count = int(min(max(probe, probe * budget_s / max(t, 1e-6)), 4_000_000))
    t = run(count)
    flops = 2.0 * K * count
    rate = flops / t
    legs = []

    def leg(name, fl, fn):
        t0 = time.perf_counter()
        fn()
        dt = time.perf_counter() - t0
        legs.append({"workload": name, "computed": "in full", "seconds": dt, "GFLOPs": fl / dt * 1e-9})

    for n, cfg in ((256, "configs[0]"), (1024, "configs[1] at N=1024")):
        if n <= min(M, N, K) and lda >= n and ldb >= n:
            a, b, c = A[:n * n], B[:n * n], C[:n * n]
            leg("%s: D = A.B + C, M=N=K=%d" % (cfg, n), 2.0 * n ** 3,
                lambda: O.gemm(n, n, n, 1.0, O.Operand(a, O.COL, n), O.Operand(b, O.COL, n), 1.0, c, None, O.COL, n, threads=threads))
    e = 256
    if A.size >= e ** 3 and B.size >= e * e:
        st3, st2 = [1, e, e * e], [1, e]
        leg("configs[4] 5a: C[a,b,c] = sum_d A[a,d,c] B[d,b], extents 256", 2.0 * e ** 4,
            lambda: O.contract({0: e, 1: e, 2: e, 3: e}, [0, 3, 2], st3, A[:e ** 3], [3, 1], st2, B[:e * e], [0, 1, 2], st3, threads=threads))
    return {"value": rate * 1e-12, "unit": "TFLOP/s", "cores": threads, "kind": "oracle",
            "sample": "%d of %d output entries of the same %dx%dx%d problem, each a full K=%d FP64 dot product; %.1f s"
                      % (count, M * N, M, N, K, K, t),
            "projected_seconds_full_problem": 2.0 * M * N * K / rate, "legs": legs}


def extras(fg, W, torch, n, A, B, mC, mD, stream, cold=True, sweep16k=True, fixed_launches=0):
    """Other rows of the hot-path table, outside the timed region: the remaining layout pairs at
    the same size, the fused-epilogue and layout-adapter configurations and the contractions.
    Each figure is flops (or algorithmic bytes) over the mean of 10 launches timed with HIP events;
    the "_cold" ones rotate over independent operand sets so that nothing is served from a cache
    filled by the previous launch (working sets below 512 MB otherwise stay in the 256 MB
    memory-side cache between launches)."""
    import math
    res = {}
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def timed(fn, reps=20):
        # After a change of kernel the engine clock needs some tens of milliseconds to settle
        # (a 4096^3 product measured 12 % slower over launches 21-40 than in the steady state), so
        # warm-up and timed region are sized by time: at least 20 launches and 60 ms of warm-up,
        # at least `reps` launches and 40 ms timed.
        if fixed_launches:                      # profiler runs: a fixed, small number of dispatches per row
            for _ in range(fixed_launches):
                fn()
            e0.record(stream)
            for _ in range(fixed_launches):
                fn()
            e1.record(stream)
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / fixed_launches * 1e-3
        e0.record(stream)
        for _ in range(5):
            fn()
        e1.record(stream)
        torch.cuda.synchronize()
        per_launch_ms = max(e0.elapsed_time(e1) / 5, 1e-3)
        for _ in range(max(15, min(4000, int(60.0 / per_launch_ms)))):
            fn()
        reps = max(reps, min(4000, int(40.0 / per_launch_ms)))
        e0.record(stream)
        for _ in range(reps):
            fn()
        e1.record(stream)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps * 1e-3

    def timed_cold(make, set_bytes, reps=3):
        """Mean launch time when no operand is left in a cache by the previous launch: `make()`
        builds one independent set of operands and returns the call on it; the launches rotate
        over enough sets that a set is touched again only after more than 768 MB of other sets
        (the memory-side cache holds 256 MB, the L2s 32 MB)."""
        calls = [make() for _ in range(max(2, -(-768_000_000 // int(set_bytes)) + 1))]
        for fn in calls:
            fn()
        e0.record(stream)
        for _ in range(reps):
            for fn in calls:
                fn()
        e1.record(stream)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / (reps * len(calls)) * 1e-3

    def guard(name, fn):
        if name.endswith(("_cold_GBps", "_cold_TFLOPs")) and not cold:
            return
        try:
            res[name] = fn()
        except Exception as ex:  # keep the headline line even if an extra cannot run
            res[name] = "error: %s" % ex

    def mfma_ceiling():
        fl = [0]

        def run():
            fl[0] = fg.fg_probe_mfma(A, 2000, stream=stream)
        t = timed(run, reps=5)
        return fl[0] / t * 1e-12
    guard("mfma_only_rate_on_this_data_TFLOPs", mfma_ceiling)

    def mfma_ceiling_k32():
        fl = [0]

        def run():
            fl[0] = fg.fg_probe_mfma(A, 2000, stream=stream, k32=True)
        t = timed(run, reps=5)
        return fl[0] / t * 1e-12
    guard("mfma_only_rate_16x16x32_on_this_data_TFLOPs", mfma_ceiling_k32)

    def kloop_mix():
        fl = [0]

        def run():
            fl[0] = fg.fg_probe_mfma(A, 1000, stream=stream, kloop_mix=True)
        t = timed(run, reps=5)
        return fl[0] / t * 1e-12
    # 16x16x32 matrix instructions + the LDS fragment reads and direct loads of the 256x256x64 K loop
    # in its proportions, nothing depending on anything: the bound of that K loop on this data
    guard("kloop_instruction_mix_rate_on_this_data_TFLOPs", kloop_mix)

    flops = 2.0 * n ** 3
    # The whole config-2 sweep, operands left in the caches by the previous launch ("hot"): every
    # size in every layout pair, plus config 1 (256^3 NN).  The sizes below the timed one use the
    # leading part of the same buffers; 16384 gets buffers of its own, released afterwards.
    pairs = (("NN", fg.FG_COL, fg.FG_COL), ("NT", fg.FG_COL, fg.FG_ROW), ("TN", fg.FG_ROW, fg.FG_COL), ("TT", fg.FG_ROW, fg.FG_ROW))

    def sweep_point(sz, a_buf, b_buf, c_buf, d_buf, layouts):
        for name, la, lb in layouts:
            if sz == n and name == "NN":
                continue                         # the timed workload itself
            a2, b2 = fg.Matrix(a_buf, la, sz), fg.Matrix(b_buf, lb, sz)
            c2, d2 = fg.Matrix(c_buf, fg.FG_COL, sz), fg.Matrix(d_buf, fg.FG_COL, sz)
            guard("gemm_%s_%d_TFLOPs" % (name, sz), lambda: 2.0 * sz ** 3 / timed(
                lambda: fg.fg_gemm(sz, sz, sz, 1.0, a2, b2, 1.0, c2, d2, stream=stream), reps=10 if sz > 8192 else 20) * 1e-12)
    sweep_point(256, A, B, mC.re, mD.re, pairs[:1])
    for sz in (1024, 2048, 4096, 8192):
        if sz <= n:
            sweep_point(sz, A, B, mC.re, mD.re, pairs)
    if n == 8192 and sweep16k:
        def big():
            sz = 16384
            a16 = W.uniform_pm1(sz * sz, W.stream_id(2, "A"), device=A.device)
            b16 = W.uniform_pm1(sz * sz, W.stream_id(2, "B"), device=A.device)
            c16 = W.uniform_pm1(sz * sz, W.stream_id(2, "C"), device=A.device, dtype=torch.float32)
            d16 = torch.empty_like(c16)
            sweep_point(sz, a16, b16, c16, d16, pairs)
            return "done"
        guard("sweep_16384", big)
        torch.cuda.empty_cache()

    m = 4096
    dev = A.device
    A4, B4 = A[:m * m], B[:m * m]
    A4i = W.uniform_pm1(m * m, W.stream_id(4, "A_im"), device=dev)
    B4i = W.uniform_pm1(m * m, W.stream_id(4, "B_im"), device=dev)
    C4 = W.uniform_pm1(m * m, W.stream_id(4, "C"), device=dev, dtype=torch.float32)
    C4i = W.uniform_pm1(m * m, W.stream_id(4, "C_im"), device=dev, dtype=torch.float32)
    D4, D4i = torch.empty_like(C4), torch.empty_like(C4)
    bias = W.uniform_pm1(8192, W.stream_id(3, "bias"), device=dev, dtype=torch.float32)
    dvec = W.uniform_pm1(m, W.stream_id(4, "d"), device=dev)
    M = fg.Matrix
    guard("config3_relu_bias_4096_TFLOPs", lambda: 2.0 * m ** 3 / timed(lambda: fg.fg_gemm(
        m, m, m, 1.0, M(A4, 0, m), M(B4, 0, m), 0.0, None, M(D4, 0, m), bias=bias, bias_dim=0, act=fg.FG_ACT_RELU, stream=stream)) * 1e-12)
    D3 = torch.empty(8192 * 1024, dtype=torch.float32, device=dev)
    guard("config3_relu_bias_8192x1024x4096_TFLOPs", lambda: 2.0 * 8192 * 1024 * 4096 / timed(lambda: fg.fg_gemm(
        8192, 1024, 4096, 1.0, M(A[:8192 * 4096], 0, 8192), M(B[:4096 * 1024], 0, 4096), 0.0, None, M(D3, 0, 8192),
        bias=bias, bias_dim=0, act=fg.FG_ACT_RELU, stream=stream)) * 1e-12)
    # last row of the fusion table (Section 5.3): bias, ReLU on C and D, a constant added to A and B
    guard("fusion_table_last_row_4096_TFLOPs", lambda: 2.0 * m ** 3 / timed(lambda: fg.fg_gemm(
        m, m, m, 1.0, M(A4, 0, m), M(B4, 0, m), 1.0, M(C4, 0, m), M(D4, 0, m), bias=bias, bias_dim=0, act=fg.FG_ACT_RELU,
        a_add=0.5, b_add=-0.25, c_act=fg.FG_ACT_RELU, stream=stream)) * 1e-12)
    guard("fusion_table_first_row_4096_TFLOPs", lambda: 2.0 * m ** 3 / timed(lambda: fg.fg_gemm(
        m, m, m, 1.0, M(A4, 0, m), M(B4, 0, m), 1.0, M(C4, 0, m), M(D4, 0, m), stream=stream)) * 1e-12)
    guard("config4_complex_planar_4096_TFLOPs", lambda: 8.0 * m ** 3 / timed(lambda: fg.fg_gemm(
        m, m, m, 1.0, M(A4, 0, m, im=A4i), M(B4, 0, m, im=B4i), 1.0, M(C4, 0, m, im=C4i), M(D4, 0, m, im=D4i), stream=stream)) * 1e-12)
    def cplx_interleaved():
        weave = lambda x, y: torch.stack((x, y), dim=-1).reshape(-1).contiguous()
        Aw, Bw, Cw = weave(A4, A4i), weave(B4, B4i), weave(C4, C4i)
        Dw = torch.empty_like(Cw)
        il = lambda t, d: M(t, 0, m, dtype=d)
        return 8.0 * m ** 3 / timed(lambda: fg.fg_gemm(m, m, m, 1.0, il(Aw, fg.FG_CF16), il(Bw, fg.FG_CF16), 1.0,
                                                        il(Cw, fg.FG_CF32), il(Dw, fg.FG_CF32), stream=stream)) * 1e-12
    guard("complex_interleaved_4096_TFLOPs", cplx_interleaved)
    guard("dual_planar_4096_TFLOPs", lambda: 6.0 * m ** 3 / timed(lambda: fg.fg_gemm_dual(
        m, m, m, 1.0, M(A4, 0, m, im=A4i), M(B4, 0, m, im=B4i), 1.0, M(C4, 0, m, im=C4i), M(D4, 0, m, im=D4i), stream=stream)) * 1e-12)
    Ab, Bb = A.to(torch.bfloat16), B.to(torch.bfloat16)
    guard("gemm_NN_bf16_%d_TFLOPs" % n, lambda: flops / timed(lambda: fg.fg_gemm(
        n, n, n, 1.0, M(Ab, 0, n), M(Bb, 0, n), 1.0, mC, mD, stream=stream)) * 1e-12)
    diag_bytes = m * m * 2 + 2 * m * m * 4 + m * 2
    # C and D stored as binary16 (the type-conversion transform of Section 4.2.3): same flops, half the C and D bytes
    Ch, Dh = mC.re.to(torch.float16), torch.empty(n * n, dtype=torch.float16, device=dev)
    guard("gemm_NN_%d_binary16_C_D_TFLOPs" % n, lambda: flops / timed(lambda: fg.fg_gemm(
        n, n, n, 1.0, M(A, 0, n), M(B, 0, n), 1.0, M(Ch, 0, n), M(Dh, 0, n), stream=stream)) * 1e-12)
    guard("config4_diagonal_A_4096_GBps", lambda: diag_bytes / timed(lambda: fg.fg_gemm(
        m, m, m, 1.0, M(dvec, fg.FG_DIAG, 0), M(B4, 0, m), 1.0, M(C4, 0, m), M(D4, 0, m), stream=stream)) * 1e-9)

    def diag_set():
        b, c, d = B4.clone(), C4.clone(), torch.empty_like(D4)
        return lambda: fg.fg_gemm(m, m, m, 1.0, M(dvec, fg.FG_DIAG, 0), M(b, 0, m), 1.0, M(c, 0, m), M(d, 0, m), stream=stream)
    guard("config4_diagonal_A_4096_cold_GBps", lambda: diag_bytes / timed_cold(diag_set, diag_bytes) * 1e-9)

    def square_set():
        a_, b, c, d = A4.clone(), B4.clone(), C4.clone(), torch.empty_like(D4)
        return lambda: fg.fg_gemm(m, m, m, 1.0, M(a_, 0, m), M(b, 0, m), 1.0, M(c, 0, m), M(d, 0, m), stream=stream)
    guard("gemm_NN_4096_cold_TFLOPs", lambda: 2.0 * m ** 3 / timed_cold(square_set, 12 * m * m) * 1e-12)

    a, b, c, d, e, f = range(6)

    def contraction(ext, mA, mB, mC, cold=False):
        sA = W.col_major_strides(tuple(ext[x] for x in mA))
        sB = W.col_major_strides(tuple(ext[x] for x in mB))
        sC = W.col_major_strides(tuple(ext[x] for x in mC))
        nA, nB, nC = (math.prod(ext[x] for x in ms) for ms in (mA, mB, mC))
        nbytes = nA * 2 + nB * 2 + nC * 4

        def one_set(copy=True):
            ta, tb = (A[:nA].clone(), B[:nB].clone()) if copy else (A[:nA], B[:nB])
            out = torch.empty(nC, dtype=torch.float32, device=dev)
            return lambda: fg.fg_contract(mA, sA, ta, mB, sB, tb, mC, sC, None, out, ext, stream=stream)
        t = timed_cold(one_set, nbytes) if cold else timed(one_set(copy=False))
        return 2.0 * math.prod(ext.values()) / t * 1e-12, nbytes / t * 1e-9

    def c5a():
        ext = {a: 256, b: 256, c: 256, d: 256}
        tf, gb = contraction(ext, [a, d, c], [d, b], [a, b, c])
        res["config5a_contraction_256_GBps"] = gb
        if cold:
            tfc, gbc = contraction(ext, [a, d, c], [d, b], [a, b, c], cold=True)
            res["config5a_contraction_256_cold_TFLOPs"] = tfc
            res["config5a_contraction_256_cold_GBps"] = gbc
        return tf
    guard("config5a_contraction_256_TFLOPs", c5a)
    guard("config5b_contraction_64_TFLOPs", lambda: contraction({a: 64, b: 64, c: 64, d: 64, e: 64, f: 64}, [a, e, b, f], [d, f, c, e], [a, b, c, d])[0])
    # the contraction the paper measures in Section 5.5: D_abc = A_bda B_dc, (a, b, c, d) = (64, 32, 2048, 2048)
    guard("paper_contraction_64_32_2048_2048_TFLOPs", lambda: contraction({a: 64, b: 32, c: 2048, d: 2048}, [b, d, a], [d, c], [a, b, c])[0])
    return res


def markdown_table(path):
    """A table of the current numbers (markdown), from a JSON line this program wrote earlier."""
    d = json.load(open(path))
    ex = d.get("extras", {})
    peak = MFMA_FP16_PEAK_TFLOPS
    rows = [("headline: " + d["config"]["kernel"] + " (timed region)", d["roofline"]["achieved"], "TFLOP/s")]
    rows += [(k[:-7], v, "TFLOP/s") for k, v in ex.items() if k.endswith("_TFLOPs") and isinstance(v, float)]
    rows += [(k[:-5], v, "GB/s") for k, v in ex.items() if k.endswith("_GBps") and isinstance(v, float)]
    print("| bench.py key | measured | of the roof |")
    print("|---|---|---|")
    for name, v, unit in rows:
        roof = "%.1f %% of 2.5 PFLOP/s" % (100 * v / peak) if unit == "TFLOP/s" else "%.1f %% of 8 TB/s" % (100 * v / 8000.0)
        print("| %s | %.0f %s | %s |" % (name, v, unit, roof))


def main():
    if len(sys.argv) == 3 and sys.argv[1] == "--table":
        return markdown_table(sys.argv[2])
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # Defaults: the engine clock dips after the first few launches of a fresh process and takes about
    # a hundred launches (0.1 s) to settle, so the default warm-up covers that and the timed region
    # measures the steady state (see profiles/gemm_nn_8192_kernel_trace.md for the series).
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--size", type=int, default=8192, help="M = N = K of the timed GEMM")
    ap.add_argument("--settle-ms", type=float, default=300.0,
                    help="untimed: run the step for this long before the warm-up steps so that the engine clock has settled")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the untimed-region extras (other layouts and configs)")
    ap.add_argument("--no-cold", action="store_true",
                    help="skip the cache-cold extras (keeps one group of launches per workload in a profile)")
    ap.add_argument("--extras-launches", type=int, default=0,
                    help="extras: this many warm-up and this many timed launches per row instead of sizing both by time (for profiler runs)")
    ap.add_argument("--no-16384", action="store_true", help="skip the 16384^3 points of the sweep (3.2 GB of extra operands)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain elementwise copy kernel (D = -C: 4 M N bytes read, 4 M N written), "
                         "so a counter profile of this command can be scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (D's tiles are independent, so the path would shard "
                 "over GPUs without any exchange, but that is not built); run with --gpus 1")

    import torch
    from paper_2009_12263_amd import binding as fg
    from paper_2009_12263_amd import workloads as W

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = "cuda"
    n = args.size
    M = N = K = n
    A = W.uniform_pm1(M * K, W.stream_id(2, "A"), device=dev)
    B = W.uniform_pm1(K * N, W.stream_id(2, "B"), device=dev)
    C = W.uniform_pm1(M * N, W.stream_id(2, "C"), device=dev, dtype=torch.float32)
    D = torch.empty_like(C)
    mA, mB = fg.Matrix(A, fg.FG_COL, M), fg.Matrix(B, fg.FG_COL, K)
    mC, mD = fg.Matrix(C, fg.FG_COL, M), fg.Matrix(D, fg.FG_COL, M)
    stream = torch.cuda.current_stream()

    def step():
        fg.fg_gemm(M, N, K, 1.0, mA, mB, 1.0, mC, mD, stream=stream)

    if args.copy_calibration:
        torch.neg(C, out=D)      # one elementwise kernel: reads 4 M N bytes, writes 4 M N bytes
    # Untimed, before the W warm-up steps: keep the GPU busy with the same call until the engine
    # clock has settled.  In a fresh process the clock dips after the first few launches and takes
    # about 0.1 s of continuous work to come back (launch durations 0.91, 0.98, 1.08, 1.08, 1.02 ...
    # 0.89 ms by the 25th launch, 0.85 from the 100th on); a run with few warm-up steps would time
    # that transient instead of the rate a job sees.  Not counted in `warmup` or `steps`.
    t_settle = time.perf_counter()
    while (time.perf_counter() - t_settle) * 1e3 < args.settle_ms:
        for _ in range(20):
            step()
        torch.cuda.synchronize()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record(stream)
    for _ in range(args.steps):
        step()
    e1.record(stream)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    kern_ms = e0.elapsed_time(e1) / args.steps
    flops = 2.0 * M * N * K
    value = flops / (wall_ms * 1e-3) * 1e-12
    achieved = flops / (kern_ms * 1e-3) * 1e-12

    # spread of single launches (outside the timed region): each launch between its own two events
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(20)]
    for b, e in evs:
        b.record(stream)
        step()
        e.record(stream)
    torch.cuda.synchronize()
    per_launch = sorted(b.elapsed_time(e) for b, e in evs)

    plan_name = fg.fg_gemm_plan(M, N, K)
    out = {
        "metric": METRIC, "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": wall_ms, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f16 in / f32 accumulate", "data": "synthetic",
        "settle_ms": args.settle_ms,
        "config": {"workload": "configs[1]: square mixed-precision GEMM D = A.B + C, M=N=K=%d, A,B FP16 column-major (NN), "
                               "C,D FP32, uniform[-1,1), alpha=beta=1" % n,
                   "kernel": plan_name},
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": MFMA_FP16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / MFMA_FP16_PEAK_TFLOPS,
                     "traffic": PROFILED_TRAFFIC["bytes"] if (n == 8192 and plan_name == PROFILED_TRAFFIC["kernel"]) else None,
                     "traffic_source": (PROFILED_TRAFFIC["source"] + " (rocprofv3 --pmc FETCH_SIZE/WRITE_SIZE of this command, not measured in this run)")
                                       if (n == 8192 and plan_name == PROFILED_TRAFFIC["kernel"]) else None,
                     "kernel_ms": kern_ms,
                     "per_launch_ms_min": per_launch[0], "per_launch_ms_median": per_launch[len(per_launch) // 2],
                     "frac_of_mfma_only_rate_on_this_data": None},
    }

    if not args.no_extras:
        out["extras"] = extras(fg, W, torch, n, A, B, mC, mD, stream, cold=not args.no_cold, sweep16k=not args.no_16384,
                               fixed_launches=args.extras_launches)
        # the MFMA-only rate in the instruction shape the timed kernel uses
        key = "mfma_only_rate_16x16x32_on_this_data_TFLOPs" if out["config"]["kernel"].endswith("_k32") else "mfma_only_rate_on_this_data_TFLOPs"
        sustained = out["extras"].get(key)
        if isinstance(sustained, float) and sustained > 0:
            out["roofline"]["frac_of_mfma_only_rate_on_this_data"] = achieved / sustained
        mix = out["extras"].get("kloop_instruction_mix_rate_on_this_data_TFLOPs")
        if isinstance(mix, float) and mix > 0 and out["config"]["kernel"].endswith("_k32"):
            # whole kernel (K loops + epilogues) against the rate of the K loop's bare instruction mix
            out["roofline"]["frac_of_kloop_instruction_mix_rate"] = achieved / mix

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(M, N, K, A.cpu().numpy(), M, B.cpu().numpy(), K, C.cpu().numpy(), M)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
