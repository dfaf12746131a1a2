#!/usr/bin/env python3
"""Benchmark of the fused RMSNorm -> MatMul library on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload IDX] [--no-extra] [--no-cpu]

A step is one library call (one pass of the whole fused path: sums of squares in the K-loop, gain,
GEMM, split-K reduction, 1/rms, and the SiLU gate for the gated workloads) over one batch of seeded
synthetic input that is already resident in HBM.  The headline workload is benchmark configuration
index 1 (decode RMSNorm -> MatMul, bf16, X[16,4096], W[4096,4096]); the other three bf16
configurations are timed too and reported under "other_workloads", and the paper's own workloads at its
shapes and in its precision (fp16, 8 or 16 rows, hidden size 1024 or 4096) under "paper_shapes", its
running example (softmax, then a matrix product, Figure 1) under "running_example", its two attention
workloads under "attention", 32 / 128 / 512 rows against the decode-sized weights under "mid_rows", and two
decode calls with about 1 GB of weights under "large_decode".

Decode workloads rotate over enough distinct weight buffers (>= 1 GiB in total) that W is streamed
from HBM and not from the 256 MB last-level cache; the cache-hot single-buffer time is reported
separately.  One JSON line goes to stdout; progress goes to stderr.
"""
import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

import prism_inputs as pi  # noqa: E402

METRIC = "fused RMSNorm+GEMM: HBM GB/s (decode) and TFLOP/s (prefill), % of roofline"
HBM_PEAK_GBS = 8000.0         # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 MFMA, published


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def counted_bytes(wl):
    """Algorithmic bytes of one call: X + g + W (+ W2) + Y, each once, in the storage type."""
    e = 2 if wl.dtype == pi.BF16 else 4
    nw = 2 if wl.gated else 1
    return e * (wl.M * wl.K + wl.K + nw * wl.K * wl.N + wl.M * wl.N)


def counted_flops(wl):
    """Algorithmic flops of one call: 2 M K N per weight matrix (norm, gain and gate not counted)."""
    return 2 * wl.M * wl.K * wl.N * (2 if wl.gated else 1)


def is_decode(wl):
    return wl.M <= 16


class Runner:
    """Pre-marshalled library calls over R rotating buffer sets of one workload."""

    def __init__(self, wl, sets, stored=None):
        import torch
        import paper_2604_15272_amd as P
        self.P, self.torch, self.wl = P, torch, wl
        stored = stored if stored is not None else pi.draw_workload(wl)
        self.stored = stored
        tdt = torch.bfloat16 if wl.dtype == pi.BF16 else torch.float32

        def dev(a):
            t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
            return t.view(torch.bfloat16) if wl.dtype == pi.BF16 else t

        self.X, self.g = dev(stored["X"]), dev(stored["g"])
        names = ("W1", "W2") if wl.gated else ("W",)
        base = [dev(stored[n]) for n in names]
        # Further sets are row-rotated copies: same distribution, different addresses.
        self.W = [base] + [[torch.roll(w, r, 0).contiguous() for w in base] for r in range(1, sets)]
        self.Y = [torch.empty((wl.M, wl.N), dtype=tdt, device="cuda") for _ in range(sets)]
        self.op = P.PRISM_OP_RMSNORM_GATED_MLP if wl.gated else P.PRISM_OP_RMSNORM_MATMUL
        self.dt = P.PRISM_BF16 if wl.dtype == pi.BF16 else P.PRISM_F32
        P.ensure_workspace(P.prism_workspace_bytes(self.op, wl.M, wl.K, wl.N, self.dt))
        self.plan = P.prism_plan(self.op, wl.M, wl.K, wl.N, self.dt)
        stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
        vp = ctypes.c_void_p
        dims = (ctypes.c_int64(wl.M), ctypes.c_int64(wl.K), ctypes.c_int64(wl.N), ctypes.c_float(wl.eps),
                ctypes.c_int32(self.dt), stream)
        fn = P.lib.prism_rmsnorm_gated_mlp if wl.gated else P.lib.prism_rmsnorm_matmul
        self.fn = fn
        self.args = [(vp(self.X.data_ptr()), vp(self.g.data_ptr()), *[vp(w.data_ptr()) for w in self.W[s]],
                      vp(self.Y[s].data_ptr())) + dims for s in range(sets)]
        self.sets = sets

    def run(self, steps, first=0):
        fn, args, sets = self.fn, self.args, self.sets
        for i in range(steps):
            st = fn(*args[(first + i) % sets])
            if st != 0:
                raise RuntimeError(f"library call failed: {self.P.prism_status_string(st)}")

    def timed(self, steps, warmup, sets_used=None, regions=1):
        """`regions` timed regions of exactly `steps` calls each, after `warmup` untimed calls; every region is
        bracketed by torch.cuda.synchronize() on both sides.  Returns (wall ms per step, HIP-event ms per step) of
        the region with the median wall time, or, with regions > 1, the two lists."""
        torch = self.torch
        if sets_used == 1:
            saved, self.args, self.sets = (self.args, self.sets), self.args[:1], 1
        self.run(warmup)
        walls, evs = [], []
        for r in range(regions):
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            t0 = time.perf_counter()
            e0.record()
            self.run(steps, first=warmup + r * steps)
            e1.record()
            while not e1.query():   # the clock stops when the last call has finished, not when a sleeping
                pass                # host thread has been woken up
            t1 = time.perf_counter()
            torch.cuda.synchronize()
            walls.append((t1 - t0) * 1e3 / steps)
            evs.append(e0.elapsed_time(e1) / steps)
        if sets_used == 1:
            self.args, self.sets = saved
        if regions == 1:
            return walls[0], evs[0]
        return walls, evs

    def probe_split(self):
        """K-slices for the probe's grid of 128-column stripes: about as many workgroups as the kernel launches."""
        tiles = -(-self.wl.N // 128)
        return max(1, round(self.plan["grid_x"] * max(1, self.plan["grid_y"]) / tiles))

    def probe(self, steps, warmup):
        """The library's read-only probe over the same rotating weight sets, with this workload's split: what
        streaming W alone costs (HIP-event ms per launch)."""
        torch, P = self.torch, self.P
        vp, i64 = ctypes.c_void_p, ctypes.c_int64
        stream = vp(torch.cuda.current_stream().cuda_stream)
        P.ensure_workspace(1 << 20)
        args = [(vp(w[0].data_ptr()), vp(w[1].data_ptr()) if self.wl.gated else None, i64(self.wl.K), i64(self.wl.N),
                 ctypes.c_int32(self.probe_split()), stream) for w in self.W]

        def run(n, first=0):
            for i in range(n):
                st = P.lib.prism_probe_stream(*args[(first + i) % self.sets])
                if st != 0:
                    raise RuntimeError(f"probe failed: {P.prism_status_string(st)}")

        run(warmup)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        run(steps, first=warmup)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / steps

    def output(self, s=0):
        import torch
        y = self.Y[s]
        if self.wl.dtype == pi.BF16:
            return pi.to_f64(y.view(torch.uint16).cpu().numpy(), pi.BF16)
        return y.cpu().numpy().astype(np.float64)


REGIONS = 5   # timed regions per workload: median and minimum are reported


def median(v):
    v = sorted(v)
    return v[len(v) // 2] if len(v) % 2 else 0.5 * (v[len(v) // 2 - 1] + v[len(v) // 2])


def measure(idx, steps, warmup):
    wl = pi.WORKLOADS[idx]
    nbytes, flops = counted_bytes(wl), counted_flops(wl)
    dec = is_decode(wl)
    wbytes = 2 * wl.K * wl.N * (2 if wl.gated else 1)
    sets = max(2, -(-(1 << 30) // wbytes)) if dec else 1
    log(f"[bench] workload {idx} {wl.name}: M={wl.M} K={wl.K} N={wl.N} gated={wl.gated} sets={sets}")
    r = Runner(wl, sets)
    walls, evs = r.timed(steps, warmup, regions=REGIONS)
    wall_ms, ev_ms = median(walls), median(evs)
    # Roofline figure: launch duration = HIP-event time of a timed region / its launches, i.e. the average
    # per launch over the region, gaps between back-to-back launches included (one event pair per launch reads
    # twice the rocprofv3 duration for a ~10 us kernel; the region average reads a few per cent above it).
    # Median over the regions; the minimum is reported beside it.
    k_mean = ev_ms
    res = {
        "workload": wl.name, "config_index": idx, "M": wl.M, "K": wl.K, "N": wl.N, "gated": wl.gated,
        "plan": r.plan, "steps": steps, "regions": REGIONS, "ms_per_step": wall_ms, "ms_per_step_min": min(walls),
        "event_ms_per_step": ev_ms, "event_ms_per_step_min": min(evs), "region_wall_ms_per_step": walls,
        "region_event_ms_per_step": evs,
        "kernel_ms": k_mean, "buffer_sets": sets, "bytes_per_launch": nbytes, "flops_per_launch": flops,
    }
    if dec:
        res.update(value=nbytes / (wall_ms * 1e-3) / 1e9, unit="GB/s", bound="hbm",
                   achieved=nbytes / (k_mean * 1e-3) / 1e9, peak=HBM_PEAK_GBS)
        hot_ms = median(r.timed(steps, warmup, sets_used=1, regions=3)[1])
        res["cache_hot_kernel_ms"] = hot_ms
        res["cache_hot_GBps"] = nbytes / (hot_ms * 1e-3) / 1e9
        res["stream_probe_ms"] = r.probe(steps, warmup)
        if r.plan["tile_n"] == 64:
            # The dispatcher chose packed tiles with more K-slices for the tiles in slow address units: the same
            # call with that turned off (two 128-column tiles per workgroup, equal slices), for comparison.
            r.P.prism_set_stream_balance(0, 0)
            try:
                r.P.ensure_workspace(r.P.prism_workspace_bytes(r.op, wl.M, wl.K, wl.N, r.dt))
                res["equal_slices_kernel_ms"] = median(r.timed(steps, warmup, regions=3)[1])
            finally:
                r.P.prism_set_stream_balance(SLOW_UNITS["mask"], 0)
    else:
        res.update(value=flops / (wall_ms * 1e-3) / 1e12, unit="TFLOP/s", bound="mfma",
                   achieved=flops / (k_mean * 1e-3) / 1e12, peak=MFMA_BF16_PEAK_TFLOPS)
        res["vendor_gemm"] = measure_vendor_gemm(wl.M, wl.K, wl.N, wl.gated, max(5, steps // 4), 3)
        log(f"[bench]   vendor GEMM on the plain product(s): {res['vendor_gemm']['TFLOPs']:.0f} TFLOP/s")
    res["frac"] = res["achieved"] / res["peak"]
    if "stream_probe_ms" in res:
        log(f"[bench]   read-only probe (128-column stripes, as many workgroups): {res['stream_probe_ms'] * 1e3:.2f} us per launch "
            f"({nbytes / (res['stream_probe_ms'] * 1e-3) / 1e9:.0f} GB/s)")
    if "equal_slices_kernel_ms" in res:
        log(f"[bench]   with equal K-slices for all tiles (two-tile form): {res['equal_slices_kernel_ms'] * 1e3:.2f} us per launch")
    log(f"[bench]   {res['value']:.1f} {res['unit']} back-to-back (median of {REGIONS} regions of {steps} calls: "
        f"{wall_ms * 1e3:.2f} us/step wall, min {min(walls) * 1e3:.2f}; by events {ev_ms * 1e3:.2f}, min "
        f"{min(evs) * 1e3:.2f}); per launch by events {k_mean * 1e3:.2f} us -> {res['achieved']:.1f} {res['unit']} "
        f"= {100 * res['frac']:.1f}% of {res['bound']} peak")
    return res, r


def cpu_baseline(runner):
    """The oracle, as it stands, timed on this host on the headline workload (all of it: it is small)."""
    import oracle  # the cpu_baseline leg is the only place the benchmark touches the oracle
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    try:
        usable = len(os.sched_getaffinity(0))
    except AttributeError:
        usable = os.cpu_count() or 1
    wl, st = runner.wl, runner.stored
    X, g = pi.to_f64(st["X"], wl.dtype), pi.to_f64(st["g"], wl.dtype)
    Ws = [pi.to_f64(st[n], wl.dtype) for n in (("W1", "W2") if wl.gated else ("W",))]
    fn = (lambda: oracle.rmsnorm_gated_mlp(X, g, Ws[0], Ws[1], wl.eps)) if wl.gated else (
        lambda: oracle.rmsnorm_matmul(X, g, Ws[0], wl.eps))
    yhat = fn()  # untimed first call (page-in), also the parity reference
    reps, t0 = 0, time.perf_counter()
    while reps < 20000 and time.perf_counter() - t0 < 12.0:   # about 12 s of CPU work
        fn()
        reps += 1
    sec = (time.perf_counter() - t0) / reps
    runner.run(1)
    runner.torch.cuda.synchronize()
    y = runner.output(0)
    err = float(np.max(np.abs(y - yhat) / (np.abs(yhat) + 1.0)))
    return {
        "value": counted_bytes(wl) / sec / 1e9, "unit": "GB/s", "cores": int(cores), "kind": "oracle",
        "nproc": int(os.cpu_count() or 1), "usable_cpus": int(usable),
        "cores_note": "cores = threads of the BLAS pool that numpy.matmul used; nproc = CPUs the host reports; "
                      "usable_cpus = CPUs this process may run on",
        "sample": f"whole {wl.name} workload (M={wl.M}), fp64 numpy oracle, mean of {reps} calls, "
                  f"inputs already widened to fp64; {sec * 1e3:.2f} ms per call",
        "gpu_vs_oracle_worst_err": err,
    }


# The paper's own workloads (Section 7.1) at its shapes (n rows, hidden size d) and in its precision
# (fp16), none with a gain tensor.  The paper does not state the output width: N = d is assumed for
# RMSNorm -> MatMul and N = 4 d for the two MLP workloads.
PAPER_SHAPES = (
    ("rmsnorm", 8, 1024, 1024), ("rmsnorm", 8, 4096, 4096),
    ("rmsnorm_mlp", 8, 1024, 4096), ("rmsnorm_mlp", 16, 1024, 4096),
    ("swiglu", 8, 1024, 4096), ("swiglu", 8, 4096, 16384),
)


def measure_paper_shape(name, M, K, N, steps=1000, warmup=50):
    """Times one of the paper's workloads in fp16 over rotating weight sets (>= 512 MiB in total, so
    the weights come from HBM).  Random fp16 values of the benchmark recipe's scale, drawn on the device."""
    import torch
    import paper_2604_15272_amd as P
    nw = 1 if name == "rmsnorm" else 2
    wbytes = 2 * K * N * nw
    sets = max(2, min(256, -(-(512 << 20) // wbytes)))
    gen = torch.Generator(device="cuda").manual_seed(0x5EED1000 + M + K + N)
    X = torch.randn((M, K), generator=gen, device="cuda").to(torch.float16)
    Ws = [[(torch.randn((K, N), generator=gen, device="cuda") / K ** 0.5).to(torch.float16) for _ in range(nw)]
          for _ in range(sets)]
    Ys = [torch.empty((M, N), dtype=torch.float16, device="cuda") for _ in range(sets)]
    op = P.PRISM_OP_RMSNORM_MATMUL if nw == 1 else P.PRISM_OP_RMSNORM_GATED_MLP
    P.ensure_workspace(P.prism_workspace_bytes(op, M, K, N, P.PRISM_F16))
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    vp, i64 = ctypes.c_void_p, ctypes.c_int64
    dims = (i64(M), i64(K), i64(N))
    dt = ctypes.c_int32(P.PRISM_F16)
    if name == "rmsnorm":
        fn = P.lib.prism_rmsnorm_matmul
        args = [(vp(X.data_ptr()), None, vp(Ws[s][0].data_ptr()), vp(Ys[s].data_ptr())) + dims +
                (ctypes.c_float(1e-6), dt, stream) for s in range(sets)]
    elif name == "rmsnorm_mlp":
        fn = P.lib.prism_rmsnorm_glu
        args = [(vp(X.data_ptr()), None, vp(Ws[s][0].data_ptr()), vp(Ws[s][1].data_ptr()), vp(Ys[s].data_ptr())) +
                dims + (ctypes.c_float(1e-6), dt, stream) for s in range(sets)]
    else:
        fn = P.lib.prism_swiglu
        args = [(vp(X.data_ptr()), vp(Ws[s][0].data_ptr()), vp(Ws[s][1].data_ptr()), vp(Ys[s].data_ptr())) + dims +
                (dt, stream) for s in range(sets)]

    def run(n, first=0):
        for i in range(n):
            st = fn(*args[(first + i) % sets])
            if st != 0:
                raise RuntimeError(f"library call failed: {P.prism_status_string(st)}")

    run(warmup)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    run(steps, first=warmup)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / steps
    nbytes = 2 * (M * K + nw * K * N + M * N)
    res = {"workload": name, "dtype": "f16", "M": M, "K": K, "N": N, "weight_sets": sets, "steps": steps,
           "us_per_call": ms * 1e3, "GBps": nbytes / (ms * 1e-3) / 1e9, "frac_of_hbm_peak": nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
           "plan": P.prism_plan(op, M, K, N, P.PRISM_F16)}
    log(f"[bench]   paper {name} n={M} d={K} N={N} fp16: {ms * 1e3:.2f} us/call, {res['GBps']:.0f} GB/s")
    return res


def measure_running_example(steps=500, warmup=30):
    """The paper's running example (Figure 1): softmax(X[4096,4096]) @ W[4096,128] in fp16.  X is the large
    operand: it rotates over 17 buffers (544 MiB) so that it is streamed from HBM.  Bound: HBM."""
    import torch
    import paper_2604_15272_amd as P
    M, K, N, sets = 4096, 4096, 128, 17
    gen = torch.Generator(device="cuda").manual_seed(0x5EED2000)
    Xs = [(torch.randn((M, K), generator=gen, device="cuda") * 3.0).to(torch.float16) for _ in range(sets)]
    W = torch.randn((K, N), generator=gen, device="cuda").to(torch.float16)
    Ys = [torch.empty((M, N), dtype=torch.float16, device="cuda") for _ in range(sets)]
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    vp, i64 = ctypes.c_void_p, ctypes.c_int64
    args = [(vp(Xs[s].data_ptr()), vp(W.data_ptr()), vp(Ys[s].data_ptr()), i64(M), i64(K), i64(N),
             ctypes.c_int32(P.PRISM_F16), stream) for s in range(sets)]
    fn = P.lib.prism_softmax_matmul
    P.ensure_workspace(P.prism_workspace_bytes(P.PRISM_OP_SOFTMAX_MATMUL, M, K, N, P.PRISM_F16))

    def run(n, first=0, used=sets):
        for i in range(n):
            st = fn(*args[(first + i) % used])
            if st != 0:
                raise RuntimeError(f"library call failed: {P.prism_status_string(st)}")

    def timed(used):
        run(warmup, used=used)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        run(steps, first=warmup, used=used)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / steps

    ms, hot_ms = timed(sets), timed(1)
    nbytes = 2 * (M * K + K * N + M * N)
    res = {"workload": "softmax_matmul_running_example", "dtype": "f16", "M": M, "K": K, "N": N, "x_buffers": sets,
           "steps": steps, "us_per_call": ms * 1e3, "bound": "hbm", "bytes_per_launch": nbytes,
           "achieved": nbytes / (ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
           "frac": nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, "cache_hot_us_per_call": hot_ms * 1e3,
           "plan": P.prism_plan(P.PRISM_OP_SOFTMAX_MATMUL, M, K, N, P.PRISM_F16)}
    log(f"[bench]   running example softmax(X[4096,4096]) W[4096,128] fp16: {ms * 1e3:.2f} us/call, "
        f"{res['achieved']:.0f} GB/s = {100 * res['frac']:.1f}% of hbm peak (cache-hot {hot_ms * 1e3:.2f} us)")
    return res


def measure_attention(h, qk_norm, steps=1000, warmup=50):
    """The paper's attention workloads (Section 7.1): b = 2, g = 8 query heads per batch entry, one query position,
    head dimension 128, h keys, fp16; K and V rotate over enough buffers (>= 512 MiB) to come from HBM."""
    import torch
    import paper_2604_15272_amd as P
    B, G, D = 2, 8, 128
    kv_bytes = 2 * B * h * D * 2
    sets = max(2, min(512, -(-(512 << 20) // kv_bytes)))
    gen = torch.Generator(device="cuda").manual_seed(0x5EED3000 + h)
    Q = torch.randn((B, G, D), generator=gen, device="cuda").to(torch.float16)
    big = torch.randn((sets, 2, B, h, D), generator=gen, device="cuda").to(torch.float16)
    Os = torch.empty((sets, B, G, D), dtype=torch.float16, device="cuda")
    P.ensure_workspace(int(P.lib.prism_attention_workspace_bytes(B, G, h, D, P.PRISM_F16)))
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    vp, i64 = ctypes.c_void_p, ctypes.c_int64
    args = [(vp(Q.data_ptr()), vp(big[s, 0].data_ptr()), vp(big[s, 1].data_ptr()), vp(Os[s].data_ptr()), i64(B), i64(G),
             i64(h), i64(D), ctypes.c_float(1.0), ctypes.c_int32(int(qk_norm)), ctypes.c_float(1e-6),
             ctypes.c_int32(P.PRISM_F16), stream) for s in range(sets)]
    fn = P.lib.prism_gqa_decode_attention
    for i in range(warmup):
        if fn(*args[i % sets]) != 0:
            raise RuntimeError("attention call failed")
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(steps):
        fn(*args[(warmup + i) % sets])
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / steps
    nbytes = 2 * (2 * B * G * D) + kv_bytes
    res = {"workload": "qk_attention" if qk_norm else "attention", "dtype": "f16", "B": B, "G": G, "H": h, "D": D,
           "kv_sets": sets, "steps": steps, "us_per_call": ms * 1e3, "bound": "hbm", "bytes_per_launch": nbytes,
           "achieved": nbytes / (ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
           "frac": nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, "plan": P.prism_attention_plan(B, G, h, D, P.PRISM_F16)}
    log(f"[bench]   paper {res['workload']} b=2 g=8 d=128 h={h} fp16: {ms * 1e3:.2f} us/call, {res['achieved']:.0f} GB/s")
    return res


COPY_CALIBRATION_BYTES = 256 << 20
SLOW_UNITS = {"mask": 0}   # filled by main() from tune.detect_slow_units()


def measure_copy_ceiling(nbytes=256 << 20, buffers=6, steps=30):
    """Device-to-device copies (torch's copy kernel) over buffers that rotate past the last-level cache: bytes read
    plus bytes written per second, the measured ceiling of HBM traffic beside the published peak."""
    import torch
    srcs = [torch.full((nbytes // 2,), 1.0, dtype=torch.bfloat16, device="cuda") for _ in range(buffers)]
    dst = torch.empty_like(srcs[0])
    for i in range(buffers):
        dst.copy_(srcs[i])
    res = []
    for _ in range(REGIONS):
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(steps):
            dst.copy_(srcs[i % buffers])
        e1.record()
        torch.cuda.synchronize()
        res.append(e0.elapsed_time(e1) / steps)
    ms = median(res)
    out = {"GBps": 2 * nbytes / (ms * 1e-3) / 1e9, "GBps_best": 2 * nbytes / (min(res) * 1e-3) / 1e9,
           "bytes_per_copy": nbytes, "ms_per_copy": ms,
           "note": "torch device-to-device copy of 256 MiB, read + written bytes, sources rotating over 1.5 GiB"}
    del srcs, dst
    torch.cuda.empty_cache()
    return out


def measure_mfma_ceiling(iters=4000):
    """The library's matrix-pipe probe (prism_probe_mfma: 32x32x16 bf16 MFMAs on registers, two workgroups of four
    wavefronts per compute unit, no memory traffic): what the part sustains under its clock and power limits."""
    import torch
    import paper_2604_15272_amd as P
    sink = torch.zeros(4, dtype=torch.float32, device="cuda")
    vp = ctypes.c_void_p
    stream = vp(torch.cuda.current_stream().cuda_stream)
    wgs = 2 * P.prism_diag_cu_count()
    P.lib.prism_probe_mfma(vp(sink.data_ptr()), wgs, 100, stream)
    res = []
    for _ in range(REGIONS):
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        st = P.lib.prism_probe_mfma(vp(sink.data_ptr()), wgs, iters, stream)
        e1.record()
        torch.cuda.synchronize()
        if st != 0:
            raise RuntimeError("prism_probe_mfma failed")
        res.append(e0.elapsed_time(e1))
    flops = 32768.0 * 16 * iters * 4 * wgs
    return {"TFLOPs": flops / (median(res) * 1e-3) / 1e12, "TFLOPs_best": flops / (min(res) * 1e-3) / 1e12,
            "ms": median(res), "workgroups": wgs,
            "note": "prism_probe_mfma: matrix pipes alone (a launch of about 1 ms; longer runs clock lower)"}


def measure_cu_load_path(reps=8):
    """The library's load-shape probe (prism_probe_loads): bytes per shader clock that one compute unit's vector-memory
    path delivers, on L2-resident data, for four shapes of load instruction.  The multi-row decode kernels and the
    softmax kernels are bound by this path, and the operand-layout shape is the slow one."""
    import torch
    import paper_2604_15272_amd as P
    vp = ctypes.c_void_p
    stream = vp(torch.cuda.current_stream().cuda_stream)
    wgs = P.prism_diag_cu_count()
    buf = torch.ones(P.PROBE_LOADS_BYTES, dtype=torch.uint8, device="cuda")
    ticks = torch.zeros(8 * wgs, dtype=torch.int64, device="cuda")
    names = ("four rows x 256 B per instruction (W of the decode kernels)", "sixteen rows x 64 B (an operand read in MFMA layout)",
             "eight rows x 128 B (X requests of the prefill kernel)", "four rows x 128 B with 8-byte loads")
    out = []
    for pattern, name in enumerate(names):
        vals = []
        for _ in range(3):
            st = P.lib.prism_probe_loads(vp(buf.data_ptr()), ctypes.c_uint64(buf.numel()), pattern, reps, wgs,
                                         vp(ticks.data_ptr()), stream)
            if st != 0:
                raise RuntimeError("prism_probe_loads failed")
            torch.cuda.synchronize()
            per_wg = reps * P.PROBE_LOADS_BYTES * (0.5 if pattern == 3 else 1.0)
            vals.append(per_wg / float(ticks.double().mean().item()))
        out.append({"pattern": name, "bytes_per_clock_per_cu": median(vals)})
        log(f"[bench]   one compute unit's load path, {name}: {median(vals):.1f} B/clk")
    return out


def measure_stream_patterns(runner, steps=400, warmup=20):
    """The headline workload's weight bytes (32 MiB per buffer set, the same rotating sets) read with other access
    patterns, nothing computed: front to back in 256 contiguous pieces, and as stripes of other shapes (the stream
    probe on the same bytes viewed as [K', N'] with K' N' = K N).  What a launch of this size can stream at all."""
    import torch
    P = runner.P
    vp, i64 = ctypes.c_void_p, ctypes.c_int64
    stream = vp(torch.cuda.current_stream().cuda_stream)
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    P.ensure_workspace(1 << 20)
    wl = runner.wl
    nbytes = 2 * wl.K * wl.N
    cus = P.prism_diag_cu_count()
    ptrs = [w[0].data_ptr() for w in runner.W]

    def timed(call):
        for i in range(warmup):
            call(ptrs[i % len(ptrs)])
        res = []
        for _ in range(REGIONS):
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for i in range(steps):
                call(ptrs[(warmup + i) % len(ptrs)])
            e1.record()
            torch.cuda.synchronize()
            res.append(e0.elapsed_time(e1) / steps * 1e3)
        return median(res), min(res)

    out = []

    def linear(wgs):
        def call(p):
            if P.lib.prism_probe_linear(vp(p), ctypes.c_uint64(nbytes), wgs, vp(sink.data_ptr()), stream) != 0:
                raise RuntimeError("prism_probe_linear failed")
        return call

    def stripes(K2, N2, S):
        def call(p):
            if P.lib.prism_probe_stream(vp(p), None, i64(K2), i64(N2), ctypes.c_int32(S), stream) != 0:
                raise RuntimeError("prism_probe_stream failed")
        return call

    total = wl.K * wl.N
    patterns = [("front to back, one contiguous piece per compute unit", linear(cus)),
                ("front to back, two pieces per compute unit", linear(2 * cus)),
                (f"128-column stripes of [{wl.K},{wl.N}] x {max(1, cus * 128 // wl.N)} K-slices (the kernel's)",
                 stripes(wl.K, wl.N, max(1, cus * 128 // wl.N)))]
    for n2 in (wl.N * 2, wl.N // 2, wl.N // 4):
        k2 = total // n2
        s2 = max(1, cus * 128 // n2)
        patterns.append((f"128-column stripes of the same bytes as [{k2},{n2}] x {s2} K-slices", stripes(k2, n2, s2)))
    for name, call in patterns:
        med, best = timed(call)
        out.append({"pattern": name, "us_per_launch": med, "us_per_launch_min": best, "GBps": nbytes / (med * 1e-6) / 1e9})
        log(f"[bench]   {nbytes >> 20} MiB read, {name}: {med:.2f} us per launch ({nbytes / (med * 1e-6) / 1e9:.0f} GB/s)")
    return out


def measure_vendor_gemm(M, K, N, two, steps, warmup):
    """The plain product(s) of a prefill configuration on the vendor GEMM library (torch.matmul, bf16, W stored
    [K, N] as here), without norm, gain or gate: context for the fused kernel's figure, same flop count."""
    import torch
    gen = torch.Generator(device="cuda").manual_seed(0x5EED5000 + N)
    X = torch.randn((M, K), generator=gen, device="cuda").to(torch.bfloat16)
    Ws = [(torch.randn((K, N), generator=gen, device="cuda") / 64).to(torch.bfloat16) for _ in range(2 if two else 1)]
    Ys = [torch.empty((M, N), dtype=torch.bfloat16, device="cuda") for _ in Ws]
    for _ in range(warmup):
        for W, Y in zip(Ws, Ys):
            torch.matmul(X, W, out=Y)
    res = []
    for _ in range(3):
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(steps):
            for W, Y in zip(Ws, Ys):
                torch.matmul(X, W, out=Y)
        e1.record()
        torch.cuda.synchronize()
        res.append(e0.elapsed_time(e1) / steps)
    flops = 2.0 * M * K * N * len(Ws)
    out = {"TFLOPs": flops / (median(res) * 1e-3) / 1e12, "ms": median(res),
           "note": "torch.matmul (vendor GEMM), plain product(s) only"}
    del X, Ws, Ys
    torch.cuda.empty_cache()
    return out


def measure_mid_rows(M, K, N, gated, steps=300, warmup=20):
    """Between decode and prefill: 17 to 512 rows on the decode path's multi-row kernel (W is still what is
    streamed; buffer sets rotate so that it comes from HBM).  Bound: HBM, algorithmic bytes X + g + W (+W2) + Y."""
    import torch
    wl = pi.Workload(f"mid_rows_M{M}_{'gated' if gated else 'plain'}", pi.BF16, M, K, N, gated, 1e-6, 0x5EED3000 + M)
    wbytes = 2 * K * N * (2 if gated else 1)
    r = Runner(wl, max(2, -(-(1 << 30) // wbytes)))
    _, ev_ms = r.timed(steps, warmup)
    nbytes = counted_bytes(wl)
    res = {"workload": wl.name, "dtype": "bf16", "M": M, "K": K, "N": N, "gated": gated, "plan": r.plan, "steps": steps,
           "us_per_call": ev_ms * 1e3, "bound": "hbm", "bytes_per_launch": nbytes,
           "achieved": nbytes / (ev_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
           "frac": nbytes / (ev_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
           "TFLOPs": counted_flops(wl) / (ev_ms * 1e-3) / 1e12}
    log(f"[bench]   {wl.name} K={K} N={N}: {ev_ms * 1e3:.2f} us/call, {res['achieved']:.0f} GB/s = "
        f"{100 * res['frac']:.1f}% of hbm peak, {res['TFLOPs']:.0f} TFLOP/s, path {r.plan['path']} "
        f"tile_m {r.plan['tile_m']} split {r.plan['split_k']} row blocks {r.plan['grid_z']}")
    del r
    torch.cuda.empty_cache()
    return res


def measure_large_decode(M, K, N, steps=40, warmup=6):
    """A decode call whose weights are far larger than any cache (an output projection onto a vocabulary, a wide
    MLP): device-generated bf16 inputs, two weight buffers in turn.  Bound: HBM, algorithmic bytes X + g + W + Y."""
    import torch
    import paper_2604_15272_amd as P
    gen = torch.Generator(device="cuda").manual_seed(0x5EED4000 + N)
    X = torch.randn((M, K), generator=gen, device="cuda").to(torch.bfloat16)
    g = (torch.rand((K,), generator=gen, device="cuda") + 0.5).to(torch.bfloat16)
    Ws = [(torch.randn((K, N), generator=gen, device="cuda") / 64).to(torch.bfloat16) for _ in range(2)]
    Y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    plan = P.prism_plan(P.PRISM_OP_RMSNORM_MATMUL, M, K, N, P.PRISM_BF16)
    P.ensure_workspace(plan["workspace_bytes"])
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    vp, i64 = ctypes.c_void_p, ctypes.c_int64
    args = [(vp(X.data_ptr()), vp(g.data_ptr()), vp(W.data_ptr()), vp(Y.data_ptr()), i64(M), i64(K), i64(N),
             ctypes.c_float(1e-6), ctypes.c_int32(P.PRISM_BF16), stream) for W in Ws]
    fn = P.lib.prism_rmsnorm_matmul
    for i in range(warmup):
        if fn(*args[i % 2]) != 0:
            raise RuntimeError("large decode call failed")
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(steps):
        fn(*args[(warmup + i) % 2])
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / steps
    nbytes = 2 * (M * K + K + K * N + M * N)
    res = {"workload": f"large_decode_M{M}_K{K}_N{N}", "dtype": "bf16", "M": M, "K": K, "N": N, "plan": plan,
           "steps": steps, "us_per_call": ms * 1e3, "bound": "hbm", "bytes_per_launch": nbytes,
           "achieved": nbytes / (ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
           "frac": nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, "data": "synthetic, generated on the device"}
    log(f"[bench]   large decode X[{M},{K}] W[{K},{N}]: {ms * 1e3:.1f} us/call, {res['achieved']:.0f} GB/s = "
        f"{100 * res['frac']:.1f}% of hbm peak, grid {plan['grid_x']} x {plan['grid_y']}")
    del Ws
    torch.cuda.empty_cache()
    return res


def measured_traffic(workload):
    """HBM bytes per launch of the workload's kernel, as measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
    and recorded in profiles/hbm_traffic.md (one line per workload: `traffic <workload> fetch_bytes=...
    write_bytes=...`).  bench.py cannot collect counters itself; None if no measurement is recorded."""
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", "hbm_traffic.md")
    try:
        for line in open(path):
            f = line.split()
            if len(f) >= 4 and f[0] == "traffic" and f[1] == workload:
                kv = dict(x.split("=") for x in f[2:] if "=" in x)
                return {"fetch_bytes": float(kv["fetch_bytes"]), "write_bytes": float(kv["write_bytes"]),
                        "source": "profiles/hbm_traffic.md (rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE, each scaled "
                                  "by its reading for a copy of known size)"}
    except (OSError, KeyError, ValueError):
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--workload", type=int, default=1, help="benchmark configuration index (1..4)")
    ap.add_argument("--no-extra", action="store_true", help="time only the headline workload")
    ap.add_argument("--only-large-decode", action="store_true",
                    help="time only the two decode calls with about 1 GB of weights (for profiling)")
    ap.add_argument("--only-attention", action="store_true",
                    help="time only the paper's attention workloads (for profiling that kernel)")
    ap.add_argument("--only-mid-rows", action="store_true",
                    help="time only the 17-to-512-row shapes (for profiling the multi-row decode kernel)")
    ap.add_argument("--only-running-example", action="store_true",
                    help="time only the softmax -> matmul running example (for profiling that kernel)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle timing")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch one device-to-device copy of 256 MiB (outside the timed region): under "
                         "rocprofv3 --pmc its FETCH_SIZE / WRITE_SIZE reading calibrates the counters")
    a = ap.parse_args()
    if a.gpus != 1:
        log("bench.py measures one GPU: this build has no multi-GPU path (no collectives, no sharding); "
            "run with --gpus 1")
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        log("bench.py needs a GPU")
        sys.exit(2)
    torch.cuda.set_device(0)

    if a.calibrate_copy:
        src = torch.full((COPY_CALIBRATION_BYTES // 2,), 1.0, dtype=torch.bfloat16, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        log(f"[bench] calibration copy: {COPY_CALIBRATION_BYTES} bytes read and as many written")
        del src, dst

    if a.only_running_example:
        print(json.dumps({"running_example": measure_running_example()}), flush=True)
        return
    if a.only_mid_rows:
        print(json.dumps({"mid_rows": [measure_mid_rows(M, K, N, g) for M, K, N, g in
                                       ((32, 4096, 4096, False), (128, 4096, 4096, False), (512, 4096, 4096, False),
                                        (32, 4096, 14336, True))]}), flush=True)
        return
    if a.only_large_decode:
        print(json.dumps({"large_decode": [measure_large_decode(16, 4096, 128256), measure_large_decode(16, 8192, 57344)]}),
              flush=True)
        return
    if a.only_attention:
        print(json.dumps({"attention": [measure_attention(h, qk) for h in (1024, 2048) for qk in (False, True)]}),
              flush=True)
        return
    # Which address units stream slowly is measured on the machine at hand, outside every timed region, and handed
    # to the library (its own default names none): the dispatcher then balances gated decode calls around them.
    import paper_2604_15272_amd as P
    from paper_2604_15272_amd import tune
    det = tune.detect_slow_units(install=True)
    SLOW_UNITS["mask"] = det["mask"]
    log(f"[bench] slow address units on this machine: mask {det['mask']:#06x} (us per unit: "
        f"{' '.join('%.1f' % t for t in det['us'])})")
    head, runner = measure(a.workload, a.steps, a.warmup)
    traffic = measured_traffic(head["workload"])
    stream_patterns = measure_stream_patterns(runner) if head["bound"] == "hbm" else None
    copy_ceiling, mfma_ceiling = measure_copy_ceiling(), measure_mfma_ceiling()
    cu_load_path = measure_cu_load_path()
    log(f"[bench] measured ceilings: device copy {copy_ceiling['GBps']:.0f} GB/s (read + written), matrix pipes alone "
        f"{mfma_ceiling['TFLOPs']:.0f} TFLOP/s")
    out = {
        "metric": METRIC, "value": head["value"], "unit": head["unit"], "n_gpus": 1, "steps": a.steps,
        "warmup": a.warmup, "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "regions": head["regions"], "ms_per_step_min": head["ms_per_step_min"],
        "region_ms_per_step": head["region_wall_ms_per_step"],
        "timing_note": f"{head['regions']} timed regions of exactly `steps` calls each, every region bracketed by "
                       "torch.cuda.synchronize(); ms_per_step and value are the median region's, ms_per_step_min the "
                       "fastest region's",
        "config": {"workload": head["workload"], "M": head["M"], "K": head["K"], "N": head["N"],
                   "gated": head["gated"], "plan": head["plan"], "buffer_sets": head["buffer_sets"],
                   "slow_units_mask": det["mask"], "compute_units": P.prism_diag_cu_count()},
        "roofline": {"bound": head["bound"], "achieved": head["achieved"], "peak": head["peak"],
                     "unit": head["unit"], "frac": head["frac"],
                     "achieved_best_region": head["bytes_per_launch"] / (head["event_ms_per_step_min"] * 1e-3) / 1e9
                     if head["bound"] == "hbm" else head["flops_per_launch"] / (head["event_ms_per_step_min"] * 1e-3) / 1e12,
                     "traffic": None if traffic is None else traffic["fetch_bytes"] + traffic["write_bytes"],
                     "traffic_unit": "bytes per launch", "traffic_detail": traffic,
                     "traffic_note": "not measured in this run: read from profiles/hbm_traffic.md (rocprofv3 --pmc runs "
                                     "of this command)",
                     "algorithmic_bytes_per_launch": head.get("bytes_per_launch"),
                     "kernel": "prism::decode_kernel" if head["bound"] == "hbm" else "prism::prefill_kernel",
                     "kernel_ms_per_launch": head["kernel_ms"],
                     "kernel_ms_per_launch_min": head["event_ms_per_step_min"],
                     "timing": "HIP events around each timed region on the launch stream, divided by the region's "
                               "launches (an average per launch, launch gaps included); median of the regions",
                     "copy_ceiling": copy_ceiling, "mfma_ceiling": mfma_ceiling, "stream_patterns": stream_patterns,
                     "cu_load_path": cu_load_path},
        "slow_units": {"mask": det["mask"], "us_per_unit": det["us"], "median_us": det["median_us"],
                       "note": "tune.detect_slow_units: prism_probe_units, all sixteen units read at once, median workgroup time per unit"},
    }
    if "stream_probe_ms" in head:
        out["roofline"]["stream_probe"] = {
            "ms_per_launch": head["stream_probe_ms"],
            "GBps": head["bytes_per_launch"] / (head["stream_probe_ms"] * 1e-3) / 1e9,
            "note": "prism_probe_stream: W read once with the kernel's access pattern and split, nothing computed"}
    if "cache_hot_GBps" in head:
        out["cache_hot"] = {"GBps": head["cache_hot_GBps"], "kernel_ms_per_launch": head["cache_hot_kernel_ms"],
                            "note": "single buffer set: W is served by the last-level cache, not HBM"}
    if not a.no_cpu:
        out["cpu_baseline"] = cpu_baseline(runner)
        log(f"[bench] oracle: {out['cpu_baseline']['value']:.2f} GB/s on {out['cpu_baseline']['cores']} threads; "
            f"GPU vs oracle worst err {out['cpu_baseline']['gpu_vs_oracle_worst_err']:.2e}")
    del runner
    if not a.no_extra:
        others = []
        for idx, st, wu in ((3, 500, 30), (2, 200, 20), (4, 40, 5)):
            if idx == a.workload:
                continue
            torch.cuda.empty_cache()
            res, r = measure(idx, st, wu)
            del r
            others.append({k: res[k] for k in ("workload", "plan", "steps", "regions", "ms_per_step", "ms_per_step_min",
                                               "event_ms_per_step", "event_ms_per_step_min",
                                               "kernel_ms", "value", "unit", "bound", "achieved", "peak", "frac",
                                               "stream_probe_ms", "equal_slices_kernel_ms", "vendor_gemm") if k in res})
        out["other_workloads"] = others
        torch.cuda.empty_cache()
        log("[bench] the paper's workloads at its shapes, fp16, no gain (output width assumed: see PAPER_SHAPES)")
        out["paper_shapes"] = []
        for name, M, K, N in PAPER_SHAPES:
            out["paper_shapes"].append(measure_paper_shape(name, M, K, N))
            torch.cuda.empty_cache()
        out["running_example"] = measure_running_example()
        torch.cuda.empty_cache()
        log("[bench] 17 to 512 rows (the decode path's multi-row kernel)")
        out["mid_rows"] = [measure_mid_rows(M, K, N, g) for M, K, N, g in
                           ((32, 4096, 4096, False), (128, 4096, 4096, False), (512, 4096, 4096, False),
                            (32, 4096, 14336, True))]
        out["attention"] = [measure_attention(h, qk) for h in (1024, 2048) for qk in (False, True)]
        log("[bench] decode calls with weights of about 1 GB (an output projection onto a vocabulary, a wide layer)")
        out["large_decode"] = [measure_large_decode(16, 4096, 128256), measure_large_decode(16, 8192, 57344)]
        torch.cuda.empty_cache()
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
