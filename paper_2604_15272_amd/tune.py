"""Parameter instantiation at run time: sample valid kernel parameters for a shape, time them, keep the best.

The paper instantiates the symbolic parameters of a program by drawing valid assignments uniformly at
random and profiling each one (Section 5, "parameter instantiation").  The kernels of this library are
correct for every admissible (kernel family, split-K factor, tile / wavefront variant), so the same
procedure applies to them: this module enumerates the admissible assignments of a call by asking the
library's own planner, draws a sample, times each candidate with HIP events on the device, and installs
the fastest in the library's plan table (``prism_plan_table_set``).  Nothing here computes any part of
the operators; the timed work is the library call itself.

    python -m paper_2604_15272_amd.tune --op plain --shape 16 4096 4096 --dtype bf16 --samples 12
"""
import argparse
import json
import random

from . import binding as B

_DECODE_VARIANTS = (4, 8, 16, 32, 64, 36, 68)   # wavefronts (at most 16 rows) or rows per workgroup (more; 36, 68:
                                                # X through LDS, one weight matrix only)
_PACKED_VARIANTS = (104, 108)           # gated, at most 16 rows: 4 or 8 wavefronts on tiles of 64 output columns
_SOFTMAX_MAX_SPLIT = 16
_DECODE_MAX_ROWS = 512                  # the decode path re-reads W per row block: not worth timing beyond
_PLAIN_TILES = (256256, 256192, 256128, 128128, 64064)
_GATED_TILES = (256256, 128256, 128128)
_TORCH_DTYPE = {B.PRISM_F32: "float32", B.PRISM_BF16: "bfloat16", B.PRISM_F16: "float16"}


def detect_slow_units(mbytes=256, repeats=7, threshold=1.18, install=False):
    """Which of the sixteen 128-byte address units of every 2 KiB stream slowly on this machine.

    ``prism_probe_units`` reads a buffer with one workgroup per (unit, run of 2 KiB blocks), all units at the same
    time, and reports every workgroup's duration.  Per unit: the median over its workgroups, then the median over
    ``repeats`` launches (after a warm-up); units that need more than ``threshold`` times the median unit are
    flagged.  Returns ``{"mask", "us", "median_us"}``; with ``install`` the mask goes to ``prism_set_stream_balance``
    (the dispatcher then gives the column tiles of gated decode calls that lie in slow units more K-slices)."""
    import ctypes
    import statistics
    import torch
    nbytes = int(mbytes) << 20
    groups = max(1, B.prism_diag_cu_count() // 16)
    buf = torch.empty(nbytes + 2048, dtype=torch.uint8, device="cuda")
    base = (buf.data_ptr() + 2047) // 2048 * 2048
    buf.fill_(1)
    ticks = torch.zeros(16 * groups, dtype=torch.int64, device="cuda")
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    vp = ctypes.c_void_p
    per_launch = []
    for it in range(repeats + 1):   # the first launch is a warm-up
        st = B.lib.prism_probe_units(vp(base), ctypes.c_uint64(nbytes), groups, vp(ticks.data_ptr()), stream)
        if st != 0:
            raise B.PrismError(st, "prism_probe_units")
        torch.cuda.synchronize()
        t = ticks.cpu().numpy().reshape(groups, 16) * 0.01   # microseconds
        if it > 0:
            per_launch.append([statistics.median(t[:, u].tolist()) for u in range(16)])
    times = [statistics.median([p[u] for p in per_launch]) for u in range(16)]
    med = statistics.median(times)
    mask = sum(1 << u for u, t in enumerate(times) if t > threshold * med)
    if install:
        B.prism_set_stream_balance(mask, 0)
    return {"mask": mask, "us": times, "median_us": med}


def candidates(op, M, K, N, dtype, max_split=64):
    """Every admissible (path, split_k, variant) for this call, as the library's planner sees it."""
    out = []
    softmax = op == B.PRISM_OP_SOFTMAX_MATMUL
    try:
        for path in ((B.PRISM_PATH_SIMPLE, B.PRISM_PATH_ROWS) if softmax else
                     (B.PRISM_PATH_SIMPLE, B.PRISM_PATH_DECODE, B.PRISM_PATH_PREFILL)):
            if path == B.PRISM_PATH_SIMPLE:
                grid = [(0, 0)]
            elif path == B.PRISM_PATH_ROWS:   # softmax: 16 rows per workgroup, or 32 rows and K-slices
                grid = [(1, 16)] + [(s, 32) for s in range(1, min(max_split, _SOFTMAX_MAX_SPLIT) + 1)]
            elif path == B.PRISM_PATH_DECODE:
                if M > _DECODE_MAX_ROWS:
                    continue
                grid = [(s, v) for v in _DECODE_VARIANTS for s in range(1, max_split + 1)]
                if op == B.PRISM_OP_RMSNORM_GATED_MLP:
                    # split 0: the library's own slices, more of them for the tiles in slow address units
                    grid += [(s, v) for v in _PACKED_VARIANTS for s in range(0, max_split + 1)]
            else:
                grid = [(0, t) for t in (_GATED_TILES if op == B.PRISM_OP_RMSNORM_GATED_MLP else _PLAIN_TILES)]
            seen = set()
            for split, variant in grid:
                B.prism_set_override(path, split, variant)
                try:
                    plan = B.prism_plan(op, M, K, N, dtype)
                except B.PrismError:
                    continue
                # the planner clamps split factors: keep one candidate per distinct plan
                key = (plan["path"], plan["split_k"], plan["tile_m"], plan["tile_n"], plan["block"], plan["grid_x"])
                if plan["path"] != path or key in seen:
                    continue
                seen.add(key)
                out.append({"path": path,
                            "split_k": plan["split_k"] if (path in (B.PRISM_PATH_DECODE, B.PRISM_PATH_ROWS) and split) else 0,
                            "variant": variant, "plan": plan})
    finally:
        B.prism_set_override(0, 0, 0)
    return out


def _time_choice(fn, args_sets, steps, warmup):
    import torch
    n = len(args_sets)
    for i in range(warmup):
        st = fn(*args_sets[i % n])
        if st != 0:
            raise B.PrismError(st, "tuned call")
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(steps):
        fn(*args_sets[(warmup + i) % n])
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps * 1e3  # microseconds


def tune(op, M, K, N, dtype=B.PRISM_BF16, samples=12, seed=0, steps=None, install=True, weight_bytes_total=1 << 30,
         verbose=False):
    """Sample up to `samples` admissible assignments (the heuristic's own choice is always one of them),
    time each on random inputs of this shape, and install the fastest in the plan table.

    Weights rotate over enough buffer sets that they are streamed from HBM (at most `weight_bytes_total`).
    Returns {"best": {...}, "default": {...}, "tried": [...]} with microseconds per call.
    """
    import ctypes
    import torch
    gated = op == B.PRISM_OP_RMSNORM_GATED_MLP
    softmax = op == B.PRISM_OP_SOFTMAX_MATMUL
    tdt = getattr(torch, _TORCH_DTYPE[dtype])
    esize = 4 if dtype == B.PRISM_F32 else 2
    nw = 2 if gated else 1
    wbytes = esize * K * N * nw
    sets = max(1, min(1024, weight_bytes_total // max(wbytes, 1)))   # well past the 256 MB last-level cache
    gen = torch.Generator(device="cuda").manual_seed(1234 + seed)
    X = (torch.randn((M, K), generator=gen, device="cuda") * (3.0 if softmax else 1.0)).to(tdt)
    g = (torch.rand((K,), generator=gen, device="cuda") + 0.5).to(tdt)
    Ws = [[(torch.randn((K, N), generator=gen, device="cuda") / K ** 0.5).to(tdt) for _ in range(nw)]
          for _ in range(sets)]
    Y = torch.empty((M, N), dtype=tdt, device="cuda")
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    vp, i64 = ctypes.c_void_p, ctypes.c_int64
    if softmax:
        tail = (vp(Y.data_ptr()), i64(M), i64(K), i64(N), ctypes.c_int32(dtype), stream)
        fn = B.lib.prism_softmax_matmul
        args_sets = [(vp(X.data_ptr()), vp(Ws[s][0].data_ptr())) + tail for s in range(sets)]
    else:
        tail = (vp(Y.data_ptr()), i64(M), i64(K), i64(N), ctypes.c_float(1e-6), ctypes.c_int32(dtype), stream)
        fn = B.lib.prism_rmsnorm_gated_mlp if gated else B.lib.prism_rmsnorm_matmul
        args_sets = [(vp(X.data_ptr()), vp(g.data_ptr()), *[vp(w.data_ptr()) for w in Ws[s]]) + tail
                     for s in range(sets)]

    B.prism_set_override(0, 0, 0)
    saved_entry_plan = B.prism_plan(op, M, K, N, dtype)  # what the library does today (table or heuristic)
    cands = candidates(op, M, K, N, dtype)
    default = next((c for c in cands if c["plan"] == saved_entry_plan), None)
    rng = random.Random(seed)
    rest = [c for c in cands if c is not default and c["path"] != B.PRISM_PATH_SIMPLE]
    rng.shuffle(rest)
    chosen = ([default] if default is not None else []) + rest[:max(0, samples - (default is not None))]

    flops = 2.0 * M * K * N * nw
    if steps is None:
        steps = int(max(20, min(1000, 2e9 / max(flops, 1e6))))
    tried = []
    try:
        for c in chosen:
            B.prism_set_override(c["path"], c["split_k"], c["variant"])
            B.ensure_workspace(B.prism_workspace_bytes(op, M, K, N, dtype))
            try:
                us = min(_time_choice(fn, args_sets, steps, max(5, steps // 10)) for _ in range(3))
            except B.PrismError as e:  # a candidate the planner admits but the launch refuses: skip it
                if verbose:
                    print(f"  {c['path']}/{c['split_k']}/{c['variant']}: {e}")
                continue
            tried.append({"path": c["path"], "split_k": c["split_k"], "variant": c["variant"], "us": us,
                          "plan": c["plan"]})
            if verbose:
                print(f"  path={c['path']} split_k={c['split_k']} variant={c['variant']}: {us:.2f} us")
    finally:
        B.prism_set_override(0, 0, 0)
    if not tried:
        raise RuntimeError("no admissible assignment could be timed")
    best = min(tried, key=lambda t: t["us"])
    dflt = next((t for t in tried if default is not None and t["plan"] == default["plan"]), None)
    if install:
        B.prism_plan_table_set(op, M, K, N, dtype, best["path"], best["split_k"], best["variant"])
        B.ensure_workspace(B.prism_workspace_bytes(op, M, K, N, dtype))
    return {"op": int(op), "M": M, "K": K, "N": N, "dtype": int(dtype), "best": best, "default": dflt, "tried": tried}


def save_table(results, path):
    """Write the winners of several tune() calls as JSON (one entry per shape)."""
    rows = [{k: r[k] for k in ("op", "M", "K", "N", "dtype")} |
            {k: r["best"][k] for k in ("path", "split_k", "variant")} for r in results]
    with open(path, "w") as f:
        json.dump(rows, f, indent=1)


def load_table(path):
    """Install a table written by save_table; returns the number of entries installed."""
    with open(path) as f:
        rows = json.load(f)
    for r in rows:
        B.prism_plan_table_set(r["op"], r["M"], r["K"], r["N"], r["dtype"], r["path"], r["split_k"], r["variant"])
    return len(rows)


def main():
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--op", choices=("plain", "gated", "softmax"), default="plain")
    ap.add_argument("--shape", type=int, nargs=3, metavar=("M", "K", "N"), required=True)
    ap.add_argument("--dtype", choices=("f32", "bf16", "f16"), default="bf16")
    ap.add_argument("--samples", type=int, default=12)
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--save", help="write the winner to this JSON file")
    a = ap.parse_args()
    op = {"plain": B.PRISM_OP_RMSNORM_MATMUL, "gated": B.PRISM_OP_RMSNORM_GATED_MLP,
          "softmax": B.PRISM_OP_SOFTMAX_MATMUL}[a.op]
    dt = {"f32": B.PRISM_F32, "bf16": B.PRISM_BF16, "f16": B.PRISM_F16}[a.dtype]
    r = tune(op, *a.shape, dtype=dt, samples=a.samples, seed=a.seed, verbose=True)
    d = r["default"]
    print(f"best: path={r['best']['path']} split_k={r['best']['split_k']} variant={r['best']['variant']} "
          f"{r['best']['us']:.2f} us" + (f"  (heuristic: {d['us']:.2f} us)" if d else ""))
    if a.save:
        save_table([r], a.save)


if __name__ == "__main__":
    main()
