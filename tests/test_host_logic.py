"""CPU-only checks: the library loads, exports what the header declares, and validates arguments."""
import ctypes
import os
import re

import numpy as np
import pytest


@pytest.fixture(scope="module")
def P(repo_root):
    lib = os.path.join(repo_root, "paper_2604_15272_amd", "libprism.so")
    if not os.path.exists(lib):
        import importlib.util  # by path: importing the package needs the library
        spec = importlib.util.spec_from_file_location("_prism_build",
                                                      os.path.join(repo_root, "paper_2604_15272_amd", "build.py"))
        mod = importlib.util.module_from_spec(spec)
        spec.loader.exec_module(mod)
        mod.build_library()
    import paper_2604_15272_amd as P
    yield P
    P.prism_set_override(0, 0, 0)


def test_every_declared_symbol_is_exported(P, repo_root):
    import glob
    names, per_header = set(), {}
    for h in sorted(glob.glob(os.path.join(repo_root, "include", "*.h"))):
        text = re.sub(r"/\*.*?\*/", "", open(h).read(), flags=re.S)
        per_header[os.path.basename(h)] = set(re.findall(r"\b(prism_[a-z0-9_]+)\s*\(", text))
        names |= per_header[os.path.basename(h)]
    assert {"prism_rmsnorm_matmul", "prism_rmsnorm_gated_mlp", "prism_set_workspace", "prism_plan",
            "prism_rmsnorm_matmul_static"} <= per_header["prism.h"]
    # probes and test hooks live in the diagnostics header, not in the operator boundary
    assert {"prism_probe_stream", "prism_probe_units", "prism_probe_mfma", "prism_probe_linear", "prism_stream_partition_blocks",
            "prism_diag_set_cu_count"} <= per_header["prism_diag.h"]
    assert not any(n.startswith(("prism_probe", "prism_diag")) for n in per_header["prism.h"])
    L = ctypes.CDLL(P.library_path())
    for n in sorted(names):
        assert hasattr(L, n), f"{n} is declared in a header but not exported"
    assert P.prism_version() >= 200


def test_status_strings(P):
    assert P.prism_status_string(0) == "ok"
    assert len({P.prism_status_string(i) for i in range(5)}) == 5


def test_argument_validation_needs_no_device(P):
    L = P.lib
    a = 0x1000  # aligned, never dereferenced: every call below fails before any launch
    ok = lambda **kw: None
    call = lambda X=a, g=a, W=a, Y=a, M=4, K=64, N=64, eps=1e-6, dt=1: L.prism_rmsnorm_matmul(
        X, g, W, Y, M, K, N, eps, dt, None)
    assert call(X=None) == 1 and call(W=None) == 1 and call(Y=None) == 1   # g = None means: no gain tensor
    assert call(X=a + 2) == 1                       # misaligned
    assert call(M=-1) == 1 and call(N=-1) == 1 and call(K=0) == 1 and call(K=-8) == 1
    assert call(eps=-1.0) == 1 and call(eps=float("nan")) == 1 and call(eps=float("inf")) == 1
    assert call(dt=7) == 2
    assert call(M=0) == 0 and call(N=0) == 0        # empty problem: success, no launch
    gcall = lambda W2=a, **kw: L.prism_rmsnorm_gated_mlp(a, a, a, W2, a, 4, 64, 64, 1e-6, 1, None)
    assert gcall(W2=None) == 1
    assert L.prism_rmsnorm_glu(a, a, a, None, a, 4, 64, 64, 1e-6, 1, None) == 1
    assert L.prism_swiglu(a, None, a, a, 4, 64, 64, 1, None) == 1 and L.prism_swiglu(a, a, a, a, 0, 64, 64, 1, None) == 0
    assert L.prism_swiglu(a, a, a, a, 4, 0, 64, 1, None) == 1 and L.prism_swiglu(a, a, a, a, 4, 64, 64, 9, None) == 2


def test_plan_picks_paths_by_shape(P):
    f32, bf16 = P.PRISM_F32, P.PRISM_BF16
    assert P.prism_plan(0, 8, 256, 512, f32)["path"] == P.PRISM_PATH_SIMPLE
    d = P.prism_plan(0, 16, 4096, 4096, bf16)
    assert d["path"] == P.PRISM_PATH_DECODE and d["split_k"] >= 1 and d["grid_x"] == 32
    assert d["workspace_bytes"] == P.prism_workspace_bytes(0, 16, 4096, 4096, bf16)
    p = P.prism_plan(0, 2048, 4096, 6144, bf16)
    assert p["path"] == P.PRISM_PATH_PREFILL and p["workspace_bytes"] == 0
    assert p["grid_x"] == -(-2048 // p["tile_m"]) * -(-6144 // p["tile_n"])
    pg = P.prism_plan(1, 4096, 4096, 14336, bf16)
    assert pg["path"] == P.PRISM_PATH_PREFILL
    assert pg["grid_x"] == -(-4096 // pg["tile_m"]) * -(-14336 // (pg["tile_n"] // 2))
    assert P.prism_plan(0, 16, 4096, 4096, P.PRISM_F16) == d
    assert P.prism_plan(1, 4096, 4096, 14336, P.PRISM_F16) == pg
    assert P.prism_plan(0, 16, 4100, 4096, P.PRISM_F16)["path"] == P.PRISM_PATH_SIMPLE
    # unaligned bf16 shapes go to the plain kernel
    assert P.prism_plan(0, 16, 4100, 4096, bf16)["path"] == P.PRISM_PATH_SIMPLE
    assert P.prism_plan(0, 16, 4096, 4100, bf16)["path"] == P.PRISM_PATH_SIMPLE


def test_override_and_workspace_size(P):
    bf16 = P.PRISM_BF16
    P.prism_set_override(P.PRISM_PATH_DECODE, 4, 8)
    d = P.prism_plan(1, 8, 4096, 14336, bf16)
    assert d["split_k"] == 4 and d["block"] == 512 and d["grid_y"] == 4
    n_tiles = 14336 // 128
    expect = 262144 + -(-n_tiles * 4 * 16 * 4 // 256) * 256 + 4 * 2 * 8 * 14336 * 4
    assert d["workspace_bytes"] == expect
    P.prism_set_override(P.PRISM_PATH_DECODE, 1, 0)
    assert P.prism_plan(0, 16, 4096, 4096, bf16)["workspace_bytes"] == 0
    # a forced path that cannot run the shape is refused, not silently replaced
    P.prism_set_override(P.PRISM_PATH_DECODE, 0, 0)
    with pytest.raises(P.PrismError):
        P.prism_plan(0, 8, 256, 512, P.PRISM_F32)
    with pytest.raises(P.PrismError):
        P.prism_plan(0, 64, 4100, 4096, bf16)
    P.prism_set_override(P.PRISM_PATH_PREFILL, 0, 999999)
    with pytest.raises(P.PrismError):
        P.prism_plan(0, 64, 4096, 4096, bf16)
    P.prism_set_override(0, 0, 0)
    with pytest.raises(P.PrismError):
        P.prism_set_override(9, 0, 0)


def test_probe_arguments_need_no_device(P):
    L, a = P.lib, 0x1000
    pr = lambda W=a, W2=None, K=4096, N=4096, S=8: L.prism_probe_stream(W, W2, K, N, S, None)
    assert pr(W=None) == 1 and pr(W=a + 2) == 1 and pr(W2=a + 2) == 1 and pr(K=0) == 1 and pr(N=0) == 1 and pr(S=0) == 1
    assert pr(N=4100) == 2 and pr(S=129) == 2 and pr(K=1 << 20, N=1 << 20, S=1) == 2


def test_load_probe_arguments_need_no_device(P):
    L, a = P.lib, 0x1000
    pr = lambda base=a, nbytes=P.PROBE_LOADS_BYTES, pattern=0, reps=1, wgs=1, ticks=a: L.prism_probe_loads(
        base, nbytes, pattern, reps, wgs, ticks, None)
    assert pr(base=None) == 1 and pr(ticks=None) == 1 and pr(base=a + 4) == 1 and pr(ticks=a + 4) == 1
    assert pr(nbytes=P.PROBE_LOADS_BYTES - 1) == 1 and pr(pattern=4) == 1 and pr(pattern=-1) == 1
    assert pr(reps=0) == 1 and pr(wgs=0) == 1 and pr(wgs=70000) == 1


def test_softmax_matmul_arguments_and_plan(P):
    L = P.lib
    a = 0x1000
    sm = lambda X=a, W=a, Y=a, M=4, K=64, N=64, dt=1: L.prism_softmax_matmul(X, W, Y, M, K, N, dt, None)
    assert sm(X=None) == 1 and sm(W=None) == 1 and sm(Y=None) == 1 and sm(X=a + 4) == 1
    assert sm(M=-1) == 1 and sm(K=0) == 1 and sm(dt=9) == 2 and sm(M=0) == 0 and sm(N=0) == 0
    op = P.PRISM_OP_SOFTMAX_MATMUL
    p = P.prism_plan(op, 4096, 4096, 128, P.PRISM_F16)   # the paper's shape: 256 workgroups of 16 rows, no slices
    assert (p["path"], p["tile_m"], p["grid_x"], p["grid_y"], p["split_k"], p["workspace_bytes"]) == (P.PRISM_PATH_ROWS, 16, 1, 256, 1, 0)
    p = P.prism_plan(op, 512, 4096, 128, P.PRISM_F16)    # fewer rows: 16 row blocks of 32 rows x 4 K-slices
    assert (p["tile_m"], p["grid_y"], p["grid_z"], p["split_k"]) == (32, 4, 16, 4)
    p = P.prism_plan(op, 512, 16384, 128, P.PRISM_F16)   # deep K: 16 row blocks x 16 K-slices
    assert (p["path"], p["tile_m"], p["grid_x"], p["grid_y"], p["grid_z"], p["split_k"]) == (P.PRISM_PATH_ROWS, 32, 1, 16, 16, 16)
    assert p["workspace_bytes"] == 262144 + 16 * 16 * 32 * 2 * 4 + 16 * 512 * 128 * 4
    assert p["workspace_bytes"] == P.prism_workspace_bytes(op, 512, 16384, 128, P.PRISM_F16)
    p = P.prism_plan(op, 16, 256, 4096, P.PRISM_BF16)    # 16 rows, nothing to split: the 16-row kernel
    assert (p["tile_m"], p["grid_x"], p["grid_y"], p["split_k"], p["workspace_bytes"]) == (16, 32, 1, 1, 0)
    p = P.prism_plan(op, 16, 32768, 128, P.PRISM_BF16)   # 16 rows, deep K: slices
    assert (p["tile_m"], p["split_k"]) == (32, 16)
    p = P.prism_plan(op, 4096, 4096, 4096, P.PRISM_BF16)  # many rounds of workgroups: 32 rows (half the W per row), no slices
    assert (p["tile_m"], p["split_k"], p["grid_x"], p["grid_z"], p["workspace_bytes"]) == (32, 1, 32, 128, 0)
    p = P.prism_plan(op, 16, 4096, 4096, P.PRISM_BF16)   # 16 rows against 32 MB of W: slices, as in the decode kernel
    assert (p["tile_m"], p["split_k"]) == (32, 4)
    try:
        P.prism_set_override(P.PRISM_PATH_ROWS, 0, 16)
        p = P.prism_plan(op, 4096, 4096, 128, P.PRISM_F16)
        assert (p["tile_m"], p["grid_y"], p["split_k"], p["workspace_bytes"]) == (16, 256, 1, 0)
        P.prism_set_override(P.PRISM_PATH_ROWS, 5, 32)
        assert P.prism_plan(op, 4096, 4096, 128, P.PRISM_F16)["split_k"] == 5
        for bad in ((P.PRISM_PATH_ROWS, 2, 16), (P.PRISM_PATH_ROWS, 17, 32), (P.PRISM_PATH_ROWS, 0, 64),
                    (P.PRISM_PATH_SIMPLE, 2, 0)):
            P.prism_set_override(*bad)
            with pytest.raises(P.PrismError):
                P.prism_plan(op, 4096, 4096, 128, P.PRISM_F16)
    finally:
        P.prism_set_override(0, 0, 0)
    assert P.prism_plan(op, 8, 256, 512, P.PRISM_F32)["path"] == P.PRISM_PATH_SIMPLE
    assert P.prism_plan(op, 8, 100, 36, P.PRISM_BF16)["path"] == P.PRISM_PATH_SIMPLE
    # the kernel families of the other operators do not apply, and the softmax kernel applies to nothing else
    for path in (P.PRISM_PATH_DECODE, P.PRISM_PATH_PREFILL):
        P.prism_set_override(path, 0, 0)
        with pytest.raises(P.PrismError):
            P.prism_plan(op, 16, 512, 128, P.PRISM_BF16)
    P.prism_set_override(P.PRISM_PATH_ROWS, 0, 0)
    with pytest.raises(P.PrismError):
        P.prism_plan(0, 16, 512, 128, P.PRISM_BF16)
    with pytest.raises(P.PrismError):
        P.prism_plan(op, 8, 256, 512, P.PRISM_F32)
    P.prism_set_override(0, 0, 0)


def test_attention_arguments_and_plan(P):
    L = P.lib
    a = 0x1000
    at = lambda Q=a, K=a, V=a, O=a, B=2, G=8, H=64, D=128, scale=1.0, eps=1e-6, dt=1: L.prism_gqa_decode_attention(
        Q, K, V, O, B, G, H, D, scale, 0, eps, dt, None)
    assert at(Q=None) == 1 and at(K=None) == 1 and at(V=None) == 1 and at(O=None) == 1 and at(K=a + 8) == 1
    assert at(H=0) == 1 and at(D=0) == 1 and at(B=-1) == 1 and at(eps=-1.0) == 1 and at(scale=float("nan")) == 1
    assert at(dt=9) == 2 and at(D=2048) == 2 and at(B=0) == 0 and at(G=0) == 0
    f16 = P.PRISM_F16
    p = P.prism_attention_plan(2, 8, 2048, 128, f16)
    assert p["path"] == P.PRISM_PATH_ATTENTION and p["split_k"] == 16 and p["tile_n"] == 128 and p["grid_y"] == 2
    assert p["workspace_bytes"] == 262144 + 2 * 16 * 16 * (2 + 128) * 4
    short = P.prism_attention_plan(2, 8, 1024, 128, f16)
    assert short["split_k"] == 8 and short["tile_n"] == 128
    assert P.prism_attention_plan(2, 8, 100, 128, f16)["split_k"] == 1
    assert P.prism_attention_plan(2, 8, 100, 128, f16)["workspace_bytes"] == 0
    big = P.prism_attention_plan(1, 8, 65536, 128, f16)
    assert big["split_k"] == 64 and big["tile_n"] == 1024
    mid = P.prism_attention_plan(1, 8, 8192, 128, f16)
    assert mid["split_k"] == 32 and mid["tile_n"] == 256
    assert P.prism_attention_plan(1, 8, 1536, 128, f16)["split_k"] == 8
    # never more workgroups than CUs over all batch entries, but up to four slices for long contexts
    assert P.prism_attention_plan(32, 8, 2048, 128, f16)["split_k"] == 8
    assert P.prism_attention_plan(32, 8, 16384, 128, f16)["split_k"] == 8
    assert P.prism_attention_plan(64, 16, 4096, 128, f16)["split_k"] == 4
    assert P.prism_attention_plan(300, 8, 1024, 128, f16)["split_k"] == 1
    assert P.prism_attention_plan(300, 8, 16384, 128, f16)["split_k"] == 4
    assert P.prism_attention_plan(1, 8, 4096, 128, f16)["split_k"] == 16
    # what the matrix-core kernel does not cover goes to the plain kernel
    for shape in ((2, 8, 2048, 64), (2, 17, 2048, 128)):
        assert P.prism_attention_plan(*shape, f16)["path"] == P.PRISM_PATH_SIMPLE
    assert P.prism_attention_plan(2, 8, 2048, 128, P.PRISM_F32)["path"] == P.PRISM_PATH_SIMPLE
    P.prism_set_override(P.PRISM_PATH_ATTENTION, 0, 0)
    with pytest.raises(P.PrismError):
        P.prism_attention_plan(2, 8, 2048, 64, f16)
    P.prism_set_override(P.PRISM_PATH_ATTENTION, 3, 0)
    s3 = P.prism_attention_plan(2, 8, 2048, 128, f16)
    assert s3["split_k"] == 3 and s3["tile_n"] == 704
    P.prism_set_override(P.PRISM_PATH_DECODE, 0, 0)
    with pytest.raises(P.PrismError):
        P.prism_attention_plan(2, 8, 2048, 128, f16)
    P.prism_set_override(0, 0, 0)


def test_decode_plan_for_more_than_sixteen_rows(P):
    """Several 16-row groups per workgroup, further rows as row blocks in the grid's z."""
    bf16 = P.PRISM_BF16
    d = P.prism_plan(0, 17, 4096, 4096, bf16)
    assert (d["path"], d["tile_m"], d["grid_x"], d["grid_z"], d["block"]) == (P.PRISM_PATH_DECODE, 32, 32, 1, 512)
    assert d["grid_y"] == d["split_k"] == 8
    # the time model of the three candidates (32 rows, 64 rows, prefill kernel) decides:
    d = P.prism_plan(0, 100, 4096, 4096, bf16)    # 64 rows in four K-slices beat 32 rows in two (17.9 against 21.0 us)
    assert (d["path"], d["tile_m"], d["grid_z"], d["split_k"]) == (P.PRISM_PATH_DECODE, 64, 2, 4)
    n_tiles, rb, S = 32, 2, 4
    assert d["workspace_bytes"] == 262144 + n_tiles * rb * S * 64 * 4 + S * 100 * 4096 * 4
    d = P.prism_plan(0, 48, 4096, 4096, bf16)     # few rows: 64 rows would need eight slices; 32 rows in four
    assert (d["path"], d["tile_m"], d["grid_z"], d["split_k"]) == (P.PRISM_PATH_DECODE, 32, 2, 4)
    d = P.prism_plan(0, 100, 14336, 4096, bf16)
    assert (d["path"], d["tile_m"], d["grid_z"], d["split_k"]) == (P.PRISM_PATH_DECODE, 64, 2, 4)
    assert P.prism_plan(0, 512, 4096, 4096, bf16)["path"] == P.PRISM_PATH_DECODE
    assert P.prism_plan(0, 512, 4096, 6144, bf16)["path"] == P.PRISM_PATH_PREFILL   # 384 workgroups: two rounds
    d = P.prism_plan(0, 100, 1024, 1024, bf16)    # shallow K: 16 K steps of the tiled kernel cost more than 8 K-blocks
    assert (d["path"], d["tile_m"], d["split_k"]) == (P.PRISM_PATH_DECODE, 32, 4)
    g = P.prism_plan(1, 192, 8192, 4096, bf16)    # gated, deep K: the prefill kernel's 128 K steps lose (131 against 76 us)
    assert (g["path"], g["tile_m"], g["grid_z"], g["split_k"]) == (P.PRISM_PATH_DECODE, 64, 3, 2)   # 81 us; 32 rows: 76
    # gated, 33 to 64 rows against the wide matrices: two row blocks of 32 would each stream the 235 MB of weights
    # (58 to 60 us); 64 rows in two K-slices read them once (52 to 58 us)
    g = P.prism_plan(1, 64, 4096, 14336, bf16)
    assert (g["path"], g["tile_m"], g["grid_z"], g["split_k"]) == (P.PRISM_PATH_DECODE, 64, 1, 2)
    g = P.prism_plan(1, 17, 8192, 28672, bf16)    # 940 MB of weights: the tiled kernel streams them slower (193 against 154 us)
    assert (g["path"], g["tile_m"], g["grid_z"], g["split_k"]) == (P.PRISM_PATH_DECODE, 32, 1, 1)
    g = P.prism_plan(1, 32, 4096, 14336, bf16)
    assert (g["path"], g["tile_m"], g["grid_z"], g["split_k"]) == (P.PRISM_PATH_DECODE, 32, 1, 2)
    assert P.prism_plan(1, 100, 4096, 14336, bf16)["path"] == P.PRISM_PATH_PREFILL
    # the variant picks the rows per workgroup; wavefront counts belong to the 16-row kernel
    try:
        P.prism_set_override(P.PRISM_PATH_DECODE, 3, 32)
        d = P.prism_plan(0, 100, 4096, 4096, bf16)
        assert (d["tile_m"], d["grid_z"], d["split_k"]) == (32, 4, 3)
        with pytest.raises(P.PrismError):
            P.prism_plan(0, 16, 4096, 4096, bf16)
        P.prism_set_override(P.PRISM_PATH_DECODE, 0, 64)
        assert P.prism_plan(1, 100, 4096, 14336, bf16)["grid_z"] == 2
        P.prism_set_override(P.PRISM_PATH_DECODE, 0, 32)
        assert P.prism_plan(1, 100, 4096, 14336, bf16)["grid_z"] == 4
        P.prism_set_override(P.PRISM_PATH_DECODE, 0, 4)
        with pytest.raises(P.PrismError):
            P.prism_plan(0, 100, 4096, 4096, bf16)
        # forced, the decode path takes any row count whose counters fit the workspace header
        P.prism_set_override(P.PRISM_PATH_DECODE, 0, 0)
        assert P.prism_plan(0, 5000, 4096, 4096, bf16)["grid_z"] == -(-5000 // 64)
        with pytest.raises(P.PrismError):
            P.prism_plan(0, 200000, 1024, 8192, bf16)   # 3125 row blocks x 64 column tiles of counters
    finally:
        P.prism_set_override(0, 0, 0)
    # beyond a few hundred rows the tiled kernel takes over
    assert P.prism_plan(0, 2048, 4096, 4096, bf16)["path"] == P.PRISM_PATH_PREFILL
    assert P.prism_plan(1, 2048, 4096, 14336, bf16)["path"] == P.PRISM_PATH_PREFILL


def test_decode_rows_plan_with_more_tiles_than_cus(P):
    """A single row block of the multi-row kernel may run in several rounds; more row blocks may not."""
    bf16 = P.PRISM_BF16
    pl = lambda op, M, K, N: (lambda d: (d["path"], d["tile_m"], d["grid_x"], d["grid_y"], d["grid_z"]))(P.prism_plan(op, M, K, N, bf16))
    assert pl(0, 32, 4096, 40960) == (P.PRISM_PATH_DECODE, 32, 320, 1, 1)
    assert pl(0, 64, 8192, 36864) == (P.PRISM_PATH_DECODE, 64, 288, 2, 1)     # 153 us; the tiled kernel 167 to 178
    assert pl(0, 64, 4096, 33280) == (P.PRISM_PATH_DECODE, 64, 260, 2, 1)     # 87 us; the tiled kernel 78 to 95
    assert pl(1, 32, 4096, 33280) == (P.PRISM_PATH_DECODE, 32, 260, 2, 1)
    assert pl(0, 128, 4096, 40960)[0] == P.PRISM_PATH_PREFILL
    assert pl(1, 64, 4096, 33280) == (P.PRISM_PATH_DECODE, 64, 260, 2, 1)     # 159 us; the tiled kernel 151 to 176
    assert pl(1, 128, 4096, 33280)[0] == P.PRISM_PATH_PREFILL


def test_plans_of_random_shapes_are_consistent(P):
    """Whatever the dispatcher picks: the grid covers the problem, the split leaves no empty slice, the workspace
    is what the kernels index, and the query functions agree with each other."""
    import random
    rng = random.Random(20260415)
    for _ in range(4000):
        op = rng.choice((0, 1, 2))
        dt = rng.choice((P.PRISM_F32, P.PRISM_BF16, P.PRISM_F16))
        M = rng.choice((1, 7, 16, 17, 31, 32, 33, 64, 65, 100, 128, 129, 256, 300, 512, 513, 2048, 5000))
        K = rng.choice((8, 64, 72, 100, 256, 1000, 1024, 2048, 2056, 4096, 14336, 32768))
        N = rng.choice((8, 16, 36, 128, 136, 264, 1024, 4096, 6144, 14336, 128256))
        p = P.prism_plan(op, M, K, N, dt)
        what = f"op={op} dt={dt} M={M} K={K} N={N} plan={p}"
        assert p["workspace_bytes"] == P.prism_workspace_bytes(op, M, K, N, dt), what
        assert 1 <= p["split_k"] <= -(-K // 32), what
        assert (p["workspace_bytes"] > 0) == (p["split_k"] > 1), what
        fast = dt != P.PRISM_F32 and K % 8 == 0 and N % 8 == 0
        if not fast:
            assert p["path"] == P.PRISM_PATH_SIMPLE, what
        cols = p["tile_n"] // 2 if (op == 1 and p["path"] == P.PRISM_PATH_PREFILL) else p["tile_n"]
        if p["path"] == P.PRISM_PATH_PREFILL:
            assert p["grid_x"] == -(-M // p["tile_m"]) * -(-N // cols), what
        elif p["path"] == P.PRISM_PATH_DECODE or (p["path"] == P.PRISM_PATH_ROWS and p["tile_m"] == 32):
            tiles = -(-N // p["tile_n"])
            if p["path"] == P.PRISM_PATH_DECODE and p["tile_n"] == 64 and N <= 2048:
                # gated, packed tiles, narrow output: equal K-slices
                assert op == 1 and M <= 16, what
                assert (p["grid_x"], p["grid_y"], max(1, p["grid_z"])) == (tiles, p["split_k"], 1), what
            elif p["path"] == P.PRISM_PATH_DECODE and p["tile_n"] == 64:
                # gated, packed tiles, more K-slices for the tiles in slow units: every workgroup on its own CU
                assert op == 1 and M <= 16 and N % 1024 == 0 and p["grid_y"] == 1, what
                assert tiles < p["grid_x"] <= 256 and 2 <= p["split_k"] <= 32, what
                assert (p["grid_x"] - tiles // 8 * p["split_k"]) % (tiles - tiles // 8) == 0, what
            elif p["path"] == P.PRISM_PATH_DECODE and p["tile_m"] == 16 and p["grid_y"] == 1 and p["grid_x"] != tiles:
                # weighted partition: 256 workgroups where tiles x slices would have been more
                assert p["grid_x"] == 256 and tiles < 256 and 2 <= p["split_k"] <= 32, what
            else:
                assert (p["grid_x"], p["grid_y"], max(1, p["grid_z"])) == (tiles, p["split_k"], -(-M // p["tile_m"])), what
            assert p["tile_m"] in (16, 32, 64) and (p["tile_m"] == 16) == (M <= 16 and op != 2), what
            if p["split_k"] > 1:
                G = 2 if op == 1 else 1
                part = (2 * 32 if op == 2 else p["tile_m"]) * 4
                ss = -(-(tiles * -(-M // p["tile_m"]) * p["split_k"] * part) // 256) * 256
                assert p["workspace_bytes"] == 262144 + ss + p["split_k"] * G * M * N * 4, what
        else:
            assert (p["grid_x"], p["grid_y"]) == (-(-N // p["tile_n"]), -(-M // p["tile_m"])), what


def _partition(P, G, kblocks, n_tiles, slow):
    """owner[tile] = list of (wg, first, count) with count > 0, in workgroup order."""
    owner = [[] for _ in range(n_tiles)]
    for wg in range(G):
        for t in range(n_tiles):
            first, count = P.prism_stream_partition_blocks(G, kblocks, n_tiles, slow, wg, t)
            if count:
                owner[t].append((wg, first, count))
    return owner


def test_weighted_partition_deals_every_k_block_out_once(P):
    """The integer functions the decode kernel runs (through their host-side entry point): every K-block of every
    tile belongs to exactly one workgroup, a tile's sharers are consecutive workgroups whose runs follow one another,
    equal weights give shares that differ by at most one block, and slow tiles get 5/4 as many sharers."""
    rng = np.random.Generator(np.random.Philox(77))
    cases = [(256, 128, 86, 0), (256, 128, 112, 0x22), (64, 32, 8, 0x22), (1, 5, 3, 0), (7, 1, 7, 0x81)]
    cases += [(int(rng.integers(1, 70)), int(rng.integers(1, 90)), int(rng.integers(1, 40)), int(rng.choice([0, 0x22, 0x44, 0xFF, 0x01])))
              for _ in range(25)]
    for G, kblocks, n_tiles, slow in cases:
        # the dispatcher keeps a share at four K-blocks or more; five weight units already give every workgroup a block
        G = max(1, min(G, sum(kblocks * (5 if (slow >> (t % 8)) & 1 else 4) for t in range(n_tiles)) // 5))
        what = f"G={G} kblocks={kblocks} n_tiles={n_tiles} slow={slow:#x}"
        owner = _partition(P, G, kblocks, n_tiles, slow)
        per_wg = np.zeros(G, dtype=np.int64)
        tiles_of_wg = [set() for _ in range(G)]
        for t, runs in enumerate(owner):
            assert runs, what
            nxt = 0
            for i, (wg, first, count) in enumerate(runs):
                assert first == nxt, (what, t, runs)
                nxt = first + count
                if i:
                    assert wg == runs[i - 1][0] + 1, (what, t, runs)   # neighbours in the grid
                per_wg[wg] += count * (5 if (slow >> (t % 8)) & 1 else 4)
                tiles_of_wg[wg].add(t)
            assert nxt == kblocks, (what, t, runs)
            assert len(runs) <= 32 or G > 32 * n_tiles, what
        T = sum(kblocks * (5 if (slow >> (t % 8)) & 1 else 4) for t in range(n_tiles))
        assert per_wg.sum() == T, what
        # shares in weight units: equal up to one K-block either way
        assert per_wg.max() - per_wg.min() <= 2 * 5 + 1, (what, per_wg)
        if T // G < 4 * kblocks:
            assert max(len(ts) for ts in tiles_of_wg) <= 2, what
    # weights (s, s') over G = the sum of s or s' over the tiles: every share is a whole slice of one tile
    G = 224 * 1 + 28
    for wg in range(G):
        runs = [(t,) + P.prism_stream_partition_blocks(G, 128, 224, 0x0808, wg, t, period=16, w_fast=1, w_slow=2)
                for t in range(224)]
        runs = [r for r in runs if r[2]]
        assert len(runs) == 1, (wg, runs)
        t, first, count = runs[0]
        assert (count, first % 64) == ((64, 0) if t % 16 in (3, 11) else (128, 0)), (wg, runs)
    # what the dispatcher relies on: a share below one tile's weight meets at most ceil(w * kblocks / q) + 1 workgroups
    owner = _partition(P, 256, 128, 112, 0x22)
    q = (112 * 4 + 28) * 128 // 256
    assert max(len(r) for r in owner) <= -(-5 * 128 // q) + 1
    slow_n = np.mean([len(owner[t]) for t in range(112) if t % 8 in (1, 5)])
    fast_n = np.mean([len(owner[t]) for t in range(112) if t % 8 not in (1, 5)])
    assert slow_n > fast_n


def test_plan_uses_the_partition_when_the_grid_would_not_fit(P):
    bf16 = P.PRISM_BF16
    # the nearest slice count would need a second round for two workgroups (86 x 3 = 258): one slice fewer
    assert (lambda d: (d["grid_x"], d["grid_y"], d["split_k"]))(P.prism_plan(0, 16, 4096, 11008, bf16)) == (86, 2, 2)
    assert (lambda d: (d["grid_x"], d["grid_y"]))(P.prism_plan(0, 16, 4096, 7168, bf16)) == (56, 4)
    assert (lambda d: (d["grid_x"], d["grid_y"]))(P.prism_plan(0, 16, 4096, 4096, bf16)) == (32, 8)
    # 144 tiles: one slice leaves 112 CUs idle, two make a second round of 32 workgroups: three; shallow K: one
    assert (lambda d: (d["grid_x"], d["grid_y"]))(P.prism_plan(0, 16, 4096, 18432, bf16)) == (144, 3)
    assert (lambda d: (d["grid_x"], d["grid_y"]))(P.prism_plan(0, 16, 2048, 18432, bf16)) == (144, 1)
    assert (lambda d: (d["grid_x"], d["grid_y"]))(P.prism_plan(0, 16, 4096, 20480, bf16)) == (160, 1)
    # between one and two rounds of workgroups: slices that fill their rounds (260, 320, 384 tiles), none from 394 on
    for N, grid in ((33280, (260, 4)), (40960, (320, 4)), (49152, (384, 2)), (51200, (400, 1)), (57344, (448, 1)),
                    (65664, (513, 1))):
        assert (lambda d: (d["grid_x"], d["grid_y"]))(P.prism_plan(0, 16, 4096, N, bf16)) == grid, N
    assert P.prism_plan(0, 16, 4096, 57344, bf16)["block"] == 256          # unsplit plain calls: four wavefronts
    assert P.prism_plan(1, 8, 4096, 57344, bf16)["block"] == 512
    # the two-pass partition is an option: 256 workgroups with equal shares
    P.prism_set_stream_balance(0x0808, 1)
    try:
        p = P.prism_plan(0, 16, 4096, 18432, bf16)
        assert (p["path"], p["grid_x"], p["grid_y"], p["block"]) == (P.PRISM_PATH_DECODE, 256, 1, 512)
        q = 144 * 4 * 128 // 256
        assert p["split_k"] == -(-4 * 128 // q) + 1
        ss = -(-(144 * p["split_k"] * 16 * 4) // 256) * 256
        assert p["workspace_bytes"] == 262144 + ss + p["split_k"] * 16 * 18432 * 4
        assert P.prism_plan(0, 16, 4096, 11008, bf16)["grid_y"] == 2          # only for 129 to 159 tiles
        P.prism_set_override(P.PRISM_PATH_DECODE, 3, 0)                        # a forced split keeps the grid
        try:
            assert P.prism_plan(0, 16, 4096, 18432, bf16)["grid_y"] == 3
        finally:
            P.prism_set_override(0, 0, 0)
    finally:
        P.prism_set_stream_balance()
    for bad in ((0x10000, 1), (-1, 1), (0, 4), (0, -1)):
        with pytest.raises(P.PrismError):
            P.prism_set_stream_balance(*bad)
    with pytest.raises(P.PrismError):
        P.prism_stream_partition_blocks(4, 8, 8, 0, 4, 0)
    with pytest.raises(P.PrismError):
        P.prism_stream_partition_blocks(4, 8, 8, 0, 0, 0, period=12)


def test_gated_decode_plan_packs_and_balances(P):
    """Gated calls with at most 16 rows: tiles of 64 output columns with more K-slices for the tiles in slow units,
    when that puts at least as many workgroups to work as the two-tile form would."""
    bf16 = P.PRISM_BF16
    # no unit is slow until the caller says so: two tiles per workgroup, equal slices
    assert (lambda d: (d["tile_n"], d["grid_x"], d["grid_y"]))(P.prism_plan(1, 8, 4096, 14336, bf16)) == (128, 112, 2)
    P.prism_set_stream_balance(0x0808, 0)                 # units 3 and 11, as measured on the MI355X at hand
    try:
        _gated_decode_plan_with_slow_units(P, bf16)
    finally:
        P.prism_set_stream_balance()


def _gated_decode_plan_with_slow_units(P, bf16):
    p = P.prism_plan(1, 8, 4096, 14336, bf16)             # the gated decode configuration: 224 tiles, 28 of them slow
    assert (p["path"], p["tile_n"], p["grid_x"], p["grid_y"], p["split_k"]) == (P.PRISM_PATH_DECODE, 64, 224 + 28, 1, 2)
    ss = -(-(224 * 2 * 16 * 4) // 256) * 256
    assert p["workspace_bytes"] == 262144 + ss + 2 * 2 * 8 * 14336 * 4
    assert P.prism_plan(1, 8, 4096, 7168, bf16)["grid_x"] == 112 * 2 + 14            # 2 slices, 3 for the slow tiles
    assert P.prism_plan(1, 8, 4096, 7168, bf16)["split_k"] == 3
    # fewer workgroups than the two-tile grid would have: two tiles
    assert (lambda d: (d["tile_n"], d["grid_x"], d["grid_y"]))(P.prism_plan(1, 8, 4096, 4096, bf16)) == (128, 32, 8)
    assert (lambda d: (d["tile_n"], d["grid_x"], d["grid_y"]))(P.prism_plan(1, 4, 8192, 8192, bf16)) == (128, 64, 4)
    # no room for more slices (256 tiles of 64 columns), N not a multiple of 1024, more than 16 rows: two tiles
    assert P.prism_plan(1, 8, 4096, 16384, bf16)["tile_n"] == 128
    assert P.prism_plan(1, 8, 4096, 14336 + 128, bf16)["tile_n"] == 128
    assert P.prism_plan(1, 24, 4096, 14336, bf16)["tile_n"] == 128
    # no slow units named, or a forced split: two tiles; the packed variants by name, with any split
    P.prism_set_stream_balance(0, 1)
    try:
        assert (lambda d: (d["tile_n"], d["grid_x"], d["grid_y"]))(P.prism_plan(1, 8, 4096, 14336, bf16)) == (128, 112, 2)
    finally:
        P.prism_set_stream_balance(0x0808, 0)
    for variant, split, expect in ((0, 2, (128, 112, 2, 512)), (108, 3, (64, 224, 3, 512)), (104, 1, (64, 224, 1, 256)),
                                   (108, 0, (64, 252, 1, 512))):
        P.prism_set_override(P.PRISM_PATH_DECODE, split, variant)
        try:
            d = P.prism_plan(1, 8, 4096, 14336, bf16)
            assert (d["tile_n"], d["grid_x"], d["grid_y"], d["block"]) == expect, (variant, split, d)
        finally:
            P.prism_set_override(0, 0, 0)
    for variant in (104, 116, 100):
        P.prism_set_override(P.PRISM_PATH_DECODE, 0, variant)
        try:
            with pytest.raises(P.PrismError):
                P.prism_plan(0 if variant == 104 else 1, 8, 4096, 14336, bf16)    # not gated; 16 wavefronts; no such count
        finally:
            P.prism_set_override(0, 0, 0)


def test_plans_follow_the_number_of_compute_units(P):
    """Grids are sized by the device's compute units (256 where there is no device to ask); the test hook plans for
    other counts: a part with 128 units gets half the K-slices, one with 304 more."""
    bf16 = P.PRISM_BF16
    base = P.prism_diag_cu_count()
    assert base >= 1
    try:
        P.prism_diag_set_cu_count(256)
        assert (lambda d: (d["grid_x"], d["grid_y"]))(P.prism_plan(0, 16, 4096, 4096, bf16)) == (32, 8)
        assert P.prism_plan(0, 256, 4096, 4096, bf16)["path"] == P.PRISM_PATH_DECODE      # 32 tiles x 8 row blocks fit
        P.prism_diag_set_cu_count(128)
        assert P.prism_diag_cu_count() == 128
        assert (lambda d: (d["grid_x"], d["grid_y"]))(P.prism_plan(0, 16, 4096, 4096, bf16)) == (32, 4)
        assert (lambda d: (d["grid_x"], d["grid_y"]))(P.prism_plan(0, 16, 4096, 7168, bf16)) == (56, 2)
        assert P.prism_plan(0, 512, 4096, 4096, bf16)["path"] == P.PRISM_PATH_PREFILL     # 32 x 8 row blocks do not fit
        P.prism_diag_set_cu_count(304)
        assert (lambda d: (d["grid_x"], d["grid_y"]))(P.prism_plan(0, 16, 8192, 4096, bf16)) == (32, 8)   # never more than 8
        assert (lambda d: (d["grid_x"], d["grid_y"]))(P.prism_plan(0, 16, 4096, 11008, bf16)) == (86, 3)  # 258 fit 304
        for bad in (-1, 70000):
            with pytest.raises(P.PrismError):
                P.prism_diag_set_cu_count(bad)
    finally:
        P.prism_diag_set_cu_count(0)
    assert P.prism_diag_cu_count() == base


def test_shapes_past_the_32_bit_offsets_take_the_plain_kernel(P):
    """2 GiB of W is what the buffer addressing of the matrix-core kernels covers; beyond, the plan says so."""
    bf16 = P.PRISM_BF16
    assert P.prism_plan(0, 1024, 16384, 65536, bf16)["path"] == P.PRISM_PATH_SIMPLE     # W = 2 GiB
    assert P.prism_plan(0, 1024, 16384, 65528, bf16)["path"] == P.PRISM_PATH_PREFILL    # just below
    big = P.prism_plan(0, 16, 16384, 131072, bf16)                                    # W = 4 GiB: decode offsets are
    assert big["path"] == P.PRISM_PATH_DECODE and big["split_k"] == 4                 # per slice, so it takes 4 slices


def test_plan_table_precedence_and_validation(P):
    """Heuristic < plan table < override; an assignment that cannot run the shape is refused when it is set."""
    bf16 = P.PRISM_BF16
    P.prism_plan_table_clear()
    base = P.prism_plan(0, 16, 4096, 4096, bf16)
    try:
        P.prism_plan_table_set(0, 16, 4096, 4096, bf16, P.PRISM_PATH_DECODE, 4, 4)
        assert P.prism_plan_table_size() == 1
        t = P.prism_plan(0, 16, 4096, 4096, bf16)
        assert t["split_k"] == 4 and t["block"] == 256 and t["grid_y"] == 4
        assert P.prism_workspace_bytes(0, 16, 4096, 4096, bf16) == t["workspace_bytes"]
        # exactly this key only: other shapes, the gated op and other storage types keep the heuristic
        assert P.prism_plan(0, 8, 4096, 4096, bf16)["split_k"] == P.prism_plan(0, 8, 4096, 4096, P.PRISM_F16)["split_k"]
        assert P.prism_plan(0, 16, 4096, 4096, P.PRISM_F16) == base
        assert P.prism_plan(1, 16, 4096, 4096, bf16)["block"] == 512
        # the override still wins
        P.prism_set_override(P.PRISM_PATH_DECODE, 2, 8)
        assert P.prism_plan(0, 16, 4096, 4096, bf16)["split_k"] == 2
        P.prism_set_override(0, 0, 0)
        # replacing an entry does not grow the table
        P.prism_plan_table_set(0, 16, 4096, 4096, bf16, P.PRISM_PATH_PREFILL, 0, 128128)
        assert P.prism_plan_table_size() == 1 and P.prism_plan(0, 16, 4096, 4096, bf16)["tile_m"] == 128
        # refused: four wavefronts for 64 rows, an unknown tile, a negative split
        for bad in ((0, 64, 4096, 4096, bf16, P.PRISM_PATH_DECODE, 0, 4), (0, 64, 4096, 4096, bf16, P.PRISM_PATH_PREFILL, 0, 999),
                    (0, 16, 4096, 4096, bf16, P.PRISM_PATH_DECODE, -1, 0), (0, 0, 4096, 4096, bf16, P.PRISM_PATH_DECODE, 1, 8)):
            with pytest.raises(P.PrismError):
                P.prism_plan_table_set(*bad)
        assert P.prism_plan_table_size() == 1
        # capacity: 256 entries, then refused
        for i in range(255):
            P.prism_plan_table_set(0, 16, 4096, 8 * (i + 1), bf16, P.PRISM_PATH_DECODE, 1, 8)
        assert P.prism_plan_table_size() == 256
        with pytest.raises(P.PrismError):
            P.prism_plan_table_set(0, 16, 4096, 8 * 1000, bf16, P.PRISM_PATH_DECODE, 1, 8)
    finally:
        P.prism_plan_table_clear()
        P.prism_set_override(0, 0, 0)
    assert P.prism_plan_table_size() == 0 and P.prism_plan(0, 16, 4096, 4096, bf16) == base


def test_tuner_enumerates_admissible_assignments(P):
    """The candidate list comes from the library's own planner: every entry is a plan it accepts."""
    from paper_2604_15272_amd import tune
    c = tune.candidates(0, 16, 2048, 1024, P.PRISM_BF16, max_split=16)
    paths = {x["path"] for x in c}
    assert paths == {P.PRISM_PATH_SIMPLE, P.PRISM_PATH_DECODE, P.PRISM_PATH_PREFILL}
    dec = [x for x in c if x["path"] == P.PRISM_PATH_DECODE]
    assert {x["plan"]["block"] for x in dec} == {256, 512, 1024}
    assert len({(x["plan"]["split_k"], x["plan"]["block"]) for x in dec}) == len(dec)  # distinct plans only
    assert all(1 <= x["split_k"] <= 16 for x in dec)
    # more than 16 rows: the variant is the rows per workgroup
    mid = [x for x in tune.candidates(0, 100, 2048, 1024, P.PRISM_BF16, max_split=4) if x["path"] == P.PRISM_PATH_DECODE]
    assert {x["plan"]["tile_m"] for x in mid} == {32, 64} and all(x["plan"]["block"] == 512 for x in mid)
    gmid = [x for x in tune.candidates(1, 100, 2048, 1024, P.PRISM_BF16, max_split=4) if x["path"] == P.PRISM_PATH_DECODE]
    assert {x["plan"]["tile_m"] for x in gmid} == {32, 64}
    # gated, at most 16 rows: the packed tile too, also with the library's own (balanced) slices
    P.prism_set_stream_balance(0x0808, 0)
    try:
        gd = [x for x in tune.candidates(1, 8, 4096, 14336, P.PRISM_BF16, max_split=4) if x["path"] == P.PRISM_PATH_DECODE]
    finally:
        P.prism_set_stream_balance()
    assert {x["plan"]["tile_n"] for x in gd} == {64, 128}
    assert any(x["variant"] == 108 and x["split_k"] == 0 and x["plan"]["grid_x"] == 252 for x in gd)
    assert all(x["plan"]["tile_n"] == 128 for x in dec)
    # the softmax operator: the plain kernel, 16 rows per workgroup, 32 rows with 1..16 K-slices
    sm = tune.candidates(P.PRISM_OP_SOFTMAX_MATMUL, 64, 16384, 128, P.PRISM_F16)
    assert {x["path"] for x in sm} == {P.PRISM_PATH_SIMPLE, P.PRISM_PATH_ROWS}
    assert sorted((x["plan"]["tile_m"], x["plan"]["split_k"]) for x in sm if x["path"] == P.PRISM_PATH_ROWS) == \
        [(16, 1)] + [(32, s) for s in range(1, 17)]
    # many rows: no decode candidates; fp32: the plain kernel only
    assert all(x["path"] != P.PRISM_PATH_DECODE for x in tune.candidates(1, 2048, 1024, 1024, P.PRISM_BF16))
    assert [x["path"] for x in tune.candidates(0, 8, 256, 512, P.PRISM_F32)] == [P.PRISM_PATH_SIMPLE]
    assert P.prism_plan(0, 16, 2048, 1024, P.PRISM_BF16)["path"] == P.PRISM_PATH_DECODE  # override is reset


def test_inputs_are_deterministic_and_bf16_exact():
    import numpy as np
    import prism_inputs as pi
    a = pi.draw(pi.BF16, 4, 64, 32, True, 5)
    b = pi.draw(pi.BF16, 4, 64, 32, True, 5)
    assert all(np.array_equal(a[k], b[k]) for k in a) and set(a) == {"X", "g", "W1", "W2"}
    assert not np.array_equal(a["W1"], a["W2"])
    # round-to-nearest-even on exact ties
    ties = np.array([1.00390625, 1.01171875, -1.00390625], dtype=np.float32)  # 1 + 2^-8, 1 + 3*2^-8
    assert list(pi.f32_to_bf16_bits(ties)) == [0x3F80, 0x3F82, 0xBF80]
    x = pi.bf16_bits_to_f32(a["X"])
    assert np.array_equal(pi.f32_to_bf16_bits(x), a["X"])
    g = pi.to_f64(a["g"], pi.BF16)
    assert g.min() >= 0.5 and g.max() <= 1.5
    h = pi.draw(pi.F16, 4, 64, 32, False, 5)
    assert h["X"].dtype == np.float16 and np.array_equal(pi.to_f64(h["X"], pi.F16), h["X"].astype(np.float64))
    # the fp16 draw is the fp32 draw of the same seed, rounded once
    f = pi.draw(pi.F32, 4, 64, 32, False, 5)
    assert np.array_equal(h["W"], f["W"].astype(np.float16))
    assert len(pi.WORKLOADS) == 5 and pi.WORKLOADS[1].N == 4096 and pi.WORKLOADS[3].gated
