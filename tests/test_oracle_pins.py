"""Pins for the CPU oracle: what the definition and the mathematics fix.

Each pin is a function of an "oracle-like" namespace so that the same pins can
be turned on deliberately broken copies of the oracle (test_pins_catch_planted
_mistakes): a plausible mistake anywhere in it must fail at least one pin.
"""
import math
import os
import types

import numpy as np
import pytest

import oracle.rmsnorm_family as O

GOLD = os.path.join(os.path.dirname(__file__), "golden", "hand_worked_2x2.txt")


def _rng(seed):
    return np.random.Generator(np.random.Philox(seed))


def _rand(seed, M, K, N):
    r = _rng(seed)
    X = r.standard_normal((M, K))
    g = r.random(K) + 0.5
    W1 = r.standard_normal((K, N)) / math.sqrt(K)
    W2 = r.standard_normal((K, N)) / math.sqrt(K)
    return X, g, W1, W2


def _golden():
    vals = {}
    with open(GOLD) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            k, v = line.split()
            vals[k] = float(v)
    return vals


# ---- pins --------------------------------------------------------------------------------

def pin_hand_worked(o):
    """tests/golden/hand_worked_2x2.txt: closed-form values of a 1x2 example."""
    gv = _golden()
    s2 = gv["sqrt2"]
    X = np.array([[3.0, 4.0]])
    W = np.array([[1.0, 2.0], [3.0, 4.0]])
    W2 = np.array([[1.0, 0.0], [0.0, 2.0]])
    one = np.array([1.0, 1.0])
    g = np.array([2.0, 0.5])
    np.testing.assert_allclose(o.rms_norm(X, one, 0.0), [[0.6 * s2, 0.8 * s2]], rtol=1e-15)
    np.testing.assert_allclose(o.rmsnorm_matmul(X, one, W, 0.0), [[3 * s2, 4.4 * s2]], rtol=1e-15)
    np.testing.assert_allclose(o.rmsnorm_matmul(X, g, W, 0.0), [[2.4 * s2, 4 * s2]], rtol=1e-15)
    np.testing.assert_allclose(o.rmsnorm_matmul(X, g, W, 3.5), [[3.0, 5.0]], rtol=1e-15)
    np.testing.assert_allclose(o.rmsnorm_gated_mlp(X, g, W, W2, 3.5),
                               [[gv["silu3"] * 1.5, gv["silu5"] * 1.0]], rtol=1e-15)


def pin_scale_invariance(o):
    """RMSNorm(cX) = RMSNorm(X) for c > 0 at eps = 0; closed-form ratio at eps > 0."""
    X, g, W, _ = _rand(1, 5, 48, 7)
    base = o.rmsnorm_matmul(X, g, W, 0.0)
    for c in (0.5, 3.0, 1e3):
        np.testing.assert_allclose(o.rmsnorm_matmul(c * X, g, W, 0.0), base, rtol=1e-12, atol=1e-14)
    eps = 1e-2
    ms = np.mean(X * X, axis=1, keepdims=True)
    for c in (0.5, 3.0):
        ratio = np.sqrt((ms + eps) / (ms + eps / c**2))
        np.testing.assert_allclose(o.rms_norm(c * X, g, eps), o.rms_norm(X, g, eps) * ratio, rtol=1e-12)


def pin_unit_rms(o):
    """g = 1: every normalised row has RMS 1 at eps = 0, sqrt(ms/(ms+eps)) otherwise."""
    X, _, _, _ = _rand(2, 6, 64, 1)
    one = np.ones(64)
    Nrm = o.rms_norm(X, one, 0.0)
    np.testing.assert_allclose(np.sqrt(np.mean(Nrm * Nrm, axis=1)), 1.0, rtol=1e-14)
    eps = 0.25
    ms = np.mean(X * X, axis=1)
    Nrm = o.rms_norm(X, one, eps)
    np.testing.assert_allclose(np.sqrt(np.mean(Nrm * Nrm, axis=1)), np.sqrt(ms / (ms + eps)), rtol=1e-13)


def pin_identity_weight(o):
    """W = I returns the normalised X."""
    X, g, _, _ = _rand(3, 4, 32, 1)
    np.testing.assert_allclose(o.rmsnorm_matmul(X, g, np.eye(32), 1e-6), o.rms_norm(X, g, 1e-6),
                               rtol=0, atol=0)
    # and the normalised X itself, element by element, from scalar arithmetic
    Nrm = o.rms_norm(X, g, 1e-6)
    for m in range(4):
        ms = sum(float(x) * float(x) for x in X[m]) / 32
        for k in range(32):
            assert Nrm[m, k] == pytest.approx(X[m, k] / math.sqrt(ms + 1e-6) * g[k], rel=1e-14)


def _brute_plain(X, g, W, eps):
    M, K, N = len(X), len(g), len(W[0])
    Y = [[0.0] * N for _ in range(M)]
    for m in range(M):
        for j in range(N):
            acc = 0.0
            for k in range(K):
                ms = 0.0
                for kk in range(K):
                    ms += X[m][kk] * X[m][kk]
                acc += X[m][k] / math.sqrt(ms / K + eps) * g[k] * W[k][j]
            Y[m][j] = acc
    return np.array(Y)


def pin_brute_force(o):
    """Deliberately naive scalar loops agree on tiny, non-square shapes."""
    for seed, (M, K, N) in enumerate([(1, 1, 1), (3, 5, 2), (4, 16, 8), (2, 7, 3)]):
        X, g, W1, W2 = _rand(10 + seed, M, K, N)
        for eps in (0.0, 1e-6, 0.3):
            ref = _brute_plain(X.tolist(), g.tolist(), W1.tolist(), eps)
            np.testing.assert_allclose(o.rmsnorm_matmul(X, g, W1, eps), ref, rtol=1e-12, atol=1e-14)
            a = _brute_plain(X.tolist(), g.tolist(), W1.tolist(), eps)
            b = _brute_plain(X.tolist(), g.tolist(), W2.tolist(), eps)
            ref_g = np.array([[a[m, j] / (1.0 + math.exp(-a[m, j])) * b[m, j] for j in range(N)]
                              for m in range(M)])
            np.testing.assert_allclose(o.rmsnorm_gated_mlp(X, g, W1, W2, eps), ref_g, rtol=1e-12, atol=1e-14)


def pin_fused_order(o):
    """Table 1, "matmul commutes with div denominator": scale after the product."""
    X, g, W, _ = _rand(4, 9, 40, 11)
    eps = 1e-6
    r = 1.0 / np.sqrt(np.mean(X * X, axis=1, keepdims=True) + eps)
    fused = ((X * g) @ W) * r
    np.testing.assert_allclose(o.rmsnorm_matmul(X, g, W, eps), fused, rtol=1e-12, atol=1e-14)


def pin_closed_form_rows(o):
    """Constant row -> sign(c) * g^T W; one-hot row a*e_j -> sign(a) sqrt(K) g_j W[j,:] (eps = 0)."""
    K, N = 24, 5
    _, g, W, _ = _rand(5, 1, K, N)
    for c in (2.5, -0.125):
        X = np.full((1, K), c)
        np.testing.assert_allclose(o.rmsnorm_matmul(X, g, W, 0.0), [math.copysign(1, c) * (g @ W)], rtol=1e-13)
    for a, j in ((3.0, 0), (-0.7, 17), (1e-3, K - 1)):
        X = np.zeros((1, K))
        X[0, j] = a
        np.testing.assert_allclose(o.rmsnorm_matmul(X, g, W, 0.0),
                                   [math.copysign(1, a) * math.sqrt(K) * g[j] * W[j]], rtol=1e-13)
    # eps > 0, zero row: output exactly zero, no NaN
    assert np.all(o.rmsnorm_matmul(np.zeros((2, K)), g, W, 1e-6) == 0.0)


def pin_partitions(o):
    """Table 1, parallelized matmul: column partition exact, split-K sums to the whole."""
    X, g, W, W2 = _rand(6, 7, 64, 24)
    eps = 1e-6
    full = o.rmsnorm_matmul(X, g, W, eps)
    np.testing.assert_allclose(o.rmsnorm_matmul(X, g, W[:, 8:16], eps), full[:, 8:16], rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(o.rmsnorm_matmul(X[2:5], g, W, eps), full[2:5], rtol=1e-13, atol=1e-15)
    Nrm = o.rms_norm(X, g, eps)
    parts = sum(Nrm[:, s:s + 16] @ W[s:s + 16] for s in range(0, 64, 16))
    np.testing.assert_allclose(parts, full, rtol=1e-12, atol=1e-14)
    fullg = o.rmsnorm_gated_mlp(X, g, W, W2, eps)
    np.testing.assert_allclose(o.rmsnorm_gated_mlp(X, g, W[:, 5:9], W2[:, 5:9], eps), fullg[:, 5:9],
                               rtol=1e-13, atol=1e-15)


def pin_gated_identities(o):
    """W1 = 0 -> 0; silu(a) - silu(-a) = a; silu(0) = 0; gated = silu(plain(W1)) * plain(W2)."""
    X, g, W1, W2 = _rand(7, 5, 32, 9)
    eps = 1e-6
    assert np.all(o.rmsnorm_gated_mlp(X, g, np.zeros_like(W1), W2, eps) == 0.0)
    a = np.linspace(-40, 40, 161)
    np.testing.assert_allclose(o.silu(a) - o.silu(-a), a, rtol=1e-13, atol=1e-15)
    assert o.silu(np.array([0.0]))[0] == 0.0
    assert o.silu(np.array([-800.0]))[0] == 0.0 and o.silu(np.array([800.0]))[0] == 800.0
    assert o.silu(np.array([1.0]))[0] == pytest.approx(1.0 / (1.0 + math.exp(-1.0)), rel=1e-15)
    ya = o.rmsnorm_matmul(X, g, W1, eps)
    yb = o.rmsnorm_matmul(X, g, W2, eps)
    np.testing.assert_allclose(o.rmsnorm_gated_mlp(X, g, W1, W2, eps), o.silu(ya) * yb, rtol=1e-13, atol=1e-300)
    # the activation sits on W1 only: swapping the weights changes the result
    assert not np.allclose(o.rmsnorm_gated_mlp(X, g, W1, W2, eps), o.rmsnorm_gated_mlp(X, g, W2, W1, eps))
    # scale goes on before the activation: silu is not homogeneous
    Xs = 4.0 * X
    np.testing.assert_allclose(o.rmsnorm_gated_mlp(Xs, g, W1, W2, 0.0), o.rmsnorm_gated_mlp(X, g, W1, W2, 0.0),
                               rtol=1e-12, atol=1e-14)


def pin_torch_second_opinion(o):
    """torch float64 CPU routines as an independent library (textbook special case)."""
    torch = pytest.importorskip("torch")
    X, g, W1, W2 = _rand(8, 6, 128, 20)
    eps = 1e-6
    tX, tg, tW1, tW2 = (torch.from_numpy(a) for a in (X, g, W1, W2))
    nrm = tX * torch.rsqrt(tX.pow(2).mean(dim=1, keepdim=True) + eps) * tg
    np.testing.assert_allclose(o.rmsnorm_matmul(X, g, W1, eps), (nrm @ tW1).numpy(), rtol=1e-12, atol=1e-14)
    ref = torch.nn.functional.silu(nrm @ tW1) * (nrm @ tW2)
    np.testing.assert_allclose(o.rmsnorm_gated_mlp(X, g, W1, W2, eps), ref.numpy(), rtol=1e-12, atol=1e-14)


def pin_output_variance(o):
    """i.i.d. inputs of the benchmark recipe: Var(Y) = E[g^2] ms/(ms+eps) = 13/12 (weak, statistical)."""
    r = _rng(9)
    M, K, N = 32, 512, 256
    X = r.standard_normal((M, K))
    g = r.random(K) + 0.5
    W = r.standard_normal((K, N)) / math.sqrt(K)
    Y = o.rmsnorm_matmul(X, g, W, 1e-6)
    assert abs(Y.var() - 13.0 / 12.0) < 0.05
    assert abs(Y.mean()) < 0.05


def pin_paper_variants(o):
    """The paper's two gated workloads as written (Section 7.1): closed forms, brute force, symmetry."""
    gv = _golden()
    # hand-worked (tests/golden): X = [[3, 4]], W = [[1, 2], [3, 4]], W2 = diag(1, 2)
    X = np.array([[3.0, 4.0]])
    W = np.array([[1.0, 2.0], [3.0, 4.0]])
    W2 = np.array([[1.0, 0.0], [0.0, 2.0]])
    g = np.array([2.0, 0.5])
    # case E: GLU with norm, g = [2, .5], eps = 3.5: Nrm = [1.5, .5]; Nrm W = [3, 5]; Nrm W2 = [1.5, 1]
    np.testing.assert_allclose(o.rmsnorm_glu(X, g, W, W2, 3.5), [[4.5, 5.0]], rtol=1e-15)
    # case F: SwiGLU without norm: X W = [15, 22], X W2 = [3, 8]
    np.testing.assert_allclose(o.swiglu(X, W, W2), [[gv["silu15"] * 3.0, gv["silu22"] * 8.0]], rtol=1e-15)
    # brute force, scalar loops
    for seed, (M, K, N) in enumerate([(1, 1, 1), (3, 5, 2), (2, 7, 3)]):
        Xr, gr, W1r, W2r = _rand(40 + seed, M, K, N)
        a = _brute_plain(Xr.tolist(), gr.tolist(), W1r.tolist(), 0.3)
        b = _brute_plain(Xr.tolist(), gr.tolist(), W2r.tolist(), 0.3)
        np.testing.assert_allclose(o.rmsnorm_glu(Xr, gr, W1r, W2r, 0.3), a * b, rtol=1e-12, atol=1e-14)
        ref = np.zeros((M, N))
        for m in range(M):
            for j in range(N):
                sa = sum(Xr[m, k] * W1r[k, j] for k in range(K))
                sb = sum(Xr[m, k] * W2r[k, j] for k in range(K))
                ref[m, j] = sa / (1.0 + math.exp(-sa)) * sb
        np.testing.assert_allclose(o.swiglu(Xr, W1r, W2r), ref, rtol=1e-12, atol=1e-14)
    Xr, gr, W1r, W2r = _rand(44, 4, 24, 6)
    # GLU: the branches are interchangeable, the result is homogeneous of degree 0 in X at eps = 0 ...
    np.testing.assert_allclose(o.rmsnorm_glu(Xr, gr, W1r, W2r, 1e-6), o.rmsnorm_glu(Xr, gr, W2r, W1r, 1e-6), rtol=1e-14)
    np.testing.assert_allclose(o.rmsnorm_glu(5.0 * Xr, gr, W1r, W2r, 0.0), o.rmsnorm_glu(Xr, gr, W1r, W2r, 0.0), rtol=1e-12)
    # ... and equals the product of two plain calls
    np.testing.assert_allclose(o.rmsnorm_glu(Xr, gr, W1r, W2r, 1e-6),
                               o.rmsnorm_matmul(Xr, gr, W1r, 1e-6) * o.rmsnorm_matmul(Xr, gr, W2r, 1e-6), rtol=1e-13)
    # one-hot row a e_j, eps = 0: Nrm = sign(a) sqrt(K) g_j e_j, so Y = K g_j^2 W1[j,:] W2[j,:]
    Xo = np.zeros((1, 24))
    Xo[0, 5] = -0.3
    np.testing.assert_allclose(o.rmsnorm_glu(Xo, gr, W1r, W2r, 0.0), [24 * gr[5] ** 2 * W1r[5] * W2r[5]], rtol=1e-13)
    # SwiGLU: not normalised (scaling X changes it), the branches are not interchangeable, W_gate = 0 -> 0,
    # one-hot row picks row j of both weights
    assert not np.allclose(o.swiglu(2.0 * Xr, W1r, W2r), o.swiglu(Xr, W1r, W2r))
    assert not np.allclose(o.swiglu(Xr, W1r, W2r), o.swiglu(Xr, W2r, W1r))
    assert np.all(o.swiglu(Xr, np.zeros_like(W1r), W2r) == 0.0)
    np.testing.assert_allclose(o.swiglu(Xo, W1r, W2r), [o.silu(-0.3 * W1r[5]) * (-0.3 * W2r[5])], rtol=1e-13)
    # relation to the target operator: dividing X by its row rms by hand, with g = 1, gives the gated MLP
    r = 1.0 / np.sqrt(np.mean(Xr * Xr, axis=1, keepdims=True) + 1e-6)
    np.testing.assert_allclose(o.swiglu(Xr * r, W1r, W2r), o.rmsnorm_gated_mlp(Xr, np.ones(24), W1r, W2r, 1e-6),
                               rtol=1e-12, atol=1e-15)
    torch = pytest.importorskip("torch")
    tX, tW1, tW2 = (torch.from_numpy(a) for a in (Xr, W1r, W2r))
    np.testing.assert_allclose(o.swiglu(Xr, W1r, W2r), (torch.nn.functional.silu(tX @ tW1) * (tX @ tW2)).numpy(),
                               rtol=1e-12, atol=1e-15)


def pin_softmax_matmul(o):
    """The running example (Figure 1): hand-worked values, closed forms, invariances, brute force."""
    gv = _golden()
    # case G (tests/golden): X = [[0, ln 3]] -> softmax = [1/4, 3/4]; W = [[1, 2], [3, 4]] -> Y = [2.5, 3.5]
    X = np.array([[0.0, gv["ln3"]]])
    W = np.array([[1.0, 2.0], [3.0, 4.0]])
    np.testing.assert_allclose(o.softmax_matmul(X, W), [[2.5, 3.5]], rtol=1e-15)
    Xr, _, W1r, _ = _rand(50, 5, 24, 7)
    Y = o.softmax_matmul(Xr, W1r)
    # W = ones: every row of softmax sums to one; W = I: the softmax itself, positive, ordered like X
    np.testing.assert_allclose(o.softmax_matmul(Xr, np.ones((24, 3))), np.ones((5, 3)), rtol=1e-14)
    Pm = o.softmax_matmul(Xr, np.eye(24))
    assert np.all(Pm > 0) and np.array_equal(np.argsort(Pm, axis=1), np.argsort(Xr, axis=1))
    np.testing.assert_allclose(Pm[:, 3] / Pm[:, 9], np.exp(Xr[:, 3] - Xr[:, 9]), rtol=1e-13)
    # shift invariance per row, and no scale invariance (unlike rms_norm)
    shift = np.array([[3.0], [-7.5], [0.25], [100.0], [-200.0]])
    np.testing.assert_allclose(o.softmax_matmul(Xr + shift, W1r), Y, rtol=1e-11, atol=1e-14)
    assert not np.allclose(o.softmax_matmul(2.0 * Xr, W1r), Y)
    # constant row: the plain mean of the rows of W; one entry far above the rest: that row of W
    np.testing.assert_allclose(o.softmax_matmul(np.full((1, 24), -1.75), W1r), [W1r.mean(axis=0)], rtol=1e-13)
    Xd = np.zeros((1, 24))
    Xd[0, 11] = 60.0
    np.testing.assert_allclose(o.softmax_matmul(Xd, W1r), [W1r[11]], rtol=1e-12, atol=1e-15)
    # column partition exact, split-K of numerator and denominator (the fused program's two accumulators)
    np.testing.assert_allclose(o.softmax_matmul(Xr, W1r[:, 2:5]), Y[:, 2:5], rtol=1e-14)
    E = np.exp(Xr)
    num = sum(E[:, s:s + 8] @ W1r[s:s + 8] for s in range(0, 24, 8))
    den = sum(E[:, s:s + 8].sum(axis=1, keepdims=True) for s in range(0, 24, 8))
    np.testing.assert_allclose(num / den, Y, rtol=1e-13)
    # brute force, scalar loops
    for seed, (M, K, N) in enumerate([(1, 1, 1), (3, 5, 2), (2, 9, 4)]):
        Xb, _, Wb, _ = _rand(60 + seed, M, K, N)
        ref = np.zeros((M, N))
        for m in range(M):
            den = 0.0
            for k in range(K):
                den += math.exp(Xb[m, k])
            for j in range(N):
                acc = 0.0
                for k in range(K):
                    acc += math.exp(Xb[m, k]) / den * Wb[k, j]
                ref[m, j] = acc
        np.testing.assert_allclose(o.softmax_matmul(Xb, Wb), ref, rtol=1e-12, atol=1e-15)
    torch = pytest.importorskip("torch")
    np.testing.assert_allclose(Y, (torch.softmax(torch.from_numpy(Xr), dim=1) @ torch.from_numpy(W1r)).numpy(),
                               rtol=1e-12, atol=1e-15)


def pin_gqa_decode_attention(o):
    """Section 7.1, Attention and QK-Attention: hand-worked case, closed forms, brute force, invariances."""
    gv = _golden()
    ln3 = gv["ln3"]
    # case H (tests/golden): one batch, one head, D = 2, two keys.  Q = [ln 3, 0], K = [[0, 5], [1, 7]]
    #   scores = [0, ln 3] -> softmax = [1/4, 3/4];  V = [[1, 2], [3, 4]] -> O = [2.5, 3.5]
    Q = np.array([[[ln3, 0.0]]])
    K = np.array([[[0.0, 5.0], [1.0, 7.0]]])
    V = np.array([[[1.0, 2.0], [3.0, 4.0]]])
    np.testing.assert_allclose(o.gqa_decode_attention(Q, K, V), [[[2.5, 3.5]]], rtol=1e-15)
    # case I: qk_norm at eps = 0 turns Q = [3, 4] into [0.6, 0.8] sqrt 2; with K = [[0, 0], [ln3/(0.6 sqrt2), 0]] the
    #   scores are again [0, ln 3]
    Q2 = np.array([[[3.0, 4.0]]])
    K2 = np.array([[[0.0, 0.0], [ln3 / (0.6 * gv["sqrt2"]), 0.0]]])
    np.testing.assert_allclose(o.gqa_decode_attention(Q2, K2, V, qk_norm=True, eps=0.0), [[[2.5, 3.5]]], rtol=1e-14)
    r = _rng(70)
    B, G, H, D = 2, 3, 9, 4
    Qr, Kr, Vr = r.standard_normal((B, G, D)), r.standard_normal((B, H, D)), r.standard_normal((B, H, D))
    for scale, qkn, eps in ((1.0, False, 0.0), (0.5, False, 0.0), (1.0, True, 1e-6), (0.37, True, 0.2)):
        ref = np.zeros((B, G, D))
        for b in range(B):
            for g in range(G):
                q = Qr[b, g].tolist()
                if qkn:
                    ms = sum(x * x for x in q) / D
                    q = [x / math.sqrt(ms + eps) for x in q]
                sc = [scale * sum(q[d] * Kr[b, hh, d] for d in range(D)) for hh in range(H)]
                den = sum(math.exp(v) for v in sc)
                for d in range(D):
                    ref[b, g, d] = sum(math.exp(sc[hh]) / den * Vr[b, hh, d] for hh in range(H))
        np.testing.assert_allclose(o.gqa_decode_attention(Qr, Kr, Vr, scale, qkn, eps), ref, rtol=1e-12, atol=1e-15)
    base = o.gqa_decode_attention(Qr, Kr, Vr)
    # heads are independent and share K, V of their batch; batches are independent
    np.testing.assert_allclose(o.gqa_decode_attention(Qr[:, 1:2], Kr, Vr), base[:, 1:2], rtol=1e-14)
    np.testing.assert_allclose(o.gqa_decode_attention(Qr[1:], Kr[1:], Vr[1:]), base[1:], rtol=1e-14)
    assert not np.allclose(o.gqa_decode_attention(Qr, Kr[::-1], Vr[::-1]), base)
    # the order of the keys does not matter as long as values move with them; a constant added to all scores cancels
    perm = r.permutation(H)
    np.testing.assert_allclose(o.gqa_decode_attention(Qr, Kr[:, perm], Vr[:, perm]), base, rtol=1e-13)
    # Q = 0: uniform weights, the mean of V; one key: that value; all values equal: that value
    np.testing.assert_allclose(o.gqa_decode_attention(np.zeros((B, G, D)), Kr, Vr),
                               np.repeat(Vr.mean(axis=1, keepdims=True), G, axis=1), rtol=1e-13)
    np.testing.assert_allclose(o.gqa_decode_attention(Qr, Kr[:, :1], Vr[:, :1]), np.repeat(Vr[:, :1], G, axis=1), rtol=1e-14)
    np.testing.assert_allclose(o.gqa_decode_attention(Qr, Kr, np.ones((B, H, D)) * 2.5), np.full((B, G, D), 2.5), rtol=1e-14)
    # scale multiplies the scores: scale s on Q equals Q * s; qk_norm makes the result independent of |Q| at eps = 0
    np.testing.assert_allclose(o.gqa_decode_attention(Qr, Kr, Vr, scale=0.25), o.gqa_decode_attention(0.25 * Qr, Kr, Vr), rtol=1e-13)
    np.testing.assert_allclose(o.gqa_decode_attention(7.0 * Qr, Kr, Vr, qk_norm=True), o.gqa_decode_attention(Qr, Kr, Vr, qk_norm=True), rtol=1e-12)
    assert not np.allclose(o.gqa_decode_attention(Qr, Kr, Vr, qk_norm=True), base)
    # reduction to the two operators it is made of
    one = np.ones(D)
    for b in range(B):
        np.testing.assert_allclose(o.gqa_decode_attention(Qr, Kr, Vr, 1.0, True, 1e-6)[b],
                                   o.softmax_matmul(o.rmsnorm_matmul(Qr[b], one, Kr[b].T.copy(), 1e-6), Vr[b]), rtol=1e-13)
    torch = pytest.importorskip("torch")
    tq, tk, tv = (torch.from_numpy(a) for a in (Qr, Kr, Vr))
    ref = torch.softmax(0.5 * tq @ tk.transpose(1, 2), dim=-1) @ tv
    np.testing.assert_allclose(o.gqa_decode_attention(Qr, Kr, Vr, scale=0.5), ref.numpy(), rtol=1e-12, atol=1e-15)


PINS = [pin_gqa_decode_attention, pin_softmax_matmul, pin_paper_variants, pin_hand_worked, pin_scale_invariance, pin_unit_rms, pin_identity_weight, pin_brute_force,
        pin_fused_order, pin_closed_form_rows, pin_partitions, pin_gated_identities,
        pin_torch_second_opinion, pin_output_variance]


@pytest.mark.parametrize("pin", PINS, ids=lambda p: p.__name__)
def test_pin(pin):
    pin(O)


# ---- planted mistakes: each broken oracle must be caught by some pin -----------------------

def _mutant(**over):
    ns = types.SimpleNamespace(rms_norm=O.rms_norm, rmsnorm_matmul=O.rmsnorm_matmul,
                               rmsnorm_gated_mlp=O.rmsnorm_gated_mlp, silu=O.silu,
                               rmsnorm_glu=O.rmsnorm_glu, swiglu=O.swiglu, softmax_matmul=O.softmax_matmul,
                               gqa_decode_attention=O.gqa_decode_attention)
    for k, v in over.items():
        setattr(ns, k, v)
    # rebuild the composite functions on top of the (possibly replaced) pieces
    if "rmsnorm_matmul" not in over:
        ns.rmsnorm_matmul = lambda X, g, W, eps: np.matmul(ns.rms_norm(X, g, eps), W)
    if "rmsnorm_gated_mlp" not in over:
        def gated(X, g, W1, W2, eps):
            n = ns.rms_norm(X, g, eps)
            return ns.silu(n @ W1) * (n @ W2)
        ns.rmsnorm_gated_mlp = gated
    if "rmsnorm_glu" not in over:
        def glu(X, g, W1, W2, eps):
            n = ns.rms_norm(X, g, eps)
            return (n @ W1) * (n @ W2)
        ns.rmsnorm_glu = glu
    if "swiglu" not in over:
        ns.swiglu = lambda X, Wg, Wu: ns.silu(X @ Wg) * (X @ Wu)
    return ns


def _norm_variant(fn):
    def rms_norm(X, g, eps):
        X = np.asarray(X, dtype=np.float64)
        return np.stack([fn(X[m], np.asarray(g), eps) for m in range(X.shape[0])]) if X.shape[0] else X.copy()
    return rms_norm


MUTANTS = {
    "sum_not_mean": _mutant(rms_norm=_norm_variant(lambda x, g, e: x / np.sqrt(np.sum(x * x) + e) * g)),
    "eps_outside_root": _mutant(rms_norm=_norm_variant(lambda x, g, e: x / (np.sqrt(np.mean(x * x)) + e) * g)),
    "eps_dropped": _mutant(rms_norm=_norm_variant(lambda x, g, e: x / np.sqrt(np.mean(x * x)) * g)),
    "bessel_K_minus_1": _mutant(rms_norm=_norm_variant(
        lambda x, g, e: x / np.sqrt(np.sum(x * x) / max(len(x) - 1, 1) + e) * g)),
    "gain_dropped": _mutant(rms_norm=_norm_variant(lambda x, g, e: x / np.sqrt(np.mean(x * x) + e))),
    "gain_inside_sum": _mutant(rms_norm=_norm_variant(
        lambda x, g, e: x * g / np.sqrt(np.mean((x * g) ** 2) + e))),
    "mean_subtracted": _mutant(rms_norm=_norm_variant(
        lambda x, g, e: (x - x.mean()) / np.sqrt(np.mean((x - x.mean()) ** 2) + e) * g)),
    "abs_mean_not_rms": _mutant(rms_norm=_norm_variant(lambda x, g, e: x / (np.mean(np.abs(x)) + e) * g)),
    "W_transposed": _mutant(rmsnorm_matmul=lambda X, g, W, eps: np.matmul(
        O.rms_norm(X, g, eps), W.T if W.shape[0] == W.shape[1] else W)),
    "silu_on_W2": _mutant(rmsnorm_gated_mlp=lambda X, g, W1, W2, eps: O.rmsnorm_gated_mlp(X, g, W2, W1, eps)),
    "no_activation": _mutant(rmsnorm_gated_mlp=lambda X, g, W1, W2, eps: (
        O.rmsnorm_matmul(X, g, W1, eps) * O.rmsnorm_matmul(X, g, W2, eps))),
    "sigmoid_not_silu": _mutant(silu=lambda a: 1.0 / (1.0 + np.exp(-np.asarray(a, dtype=np.float64)))),
    "silu_wrong_sign": _mutant(silu=lambda a: np.asarray(a) / (1.0 + np.exp(np.asarray(a, dtype=np.float64)))),
    "glu_with_activation": _mutant(rmsnorm_glu=lambda X, g, W1, W2, eps: O.rmsnorm_gated_mlp(X, g, W1, W2, eps)),
    "glu_sum_not_product": _mutant(rmsnorm_glu=lambda X, g, W1, W2, eps: (
        O.rmsnorm_matmul(X, g, W1, eps) + O.rmsnorm_matmul(X, g, W2, eps))),
    "swiglu_normalised": _mutant(swiglu=lambda X, Wg, Wu: O.rmsnorm_gated_mlp(X, np.ones(X.shape[1]), Wg, Wu, 0.0)),
    "swiglu_silu_on_up": _mutant(swiglu=lambda X, Wg, Wu: O.swiglu(X, Wu, Wg)),
    "swiglu_no_activation": _mutant(swiglu=lambda X, Wg, Wu: (X @ Wg) * (X @ Wu)),
    "softmax_no_denominator": _mutant(softmax_matmul=lambda X, W: np.exp(X) @ W),
    "softmax_over_rows_of_X": _mutant(softmax_matmul=lambda X, W: (np.exp(X) / np.exp(X).sum(axis=0, keepdims=True)) @ W),
    "softmax_base_2": _mutant(softmax_matmul=lambda X, W: (np.exp2(X) / np.exp2(X).sum(axis=1, keepdims=True)) @ W),
    "softmax_divides_by_K": _mutant(softmax_matmul=lambda X, W: (np.exp(X) / X.shape[1]) @ W),
    "softmax_of_abs": _mutant(softmax_matmul=lambda X, W: (np.exp(np.abs(X)) / np.exp(np.abs(X)).sum(axis=1, keepdims=True)) @ W),
    "softmax_W_transposed": _mutant(softmax_matmul=lambda X, W: O.softmax_matmul(X, W.T if W.shape[0] == W.shape[1] else W)),
    "attn_scores_not_scaled": _mutant(gqa_decode_attention=lambda Q, K, V, scale=1.0, qk_norm=False, eps=0.0: (
        O.gqa_decode_attention(Q, K, V, 1.0, qk_norm, eps))),
    "attn_norm_on_keys_too": _mutant(gqa_decode_attention=lambda Q, K, V, scale=1.0, qk_norm=False, eps=0.0: (
        O.gqa_decode_attention(Q, np.stack([O.rms_norm(k, np.ones(k.shape[1]), eps) for k in K]) if qk_norm else K, V,
                               scale, qk_norm, eps))),
    "attn_norm_ignored": _mutant(gqa_decode_attention=lambda Q, K, V, scale=1.0, qk_norm=False, eps=0.0: (
        O.gqa_decode_attention(Q, K, V, scale, False, eps))),
    "attn_softmax_over_heads": _mutant(gqa_decode_attention=lambda Q, K, V, scale=1.0, qk_norm=False, eps=0.0: np.stack([
        (lambda S: (np.exp(S) / np.exp(S).sum(axis=0, keepdims=True)) @ V[b])(
            scale * (O.rms_norm(Q[b], np.ones(Q.shape[2]), eps) if qk_norm else Q[b]) @ K[b].T) for b in range(Q.shape[0])])),
    "attn_values_of_other_batch": _mutant(gqa_decode_attention=lambda Q, K, V, scale=1.0, qk_norm=False, eps=0.0: (
        O.gqa_decode_attention(Q, K, V[::-1] if V.shape[0] > 1 else V, scale, qk_norm, eps))),
    "attn_inverse_sqrt_d_added": _mutant(gqa_decode_attention=lambda Q, K, V, scale=1.0, qk_norm=False, eps=0.0: (
        O.gqa_decode_attention(Q, K, V, scale / math.sqrt(Q.shape[2]), qk_norm, eps))),
    "scale_after_silu": _mutant(rmsnorm_gated_mlp=lambda X, g, W1, W2, eps: (
        O.silu((X * g) @ W1) * ((X * g) @ W2) / (np.mean(X * X, axis=1, keepdims=True) + eps))),
}


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_pins_catch_planted_mistakes(name):
    mutant = MUTANTS[name]
    caught = []
    for pin in PINS:
        try:
            with np.errstate(all="ignore"):
                pin(mutant)
        except (AssertionError, FloatingPointError, ZeroDivisionError):
            caught.append(pin.__name__)
    assert caught, f"no pin notices the planted mistake {name!r}"
