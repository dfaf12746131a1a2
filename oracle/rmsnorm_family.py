"""Plain fp64 definition of RMSNorm followed by a matrix product.

TEST INFRASTRUCTURE ONLY: nothing on the product path may import this file.

What it follows
---------------
* Paper, Section 7.1, workload "RMSNorm": O = matmul(rms_norm(X), W).
* Paper, Section 7.1, workload "RMSNorm-MLP": two products that share
  rms_norm(X), multiplied element by element.
* Paper, Section 7.1, workload "SwiGLU": silu(X W_gate) * (X W_up), which fixes
  that the activation sits on the gate branch.
The paper treats rms_norm as an opaque operator and never writes it out, has no
gain tensor and no epsilon.  The readings used here (all listed again in the
design notes): rms(x) = sqrt(mean_k x_k^2 + eps) with eps inside the root and
the mean dividing by K; a gain g[K] multiplies the normalised row element by
element; W1 is the gate (SiLU) branch and W2 the linear one; the 1/rms scale is
applied before the SiLU.

The fused programs the paper derives reach exactly this result (the rewrite is
the axiom "matmul commutes with div denominator", Table 1), so the oracle is
the definition written out in the unfused order: normalise first, then
multiply.  Every array is float64; callers widen stored bf16/fp32 inputs
exactly before calling.  ``numpy.matmul`` is the one library step.

The paper's own two gated workloads are here as written there, beside the
target operator that combines them: ``rmsnorm_glu`` ("RMSNorm-MLP": shared
normalisation, no activation) and ``swiglu`` ("SwiGLU": activation, no
normalisation, no gain).

Pins (tests/test_oracle_pins.py): scale invariance and unit row RMS at eps=0
and their closed forms at eps>0, W = I, a triple-loop brute force, the
fused-order identity, constant-row and one-hot-row closed forms, column and
split-K partition identities, gated identities, and a second opinion from
torch's float64 CPU routines.
"""
import numpy as np


def _f64(a, ndim, name):
    a = np.asarray(a)
    if a.dtype != np.float64:
        raise TypeError(f"{name}: oracle inputs must be float64 (widen stored values exactly first)")
    if a.ndim != ndim:
        raise ValueError(f"{name}: expected {ndim} dims, got {a.ndim}")
    return a


def rms_norm(X, g, eps):
    """N[m,k] = X[m,k] / sqrt(mean_k X[m,:]^2 + eps) * g[k].

    X is [M,K], g is [K]; returns [M,K].  Paper Section 7.1 (operator
    rms_norm); eps, g and the eps-inside-the-root convention are readings.
    """
    X = _f64(X, 2, "X")
    g = _f64(g, 1, "g")
    M, K = X.shape
    if g.shape[0] != K:
        raise ValueError("g must have K entries")
    eps = float(eps)
    N = np.empty_like(X)
    for m in range(M):
        ms = np.sum(X[m] * X[m]) / K
        r = 1.0 / np.sqrt(ms + eps)
        N[m] = X[m] * r * g
    return N


def rmsnorm_matmul(X, g, W, eps):
    """Y[M,N] = rms_norm(X; g, eps) @ W, W is [K,N].  Paper Section 7.1, "RMSNorm"."""
    W = _f64(W, 2, "W")
    Nrm = rms_norm(X, g, eps)
    if W.shape[0] != Nrm.shape[1]:
        raise ValueError("W must be [K,N]")
    return np.matmul(Nrm, W)


def silu(a):
    """silu(a) = a / (1 + exp(-a)), evaluated without overflow for either sign."""
    a = np.asarray(a, dtype=np.float64)
    out = np.empty_like(a)
    pos = a >= 0
    out[pos] = a[pos] / (1.0 + np.exp(-a[pos]))
    e = np.exp(a[~pos])
    out[~pos] = a[~pos] * e / (1.0 + e)
    return out


def rmsnorm_gated_mlp(X, g, W1, W2, eps):
    """Y = silu(Nrm @ W1) * (Nrm @ W2), Nrm = rms_norm(X; g, eps); W1 is the gate.

    Paper Section 7.1: "RMSNorm-MLP" gives the two products sharing the
    normalised input, "SwiGLU" puts the activation on the gate branch.
    """
    W1 = _f64(W1, 2, "W1")
    W2 = _f64(W2, 2, "W2")
    if W1.shape != W2.shape:
        raise ValueError("W1 and W2 must have the same shape")
    Nrm = rms_norm(X, g, eps)
    if W1.shape[0] != Nrm.shape[1]:
        raise ValueError("W1/W2 must be [K,N]")
    a = np.matmul(Nrm, W1)
    b = np.matmul(Nrm, W2)
    return silu(a) * b


def rmsnorm_glu(X, g, W1, W2, eps):
    """Y = (Nrm @ W1) * (Nrm @ W2), Nrm = rms_norm(X; g, eps): no activation.

    Paper Section 7.1, "RMSNorm-MLP": (rms_norm(X) W_up) * (rms_norm(X) W_gate),
    the two branches being interchangeable.  The paper's operator has no gain:
    pass g = ones.
    """
    W1 = _f64(W1, 2, "W1")
    W2 = _f64(W2, 2, "W2")
    if W1.shape != W2.shape:
        raise ValueError("W1 and W2 must have the same shape")
    Nrm = rms_norm(X, g, eps)
    if W1.shape[0] != Nrm.shape[1]:
        raise ValueError("W1/W2 must be [K,N]")
    return np.matmul(Nrm, W1) * np.matmul(Nrm, W2)


def swiglu(X, W_gate, W_up):
    """Y = silu(X @ W_gate) * (X @ W_up): no normalisation, no gain.  Paper Section 7.1, "SwiGLU"."""
    X = _f64(X, 2, "X")
    W_gate = _f64(W_gate, 2, "W_gate")
    W_up = _f64(W_up, 2, "W_up")
    if W_gate.shape != W_up.shape or W_gate.shape[0] != X.shape[1]:
        raise ValueError("W_gate and W_up must both be [K,N]")
    return silu(np.matmul(X, W_gate)) * np.matmul(X, W_up)


def softmax_matmul(X, W):
    """Y[M,N] = softmax(X, over k) @ W: the paper's running example (Figure 1(a): Softmax, then Matmul).

    softmax(x)[k] = exp(x[k]) / sum_j exp(x[j]), written out as the definition; the fused program of
    Figure 1(b) (exp and the row sum in the loop, the division after it) reaches the same result.
    In float64 exp overflows only above 709: callers keep |x| far below that (subtracting a constant
    from a row does not change its softmax, which one of the pins checks).
    """
    X = _f64(X, 2, "X")
    W = _f64(W, 2, "W")
    if W.shape[0] != X.shape[1]:
        raise ValueError("W must be [K,N]")
    P = np.empty_like(X)
    for m in range(X.shape[0]):
        e = np.exp(X[m])
        P[m] = e / np.sum(e)
    return np.matmul(P, W)


def gqa_decode_attention(Q, K, V, scale=1.0, qk_norm=False, eps=0.0):
    """O[b,g,:] = softmax(scale * Qn[b,g,:] . K[b]^T) . V[b], one query position, g query heads per KV head.

    Q is [B,G,D], K and V are [B,H,D] (H keys and values of D numbers each), O is [B,G,D].
    Paper Section 7.1, workloads "Attention" (qk_norm off: Qn = Q) and "QK-Attention" (qk_norm on:
    Qn = rms_norm(Q) over D, without gain, with the eps-inside-the-root reading used throughout).  The
    paper's formulas carry no 1/sqrt(D): scale = 1 is the paper's operator.  Plain loops over batch and
    head; the softmax is the definition, as in softmax_matmul.
    """
    Q = _f64(Q, 3, "Q")
    K = _f64(K, 3, "K")
    V = _f64(V, 3, "V")
    B, G, D = Q.shape
    if K.shape != V.shape or K.shape[0] != B or K.shape[2] != D:
        raise ValueError("K and V must both be [B,H,D]")
    one = np.ones(D)
    O = np.empty_like(Q)
    for b in range(B):
        Qn = rms_norm(Q[b], one, eps) if qk_norm else Q[b]
        S = float(scale) * np.matmul(Qn, K[b].T)          # [G,H]
        O[b] = softmax_matmul(S, V[b])
    return O
