"""Helpers shared by the GPU tests: move stored inputs to the device, run the library, read back."""
import numpy as np

import prism_inputs as pi


DTYPE_CODE = {pi.F32: 0, pi.BF16: 1, pi.F16: 2}   # prism_dtype_t


def torch_dtype(dtype):
    import torch
    return {pi.F32: torch.float32, pi.BF16: torch.bfloat16, pi.F16: torch.float16}[dtype]


def to_device(stored, dtype):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(stored)).cuda()
    return t.view(torch.bfloat16) if dtype == pi.BF16 else t


def from_device(t, dtype):
    import torch
    if dtype == pi.BF16:
        return pi.to_f64(t.view(torch.uint16).cpu().numpy(), pi.BF16)
    return t.cpu().numpy().astype(np.float64)   # fp32 and fp16 widen exactly


def run_gpu(stored, dtype, gated, eps, poison=True):
    """One library call on the current device; returns Y as float64 (exact widening of what was stored)."""
    import torch
    import paper_2604_15272_amd as P
    X = to_device(stored["X"], dtype)
    g = to_device(stored["g"], dtype)
    M = X.shape[0]
    tdt = torch_dtype(dtype)
    if gated:
        W1, W2 = to_device(stored["W1"], dtype), to_device(stored["W2"], dtype)
        N = W1.shape[1]
        Y = torch.full((M, N), float("nan"), dtype=tdt, device="cuda") if poison else torch.empty(
            (M, N), dtype=tdt, device="cuda")
        P.prism_rmsnorm_gated_mlp(X, g, W1, W2, Y, eps=eps)
    else:
        W = to_device(stored["W"], dtype)
        N = W.shape[1]
        Y = torch.full((M, N), float("nan"), dtype=tdt, device="cuda") if poison else torch.empty(
            (M, N), dtype=tdt, device="cuda")
        P.prism_rmsnorm_matmul(X, g, W, Y, eps=eps)
    torch.cuda.synchronize()
    return from_device(Y, dtype)


def run_gpu_variant(stored, dtype, variant, eps):
    """The paper's own members of the family through their entry points.

    variant: "plain_nogain" (rms_norm without gain, then W), "glu" (RMSNorm-MLP: no activation),
    "glu_nogain", "swiglu" (no normalisation, no gain).  Returns Y as float64.
    """
    import torch
    import paper_2604_15272_amd as P
    X = to_device(stored["X"], dtype)
    g = to_device(stored["g"], dtype)
    M = X.shape[0]
    tdt = torch_dtype(dtype)
    names = ("W",) if variant == "plain_nogain" else ("W1", "W2")
    Ws = [to_device(stored[n], dtype) for n in names]
    N = Ws[0].shape[1]
    Y = torch.full((M, N), float("nan"), dtype=tdt, device="cuda")
    if variant == "plain_nogain":
        P.prism_rmsnorm_matmul(X, None, Ws[0], Y, eps=eps)
    elif variant == "glu":
        P.prism_rmsnorm_glu(X, g, Ws[0], Ws[1], Y, eps=eps)
    elif variant == "glu_nogain":
        P.prism_rmsnorm_glu(X, None, Ws[0], Ws[1], Y, eps=eps)
    elif variant == "swiglu":
        P.prism_swiglu(X, Ws[0], Ws[1], Y)
    else:
        raise ValueError(variant)
    torch.cuda.synchronize()
    return from_device(Y, dtype)


def run_oracle_variant(stored, dtype, variant, eps, rows=None):
    import oracle
    X = pi.to_f64(stored["X"], dtype)
    if rows is not None:
        X = X[rows]
    g = pi.to_f64(stored["g"], dtype)
    one = np.ones_like(g)
    if variant == "plain_nogain":
        return oracle.rmsnorm_matmul(X, one, pi.to_f64(stored["W"], dtype), eps)
    W1, W2 = pi.to_f64(stored["W1"], dtype), pi.to_f64(stored["W2"], dtype)
    if variant == "glu":
        return oracle.rmsnorm_glu(X, g, W1, W2, eps)
    if variant == "glu_nogain":
        return oracle.rmsnorm_glu(X, one, W1, W2, eps)
    if variant == "swiglu":
        return oracle.swiglu(X, W1, W2)
    raise ValueError(variant)


def run_gpu_softmax(stored, dtype):
    import torch
    import paper_2604_15272_amd as P
    X, W = to_device(stored["X"], dtype), to_device(stored["W"], dtype)
    Y = torch.full((X.shape[0], W.shape[1]), float("nan"), dtype=torch_dtype(dtype), device="cuda")
    P.prism_softmax_matmul(X, W, Y)
    torch.cuda.synchronize()
    return from_device(Y, dtype)


def run_oracle_softmax(stored, dtype, rows=None):
    import oracle
    X = pi.to_f64(stored["X"], dtype)
    if rows is not None:
        X = X[rows]
    return oracle.softmax_matmul(X, pi.to_f64(stored["W"], dtype))


def run_gpu_attention(stored, dtype, scale=1.0, qk_norm=False, eps=1e-6):
    import torch
    import paper_2604_15272_amd as P
    Q, K, V = (to_device(stored[k], dtype) for k in ("Q", "K", "V"))
    O = torch.full(Q.shape, float("nan"), dtype=torch_dtype(dtype), device="cuda")
    P.prism_gqa_decode_attention(Q, K, V, O, scale=scale, qk_norm=qk_norm, eps=eps)
    torch.cuda.synchronize()
    return from_device(O, dtype)


def run_oracle_attention(stored, dtype, scale=1.0, qk_norm=False, eps=1e-6):
    import oracle
    Q, K, V = (pi.to_f64(stored[k], dtype) for k in ("Q", "K", "V"))
    return oracle.gqa_decode_attention(Q, K, V, scale, qk_norm, float(np.float32(eps)))


def run_oracle(stored, dtype, gated, eps, rows=None):
    import oracle
    X = pi.to_f64(stored["X"], dtype)
    if rows is not None:
        X = X[rows]
    g = pi.to_f64(stored["g"], dtype)
    if gated:
        return oracle.rmsnorm_gated_mlp(X, g, pi.to_f64(stored["W1"], dtype), pi.to_f64(stored["W2"], dtype), eps)
    return oracle.rmsnorm_matmul(X, g, pi.to_f64(stored["W"], dtype), eps)


# fp32 and bf16: stated by the benchmark spec.  fp16: the bf16 bar scaled by the three extra significand bits
# (both error sources, the rounding of x * g on its way into the matrix core and the rounding of y,
# are 2^-11 instead of 2^-8 relative).
TOL = {pi.F32: 1e-5, pi.BF16: 2e-2, pi.F16: 2.5e-3}


def worst_error(y, yhat):
    """max |y - yhat| / (|yhat| + 1): the parity bar is this <= 1e-5 (fp32), 2e-2 (bf16), 2.5e-3 (fp16)."""
    y = np.asarray(y, dtype=np.float64)
    yhat = np.asarray(yhat, dtype=np.float64)
    assert y.shape == yhat.shape
    if y.size == 0:
        return 0.0
    err = np.abs(y - yhat) / (np.abs(yhat) + 1.0)
    return float(np.nanmax(np.where(np.isnan(err), np.inf, err)))


def assert_parity(y, yhat, dtype, what=""):
    w = worst_error(y, yhat)
    assert w <= TOL[dtype], f"{what}: worst |y-yhat|/(|yhat|+1) = {w:.3e} > {TOL[dtype]:.0e}"
    return w
