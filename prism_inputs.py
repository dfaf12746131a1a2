"""Seeded synthetic inputs for the fused RMSNorm -> MatMul family.

This module only draws random numbers and converts between storage formats.
It holds none of the method's arithmetic, so both the CPU oracle's callers and
the HIP path's callers may use it; neither of those two imports the other.

The paper measures on tensor shapes taken from LLM layers, not on a dataset
(Section 7.1), so every input is dense i.i.d. noise of the workload's shape:
X ~ N(0,1), g ~ U(0.5,1.5), W ~ N(0, variance 1/K).  bf16 and fp16 workloads round
the fp32 draw once, to nearest even, and that stored value is the input for
both sides.
"""
from dataclasses import dataclass

import numpy as np

F32 = "f32"
BF16 = "bf16"
F16 = "f16"   # the paper's own precision (Section 7.1); stored as numpy float16


@dataclass(frozen=True)
class Workload:
    name: str
    dtype: str      # storage type of X, g, W*, Y
    M: int
    K: int
    N: int
    gated: bool
    eps: float
    seed: int


# The five benchmark configurations (index = position in the benchmark list).
WORKLOADS = (
    Workload("tiny_f32_rmsnorm_matmul", F32, 8, 256, 512, False, 1e-6, 0x5EED0000),
    Workload("decode_rmsnorm_matmul", BF16, 16, 4096, 4096, False, 1e-6, 0x5EED0001),
    Workload("prefill_qkv", BF16, 2048, 4096, 6144, False, 1e-6, 0x5EED0002),
    Workload("decode_gated_mlp", BF16, 8, 4096, 14336, True, 1e-6, 0x5EED0003),
    Workload("prefill_gated_mlp", BF16, 4096, 4096, 14336, True, 1e-6, 0x5EED0004),
)


def f32_to_bf16_bits(a):
    """Round float32 to bfloat16 (nearest, ties to even); returns uint16 bit patterns.

    Finite inputs only: NaN payloads are not preserved.
    """
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    # 32-bit arithmetic suffices for finite values (the largest, 0x7F7FFFFF, plus 0x8000 does not wrap)
    r = (u >> np.uint32(16)) & np.uint32(1)
    r += np.uint32(0x7FFF)
    r += u
    r >>= np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b):
    """Widen bfloat16 bit patterns (uint16) exactly to float32."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_f64(stored, dtype):
    """Exact float64 value of a stored array (fp32 array, or uint16 bf16 bit patterns)."""
    if dtype == BF16:
        return bf16_bits_to_f32(stored).astype(np.float64)
    if dtype == F16:
        return np.asarray(stored, dtype=np.float16).astype(np.float64)
    return np.asarray(stored, dtype=np.float32).astype(np.float64)


def _store(a32, dtype):
    if dtype == BF16:
        return f32_to_bf16_bits(a32)
    if dtype == F16:
        return np.ascontiguousarray(a32, dtype=np.float32).astype(np.float16)  # nearest even
    return np.ascontiguousarray(a32, dtype=np.float32)


def _stream(seed, tensor_id):
    return np.random.Generator(np.random.Philox(np.random.SeedSequence([int(seed), int(tensor_id)])))


def draw(dtype, M, K, N, gated, seed, w_scale=None):
    """Draw X[M,K], g[K] and W[K,N] (or W1, W2) in storage format.

    Returns a dict of stored arrays: float32 arrays for F32, uint16 bit
    patterns for BF16, float16 arrays for F16.  Each tensor has its own counter-based stream, so a
    tensor's values do not depend on which others were drawn.
    """
    std = (1.0 / np.sqrt(K)) if w_scale is None else float(w_scale)
    out = {}
    out["X"] = _store(_stream(seed, 0).standard_normal((M, K), dtype=np.float32), dtype)
    out["g"] = _store(_stream(seed, 1).random(K, dtype=np.float32) + np.float32(0.5), dtype)
    names = ("W1", "W2") if gated else ("W",)
    for i, nm in enumerate(names):
        w = _stream(seed, 2 + i).standard_normal((K, N), dtype=np.float32)
        w *= np.float32(std)
        out[nm] = _store(w, dtype)
    return out


def draw_softmax(dtype, M, K, N, seed, x_std=3.0):
    """Inputs of the softmax -> matmul operator (the paper's running example): X[M,K] ~ N(0, x_std^2),
    W[K,N] ~ N(0, 1).  With x_std = 3 a row's softmax is carried by a handful of entries, so the outputs
    are of order one and a tolerance of the form tol * (|y| + 1) is a real constraint."""
    x = _stream(seed, 0).standard_normal((M, K), dtype=np.float32) * np.float32(x_std)
    w = _stream(seed, 2).standard_normal((K, N), dtype=np.float32)
    return {"X": _store(x, dtype), "W": _store(w, dtype)}


def draw_attention(dtype, B, G, H, D, seed, q_std=1.0):
    """Inputs of group-query attention at one query position: Q[B,G,D] ~ N(0, q_std^2), K[B,H,D] and
    V[B,H,D] ~ N(0,1).  With D = 128 the scores have a standard deviation of about 11 q_std, so a softmax
    row is carried by few keys and the outputs are of order one."""
    q = _stream(seed, 0).standard_normal((B, G, D), dtype=np.float32) * np.float32(q_std)
    k = _stream(seed, 1).standard_normal((B, H, D), dtype=np.float32)
    v = _stream(seed, 2).standard_normal((B, H, D), dtype=np.float32)
    return {"Q": _store(q, dtype), "K": _store(k, dtype), "V": _store(v, dtype)}


def draw_workload(wl, M=None):
    """Inputs of a benchmark configuration; ``M`` keeps only the first M rows of X."""
    d = draw(wl.dtype, wl.M, wl.K, wl.N, wl.gated, wl.seed)
    if M is not None:
        d["X"] = np.ascontiguousarray(d["X"][:M])
    return d
