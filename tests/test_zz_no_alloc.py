"""The entry point that allocates nothing (prism_rmsnorm_matmul_static) against prism_rmsnorm_matmul.

Same kernels, the split-K partials in the library's static device array instead of the registered workspace: the
outputs must agree bit for bit, and with the oracle within the stated bar.  Two calls in a row, the second with a
smaller input (the array keeps the first call's contents); then a call that needs more than the array holds.
"""
import ctypes

import numpy as np
import pytest

import prism_inputs as pi
from gpu_util import assert_parity, run_oracle, to_device, from_device

pytestmark = pytest.mark.gpu


def _both(P, M, K, N, seed):
    import torch
    stored = pi.draw(pi.BF16, M, K, N, False, seed)
    X, g, W = (to_device(stored[k], pi.BF16) for k in ("X", "g", "W"))
    plan = P.prism_plan(P.PRISM_OP_RMSNORM_MATMUL, M, K, N, P.PRISM_BF16)
    assert plan["split_k"] > 1 and 0 < plan["workspace_bytes"] <= P.STATIC_SCRATCH_BYTES, plan
    Y_ref = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
    P.prism_rmsnorm_matmul(X, g, W, Y_ref)
    Y = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
    vp, i64 = ctypes.c_void_p, ctypes.c_int64
    print(f"static entry point: M={M} K={K} N={N} plan={plan}", flush=True)
    st = P.lib.prism_rmsnorm_matmul_static(vp(X.data_ptr()), vp(g.data_ptr()), vp(W.data_ptr()), vp(Y.data_ptr()),
                                           i64(M), i64(K), i64(N), ctypes.c_float(1e-6), ctypes.c_int32(P.PRISM_BF16),
                                           vp(torch.cuda.current_stream().cuda_stream))
    assert st == 0, P.prism_status_string(st)
    torch.cuda.synchronize()
    assert torch.equal(Y.view(torch.uint16), Y_ref.view(torch.uint16))
    assert_parity(from_device(Y, pi.BF16), run_oracle(stored, pi.BF16, False, 1e-6), pi.BF16, f"static M={M} K={K} N={N}")


def test_static_scratch_entry_point_two_calls_in_a_row_then_too_large():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2604_15272_amd as P
    P.prism_set_override(0, 0, 0)
    _both(P, 16, 4096, 4096, 8101)     # benchmark configuration 2: eight K-slices, 2.3 MB of scratch
    _both(P, 7, 1024, 1000, 8102)      # smaller, ragged: the array still holds the first call's partials
    _both(P, 16, 4096, 4096, 8103)
    # a call that needs more scratch than the array holds is refused, and nothing is launched
    M, K, N = 64, 8192, 8192
    need = P.prism_workspace_bytes(P.PRISM_OP_RMSNORM_MATMUL, M, K, N, P.PRISM_BF16)
    assert need > P.STATIC_SCRATCH_BYTES, need
    X = torch.zeros((M, K), dtype=torch.bfloat16, device="cuda")
    W = torch.zeros((K, N), dtype=torch.bfloat16, device="cuda")
    Y = torch.full((M, N), 7.0, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(P.PrismError) as e:
        P.prism_rmsnorm_matmul_static(X, None, W, Y)
    assert e.value.status == 3
    torch.cuda.synchronize()
    assert torch.all(Y == 7.0)
    # calls that need no scratch run as usual (prefill kernel, plain kernel)
    for dt, M, K, N in ((pi.BF16, 300, 512, 384), (pi.F32, 8, 256, 512)):
        stored = pi.draw(dt, M, K, N, False, 8104)
        Xd, gd, Wd = (to_device(stored[k], dt) for k in ("X", "g", "W"))
        Yd = torch.empty((M, N), dtype=Xd.dtype, device="cuda")
        P.prism_rmsnorm_matmul_static(Xd, gd, Wd, Yd)
        torch.cuda.synchronize()
        assert_parity(from_device(Yd, dt), run_oracle(stored, dt, False, 1e-6), dt, f"static, no scratch, {dt}")
