"""ctypes marshalling for the C ABI in include/prism.h."""
import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(HERE, "libprism.so")

PRISM_F32, PRISM_BF16, PRISM_F16 = 0, 1, 2
PRISM_OP_RMSNORM_MATMUL, PRISM_OP_RMSNORM_GATED_MLP, PRISM_OP_SOFTMAX_MATMUL = 0, 1, 2
PRISM_PATH_AUTO, PRISM_PATH_SIMPLE, PRISM_PATH_DECODE, PRISM_PATH_PREFILL, PRISM_PATH_ROWS = 0, 1, 2, 3, 4
PRISM_PATH_ATTENTION = 5
WORKSPACE_HEADER_BYTES = 262144


class PrismError(RuntimeError):
    def __init__(self, status, what):
        self.status = int(status)
        super().__init__(f"{what}: {prism_status_string(status)} (status {int(status)})")


class Plan(ctypes.Structure):
    _fields_ = [
        ("path", ctypes.c_int32), ("split_k", ctypes.c_int32),
        ("tile_m", ctypes.c_int32), ("tile_n", ctypes.c_int32),
        ("grid_x", ctypes.c_int32), ("grid_y", ctypes.c_int32),
        ("block", ctypes.c_int32), ("grid_z", ctypes.c_int32),
        ("workspace_bytes", ctypes.c_uint64),
    ]

    def as_dict(self):
        return {n: int(getattr(self, n)) for n, _ in self._fields_}


def library_path():
    return _LIB_PATH


def _load():
    if not os.path.exists(_LIB_PATH):
        raise ImportError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_2604_15272_amd.build` "
            "(there is no fallback implementation)")
    # PyTorch ships its own copy of the HIP runtime, and the memory and streams the library is handed
    # come from it: load torch first, so that the library's dependency on the runtime resolves to the
    # copy that is already in the process and not to a second one.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    L = ctypes.CDLL(_LIB_PATH)
    vp, i64, f32, i32, u64 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_float, ctypes.c_int32, ctypes.c_uint64
    L.prism_rmsnorm_matmul.argtypes = [vp, vp, vp, vp, i64, i64, i64, f32, i32, vp]
    L.prism_rmsnorm_gated_mlp.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, f32, i32, vp]
    for sfx in ("bf16", "f32"):
        getattr(L, f"prism_rmsnorm_matmul_{sfx}").argtypes = [vp, vp, vp, vp, i64, i64, i64, f32, vp]
        getattr(L, f"prism_rmsnorm_gated_mlp_{sfx}").argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, f32, vp]
        getattr(L, f"prism_rmsnorm_matmul_{sfx}").restype = i32
        getattr(L, f"prism_rmsnorm_gated_mlp_{sfx}").restype = i32
    L.prism_rmsnorm_matmul.restype = i32
    L.prism_rmsnorm_matmul_static.argtypes = [vp, vp, vp, vp, i64, i64, i64, f32, i32, vp]
    L.prism_rmsnorm_matmul_static.restype = i32
    L.prism_rmsnorm_gated_mlp.restype = i32
    L.prism_rmsnorm_glu.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, f32, i32, vp]
    L.prism_rmsnorm_glu.restype = i32
    L.prism_swiglu.argtypes = [vp, vp, vp, vp, i64, i64, i64, i32, vp]
    L.prism_swiglu.restype = i32
    L.prism_softmax_matmul.argtypes = [vp, vp, vp, i64, i64, i64, i32, vp]
    L.prism_softmax_matmul.restype = i32
    L.prism_gqa_decode_attention.argtypes = [vp, vp, vp, vp, i64, i64, i64, i64, f32, i32, f32, i32, vp]
    L.prism_gqa_decode_attention.restype = i32
    L.prism_attention_workspace_bytes.argtypes = [i64, i64, i64, i64, i32]
    L.prism_attention_workspace_bytes.restype = u64
    L.prism_attention_plan.argtypes = [i64, i64, i64, i64, i32, ctypes.POINTER(Plan)]
    L.prism_attention_plan.restype = i32
    L.prism_workspace_bytes.argtypes = [i32, i64, i64, i64, i32]
    L.prism_workspace_bytes.restype = u64
    L.prism_set_workspace.argtypes = [vp, u64]
    L.prism_set_workspace.restype = i32
    L.prism_set_stream_workspace.argtypes = [vp, vp, u64]
    L.prism_set_stream_workspace.restype = i32
    L.prism_probe_units.argtypes = [vp, u64, i32, vp, vp]
    L.prism_probe_units.restype = i32
    L.prism_probe_loads.argtypes = [vp, u64, i32, i32, i32, vp, vp]
    L.prism_probe_loads.restype = i32
    L.prism_probe_linear.argtypes = [vp, u64, i32, vp, vp]
    L.prism_probe_linear.restype = i32
    L.prism_probe_mfma.argtypes = [vp, i32, i32, vp]
    L.prism_probe_mfma.restype = i32
    L.prism_diag_set_cu_count.argtypes = [i32]
    L.prism_diag_set_cu_count.restype = i32
    L.prism_diag_cu_count.argtypes = []
    L.prism_diag_cu_count.restype = i32
    L.prism_plan.argtypes = [i32, i64, i64, i64, i32, ctypes.POINTER(Plan)]
    L.prism_plan.restype = i32
    L.prism_plan_table_set.argtypes = [i32, i64, i64, i64, i32, i32, i32, i32]
    L.prism_plan_table_set.restype = i32
    L.prism_plan_table_clear.argtypes = []
    L.prism_plan_table_clear.restype = i32
    L.prism_plan_table_size.argtypes = []
    L.prism_plan_table_size.restype = i32
    L.prism_set_override.argtypes = [i32, i32, i32]
    L.prism_set_override.restype = i32
    L.prism_status_string.argtypes = [i32]
    L.prism_status_string.restype = ctypes.c_char_p
    L.prism_probe_stream.argtypes = [vp, vp, i64, i64, i32, vp]
    L.prism_probe_stream.restype = i32
    L.prism_set_stream_balance.argtypes = [i32, i32]
    L.prism_stream_partition_blocks.argtypes = [i32] * 9 + [ctypes.POINTER(i32), ctypes.POINTER(i32)]
    L.prism_stream_partition_blocks.restype = i32
    L.prism_set_stream_balance.restype = i32
    L.prism_version.argtypes = []
    L.prism_version.restype = i32
    return L


lib = _load()


def prism_status_string(status):
    return lib.prism_status_string(int(status)).decode()


def prism_version():
    return int(lib.prism_version())


def _ptr(t):
    """Device address of a torch tensor (or a plain integer address)."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if not t.is_contiguous():
        raise ValueError("tensors must be contiguous")
    return t.data_ptr()


def _stream_handle(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _dtype_of(t, dtype):
    if dtype is not None:
        return int(dtype)
    import torch
    if t.dtype == torch.float32:
        return PRISM_F32
    if t.dtype == torch.bfloat16:
        return PRISM_BF16
    if t.dtype == torch.float16:
        return PRISM_F16
    raise TypeError(f"unsupported tensor dtype {t.dtype}")


def prism_workspace_bytes(op, M, K, N, dtype):
    return int(lib.prism_workspace_bytes(int(op), int(M), int(K), int(N), int(dtype)))


def prism_set_workspace(dev_ptr, nbytes):
    st = lib.prism_set_workspace(dev_ptr, int(nbytes))
    if st != 0:
        raise PrismError(st, "prism_set_workspace")


def prism_set_stream_workspace(stream, dev_ptr, nbytes):
    st = lib.prism_set_stream_workspace(_stream_handle(stream), dev_ptr, int(nbytes))
    if st != 0:
        raise PrismError(st, "prism_set_stream_workspace")


def prism_diag_set_cu_count(cus=0):
    """Plan for `cus` compute units (0: the current device's count)."""
    st = lib.prism_diag_set_cu_count(int(cus))
    if st != 0:
        raise PrismError(st, "prism_diag_set_cu_count")


def prism_diag_cu_count():
    return int(lib.prism_diag_cu_count())


def prism_plan(op, M, K, N, dtype):
    p = Plan()
    st = lib.prism_plan(int(op), int(M), int(K), int(N), int(dtype), ctypes.byref(p))
    if st != 0:
        raise PrismError(st, "prism_plan")
    return p.as_dict()


def prism_set_override(path=0, split_k=0, variant=0):
    st = lib.prism_set_override(int(path), int(split_k), int(variant))
    if st != 0:
        raise PrismError(st, "prism_set_override")


def prism_set_stream_balance(slow_units=0, mode=0):
    """Without arguments: the library's defaults (no unit taken to be slow, no two-pass partition)."""
    st = lib.prism_set_stream_balance(int(slow_units), int(mode))
    if st != 0:
        raise PrismError(st, "prism_set_stream_balance")


def prism_stream_partition_blocks(workgroups, kblocks, n_tiles, slow_tiles, wg, tile, period=8, w_fast=4, w_slow=5):
    """(first, count) of the K-blocks of `tile` that workgroup `wg` of a weighted partition works on."""
    first, count = ctypes.c_int32(0), ctypes.c_int32(0)
    st = lib.prism_stream_partition_blocks(int(workgroups), int(kblocks), int(n_tiles), int(slow_tiles), int(period),
                                           int(w_fast), int(w_slow), int(wg), int(tile), ctypes.byref(first),
                                           ctypes.byref(count))
    if st != 0:
        raise PrismError(st, "prism_stream_partition_blocks")
    return first.value, count.value


def prism_plan_table_set(op, M, K, N, dtype, path, split_k=0, variant=0):
    st = lib.prism_plan_table_set(int(op), int(M), int(K), int(N), int(dtype), int(path), int(split_k), int(variant))
    if st != 0:
        raise PrismError(st, "prism_plan_table_set")


def prism_plan_table_clear():
    lib.prism_plan_table_clear()


def prism_plan_table_size():
    return int(lib.prism_plan_table_size())


# Device memory for the split-K workspace comes from torch (one tensor per device, grown on demand).
_workspaces = {}


def ensure_workspace(nbytes, device=None):
    """Make sure the current device has a registered workspace of at least nbytes."""
    import torch
    dev = torch.cuda.current_device() if device is None else torch.device(device).index
    cur = _workspaces.get(dev)
    if nbytes <= 0 or (cur is not None and cur.numel() >= nbytes):
        return
    torch.cuda.synchronize(dev)
    size = max(int(nbytes), 2 * WORKSPACE_HEADER_BYTES)
    buf = torch.empty(size, dtype=torch.uint8, device=f"cuda:{dev}")
    with torch.cuda.device(dev):
        prism_set_workspace(buf.data_ptr(), size)
    _workspaces[dev] = buf


def prism_rmsnorm_matmul(X, g, W, Y, M=None, K=None, N=None, eps=1e-6, dtype=None, stream=None):
    """Y[M,N] = rms_norm(X; g, eps) @ W on the GPU.  Tensors are torch CUDA tensors or addresses."""
    if M is None:
        M, K = X.shape
        N = W.shape[1]
    dt = _dtype_of(X, dtype)
    if not isinstance(X, int):
        ensure_workspace(prism_workspace_bytes(PRISM_OP_RMSNORM_MATMUL, M, K, N, dt))
    st = lib.prism_rmsnorm_matmul(_ptr(X), _ptr(g), _ptr(W), _ptr(Y), int(M), int(K), int(N), float(eps), dt,
                                  _stream_handle(stream))
    if st != 0:
        raise PrismError(st, "prism_rmsnorm_matmul")
    return Y


STATIC_SCRATCH_BYTES = 8388608
PROBE_LOADS_BYTES = 1048576   # PRISM_PROBE_LOADS_BYTES: what prism_probe_loads reads


def prism_rmsnorm_matmul_static(X, g, W, Y, M=None, K=None, N=None, eps=1e-6, dtype=None, stream=None):
    """prism_rmsnorm_matmul through the library's own static device scratch: registers and allocates nothing."""
    if M is None:
        M, K = X.shape
        N = W.shape[1]
    st = lib.prism_rmsnorm_matmul_static(_ptr(X), _ptr(g), _ptr(W), _ptr(Y), int(M), int(K), int(N), float(eps),
                                         _dtype_of(X, dtype), _stream_handle(stream))
    if st != 0:
        raise PrismError(st, "prism_rmsnorm_matmul_static")
    return Y


def prism_rmsnorm_gated_mlp(X, g, W1, W2, Y, M=None, K=None, N=None, eps=1e-6, dtype=None, stream=None):
    """Y[M,N] = silu(Nrm @ W1) * (Nrm @ W2), Nrm = rms_norm(X; g, eps), on the GPU."""
    if M is None:
        M, K = X.shape
        N = W1.shape[1]
    dt = _dtype_of(X, dtype)
    if not isinstance(X, int):
        ensure_workspace(prism_workspace_bytes(PRISM_OP_RMSNORM_GATED_MLP, M, K, N, dt))
    st = lib.prism_rmsnorm_gated_mlp(_ptr(X), _ptr(g), _ptr(W1), _ptr(W2), _ptr(Y), int(M), int(K), int(N),
                                     float(eps), dt, _stream_handle(stream))
    if st != 0:
        raise PrismError(st, "prism_rmsnorm_gated_mlp")
    return Y


def prism_rmsnorm_glu(X, g, W1, W2, Y, M=None, K=None, N=None, eps=1e-6, dtype=None, stream=None):
    """Y[M,N] = (Nrm @ W1) * (Nrm @ W2), Nrm = rms_norm(X; g, eps): the paper's RMSNorm-MLP (no activation)."""
    if M is None:
        M, K = X.shape
        N = W1.shape[1]
    dt = _dtype_of(X, dtype)
    if not isinstance(X, int):
        ensure_workspace(prism_workspace_bytes(PRISM_OP_RMSNORM_GATED_MLP, M, K, N, dt))
    st = lib.prism_rmsnorm_glu(_ptr(X), _ptr(g), _ptr(W1), _ptr(W2), _ptr(Y), int(M), int(K), int(N), float(eps), dt,
                               _stream_handle(stream))
    if st != 0:
        raise PrismError(st, "prism_rmsnorm_glu")
    return Y


def prism_swiglu(X, W_gate, W_up, Y, M=None, K=None, N=None, dtype=None, stream=None):
    """Y[M,N] = silu(X @ W_gate) * (X @ W_up): the paper's SwiGLU (no normalisation, no gain)."""
    if M is None:
        M, K = X.shape
        N = W_gate.shape[1]
    dt = _dtype_of(X, dtype)
    if not isinstance(X, int):
        ensure_workspace(prism_workspace_bytes(PRISM_OP_RMSNORM_GATED_MLP, M, K, N, dt))
    st = lib.prism_swiglu(_ptr(X), _ptr(W_gate), _ptr(W_up), _ptr(Y), int(M), int(K), int(N), dt,
                          _stream_handle(stream))
    if st != 0:
        raise PrismError(st, "prism_swiglu")
    return Y


def prism_softmax_matmul(X, W, Y, M=None, K=None, N=None, dtype=None, stream=None):
    """Y[M,N] = softmax(X, over k) @ W: the paper's running example (Figure 1)."""
    if M is None:
        M, K = X.shape
        N = W.shape[1]
    dt = _dtype_of(X, dtype)
    if not isinstance(X, int):
        ensure_workspace(prism_workspace_bytes(PRISM_OP_SOFTMAX_MATMUL, M, K, N, dt))
    st = lib.prism_softmax_matmul(_ptr(X), _ptr(W), _ptr(Y), int(M), int(K), int(N), dt, _stream_handle(stream))
    if st != 0:
        raise PrismError(st, "prism_softmax_matmul")
    return Y


def prism_attention_plan(B, G, H, D, dtype):
    p = Plan()
    st = lib.prism_attention_plan(int(B), int(G), int(H), int(D), int(dtype), ctypes.byref(p))
    if st != 0:
        raise PrismError(st, "prism_attention_plan")
    return p.as_dict()


def prism_gqa_decode_attention(Q, K, V, O, scale=1.0, qk_norm=False, eps=1e-6, dtype=None, stream=None):
    """O[B,G,D] = softmax(scale * Qn @ K^T) @ V per batch entry (Q [B,G,D]; K, V [B,H,D]); Qn = rms_norm(Q) if qk_norm."""
    B, G, D = Q.shape
    H = K.shape[1]
    dt = _dtype_of(Q, dtype)
    ensure_workspace(int(lib.prism_attention_workspace_bytes(B, G, H, D, dt)))
    st = lib.prism_gqa_decode_attention(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), B, G, H, D, float(scale), int(bool(qk_norm)),
                                        float(eps), dt, _stream_handle(stream))
    if st != 0:
        raise PrismError(st, "prism_gqa_decode_attention")
    return O
