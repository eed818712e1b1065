"""Thin ctypes face of libsbi_gemm.so: argument marshalling only.

Every function takes torch CUDA tensors (device memory owned by the caller), passes their
data pointers and the current HIP stream through the C ABI declared in include/sbi_gemm.h
and raises SbiError on a non-zero status.  Nothing is computed here and there is no
fallback: a missing library is an error.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
# SBI_GEMM_LIB points at another build of the same library (e.g. one with tracing compiled in)
LIB_PATH = os.environ.get("SBI_GEMM_LIB") or os.path.join(_HERE, "libsbi_gemm.so")

MAX_BATCH = 64
# sbi_epilogue
EPI_NONE, EPI_BIAS, EPI_BIAS_GELU, EPI_BIAS_RESIDUAL, EPI_GELU, EPI_RESIDUAL = range(6)
EPILOGUES = {"none": EPI_NONE, "bias": EPI_BIAS, "bias_gelu": EPI_BIAS_GELU,
             "bias_residual": EPI_BIAS_RESIDUAL, "gelu": EPI_GELU, "residual": EPI_RESIDUAL}
# sbi_path
PATH_AUTO, PATH_STREAM, PATH_MFMA, PATH_STREAMK = 0, 1, 2, 3
PATH_NAMES = {PATH_AUTO: "auto", PATH_STREAM: "stream", PATH_MFMA: "mfma", PATH_STREAMK: "streamk"}
# sbi_status
OK = 0
STATUS_NAMES = ["SBI_OK", "SBI_ERR_NULL", "SBI_ERR_SHAPE", "SBI_ERR_ALIGN", "SBI_ERR_BATCH",
                "SBI_ERR_LAYOUT_MISMATCH", "SBI_ERR_WORKSPACE", "SBI_ERR_EPILOGUE", "SBI_ERR_HIP",
                "SBI_ERR_OVERLAP", "SBI_ERR_TUNING"]

EXPORTS = ["sbi_gemm_layout_bytes", "sbi_gemm_workspace_bytes", "sbi_gemm_layout_weights",
           "sbi_gemm_unlayout_weights", "sbi_gemm_layout_check", "sbi_gemm", "sbi_gemm_ex",
           "sbi_gemm_plan", "sbi_layer_gemms", "sbi_layer_workspace_bytes", "sbi_status_string",
           "sbi_version", "sbi_calib_read", "sbi_calib_copy", "sbi_layer_plan", "sbi_gemm_ln",
           "sbi_gemm_ln_workspace_bytes", "sbi_gemm_i8_layout_bytes", "sbi_gemm_i8_workspace_bytes",
           "sbi_gemm_i8_quantize_weights", "sbi_gemm_i8_layout_weights", "sbi_gemm_i8_layout_check", "sbi_gemm_i8",
           "sbi_gemm_moments", "sbi_attn_decode", "sbi_attn_decode_workspace_bytes",
           "sbi_attn_decode_ragged", "sbi_gemm_static", "sbi_layer_tune", "sbi_gemm_tune", "sbi_gemm_i8_ln",
           "sbi_kernel_registers"]


class SbiError(RuntimeError):
    def __init__(self, status, where):
        self.status = int(status)
        name = STATUS_NAMES[self.status] if 0 <= self.status < len(STATUS_NAMES) else str(status)
        super().__init__(f"{where}: {name} ({status_string(self.status)})")


class Tuning(ctypes.Structure):
    _fields_ = [("path", ctypes.c_int32), ("split_k", ctypes.c_int32),
                ("waves", ctypes.c_int32), ("depth", ctypes.c_int32), ("blocks", ctypes.c_int32),
                ("panels", ctypes.c_int32), ("layernorm", ctypes.c_int32), ("int8", ctypes.c_int32)]


class LayerNorm(ctypes.Structure):
    _fields_ = [("gamma", ctypes.c_void_p), ("beta", ctypes.c_void_p), ("eps", ctypes.c_float),
                ("moments", ctypes.c_void_p)]


class Plan(ctypes.Structure):
    _fields_ = [("path", ctypes.c_int32), ("waves", ctypes.c_int32), ("depth", ctypes.c_int32),
                ("split_k", ctypes.c_int32), ("ksteps_per_split", ctypes.c_int32),
                ("ksteps_per_chunk", ctypes.c_int32), ("grid", ctypes.c_int32), ("block", ctypes.c_int32),
                ("panels", ctypes.c_int32), ("reserved", ctypes.c_int32),
                ("lds_bytes", ctypes.c_int64), ("workspace_bytes", ctypes.c_int64)]

    def as_dict(self):
        return {f: getattr(self, f) for f, _ in self._fields_}


class Layer(ctypes.Structure):
    _fields_ = [("Wqkv", ctypes.c_void_p), ("Wout", ctypes.c_void_p), ("Wffn1", ctypes.c_void_p),
                ("Wffn2", ctypes.c_void_p), ("bqkv", ctypes.c_void_p), ("bout", ctypes.c_void_p),
                ("bffn1", ctypes.c_void_p), ("bffn2", ctypes.c_void_p),
                ("h", ctypes.c_int64), ("n_qkv", ctypes.c_int64), ("k_out", ctypes.c_int64),
                ("n_ffn1", ctypes.c_int64), ("k_ffn2", ctypes.c_int64), ("ffn1_gelu", ctypes.c_int32),
                ("ln1_gamma", ctypes.c_void_p), ("ln1_beta", ctypes.c_void_p),
                ("ln2_gamma", ctypes.c_void_p), ("ln2_beta", ctypes.c_void_p), ("ln_eps", ctypes.c_float),
                ("sqkv", ctypes.c_void_p), ("sout", ctypes.c_void_p), ("sffn1", ctypes.c_void_p),
                ("sffn2", ctypes.c_void_p)]


_lib = None


def load():
    """Open libsbi_gemm.so (built by `python -m paper_2207_00032_amd.csrc.build` or
    __graft_entry__.build()).  Raises if it is missing: there is no other implementation."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} not found: build the HIP library first "
                          f"(python paper_2207_00032_amd/csrc/build.py)")
    L = ctypes.CDLL(LIB_PATH)
    vp, i64, sz, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_size_t, ctypes.c_int32
    L.sbi_gemm_layout_bytes.restype = sz
    L.sbi_gemm_layout_bytes.argtypes = [i64, i64]
    L.sbi_gemm_workspace_bytes.restype = sz
    L.sbi_gemm_workspace_bytes.argtypes = [i64, i64, i64]
    L.sbi_gemm_layout_weights.restype = i32
    L.sbi_gemm_layout_weights.argtypes = [vp, i64, i64, vp, sz, vp]
    L.sbi_gemm_unlayout_weights.restype = i32
    L.sbi_gemm_unlayout_weights.argtypes = [vp, i64, i64, vp, vp]
    L.sbi_gemm_layout_check.restype = i32
    L.sbi_gemm_layout_check.argtypes = [vp, i64, i64, vp]
    L.sbi_gemm.restype = i32
    L.sbi_gemm.argtypes = [vp, i64, i64, vp, i64, vp, vp, i32, vp, vp, sz, vp]
    L.sbi_gemm_static.restype = i32
    L.sbi_gemm_static.argtypes = [vp, i64, i64, vp, i64, vp, vp, i32, vp, vp]
    L.sbi_gemm_ex.restype = i32
    L.sbi_gemm_ex.argtypes = [vp, i64, i64, vp, i64, vp, vp, i32, vp, vp, sz, vp, ctypes.POINTER(Tuning)]
    L.sbi_gemm_ln.restype = i32
    L.sbi_gemm_ln.argtypes = [vp, i64, i64, vp, i64, ctypes.POINTER(LayerNorm), vp, vp, i32, vp, vp, sz, vp,
                              ctypes.POINTER(Tuning)]
    L.sbi_gemm_moments.restype = i32
    L.sbi_gemm_moments.argtypes = [vp, i64, i64, vp, i64, ctypes.POINTER(LayerNorm), vp, vp, i32, vp, vp, vp, sz, vp,
                                   ctypes.POINTER(Tuning)]
    L.sbi_attn_decode_workspace_bytes.restype = sz
    L.sbi_attn_decode_workspace_bytes.argtypes = [i64, i32, i32, i64]
    L.sbi_attn_decode.restype = i32
    L.sbi_attn_decode.argtypes = [vp, vp, vp, i64, i32, i32, i64, i64, ctypes.c_float, vp, vp, sz, vp]
    L.sbi_attn_decode_ragged.restype = i32
    L.sbi_attn_decode_ragged.argtypes = [vp, vp, vp, i64, i32, i32, i64, vp, i64, ctypes.c_float, vp, vp, sz, vp]
    L.sbi_gemm_ln_workspace_bytes.restype = sz
    L.sbi_gemm_ln_workspace_bytes.argtypes = [i64, i64, i64]
    L.sbi_gemm_i8_layout_bytes.restype = sz
    L.sbi_gemm_i8_layout_bytes.argtypes = [i64, i64]
    L.sbi_gemm_i8_workspace_bytes.restype = sz
    L.sbi_gemm_i8_workspace_bytes.argtypes = [i64, i64, i64]
    L.sbi_gemm_i8_quantize_weights.restype = i32
    L.sbi_gemm_i8_quantize_weights.argtypes = [vp, i64, i64, vp, vp, vp]
    L.sbi_gemm_i8_layout_weights.restype = i32
    L.sbi_gemm_i8_layout_weights.argtypes = [vp, i64, i64, vp, sz, vp]
    L.sbi_gemm_i8_layout_check.restype = i32
    L.sbi_gemm_i8_layout_check.argtypes = [vp, i64, i64, vp]
    L.sbi_gemm_i8.restype = i32
    L.sbi_gemm_i8.argtypes = [vp, vp, i64, i64, vp, i64, vp, vp, i32, vp, vp, sz, vp, ctypes.POINTER(Tuning)]
    L.sbi_gemm_i8_ln.restype = i32
    L.sbi_gemm_i8_ln.argtypes = [vp, vp, i64, i64, vp, i64, ctypes.POINTER(LayerNorm), vp, vp, i32, vp, vp, sz, vp,
                                 ctypes.POINTER(Tuning)]
    L.sbi_gemm_plan.restype = i32
    L.sbi_gemm_plan.argtypes = [i64, i64, i64, ctypes.POINTER(Tuning), ctypes.POINTER(Plan)]
    L.sbi_layer_gemms.restype = i32
    L.sbi_layer_gemms.argtypes = [ctypes.POINTER(Layer), i64] + [vp] * 9 + [vp, sz, vp]
    L.sbi_layer_workspace_bytes.restype = sz
    L.sbi_layer_workspace_bytes.argtypes = [ctypes.POINTER(Layer), i64]
    L.sbi_layer_plan.restype = i32
    L.sbi_layer_plan.argtypes = [ctypes.POINTER(Layer), i64, i32, ctypes.POINTER(Plan), ctypes.POINTER(i32)]
    L.sbi_layer_tune.restype = i32
    L.sbi_layer_tune.argtypes = [vp, i32, i64] + [vp] * 9 + [vp, sz, vp, vp]
    L.sbi_gemm_tune.restype = i32
    L.sbi_gemm_tune.argtypes = [vp, i32, i64, i64, vp, i64, vp, vp, i32, vp, vp, sz, vp, vp]
    L.sbi_kernel_registers.restype = i32
    L.sbi_kernel_registers.argtypes = [i64, i32, i32, i32, i32, vp, vp]
    L.sbi_calib_read.restype = i32
    L.sbi_calib_read.argtypes = [vp, sz, vp, sz, i32, i32, i32, i32, vp]
    L.sbi_calib_copy.restype = i32
    L.sbi_calib_copy.argtypes = [vp, vp, sz, vp]
    L.sbi_status_string.restype = ctypes.c_char_p
    L.sbi_status_string.argtypes = [i32]
    L.sbi_version.restype = i32
    L.sbi_version.argtypes = []
    _lib = L
    return L


def status_string(status):
    return load().sbi_status_string(int(status)).decode()


def _check(status, where):
    if status != OK:
        raise SbiError(status, where)


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _need(t, shape, what):
    """The C ABI takes bare pointers: make sure the tensor behind one really has the extent the call
    will read or write (an undersized tensor would be a GPU memory fault, not an error code)."""
    import torch
    if t is None:
        return
    if not (t.is_cuda and t.dtype == torch.float16 and t.is_contiguous() and tuple(t.shape) == tuple(shape)):
        raise ValueError(f"{what}: expected a contiguous CUDA fp16 tensor of shape {tuple(shape)}, got "
                         f"{t.dtype} {tuple(t.shape)} on {t.device}")


def _need_bytes(t, nbytes, what):
    if t is None:
        if nbytes:
            raise ValueError(f"{what}: missing ({nbytes} bytes needed)")
        return
    if not t.is_cuda or not t.is_contiguous() or t.numel() * t.element_size() < nbytes:
        raise ValueError(f"{what}: needs {nbytes} contiguous bytes on the GPU, has {t.numel() * t.element_size()}")


def _stream():
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _tuning(path=PATH_AUTO, split_k=0, waves=0, depth=0, blocks=0, panels=0, layernorm=0, int8=0):
    if path == PATH_AUTO and not (split_k or waves or depth or blocks or panels or layernorm or int8):
        return None
    return ctypes.pointer(Tuning(int(path), int(split_k), int(waves), int(depth), int(blocks), int(panels),
                                 1 if layernorm else 0, 1 if int8 else 0))


# ---------------------------------------------------------------------------------- sizes
def layout_bytes(K, N):
    return int(load().sbi_gemm_layout_bytes(K, N))


def workspace_bytes(B, K, N):
    return int(load().sbi_gemm_workspace_bytes(B, K, N))


def ln_workspace_bytes(B, K, N):
    return int(load().sbi_gemm_ln_workspace_bytes(B, K, N))


def plan(B, K, N, path=PATH_AUTO, split_k=0, waves=0, depth=0, blocks=0, panels=0, layernorm=False, int8=False):
    pl = Plan()
    _check(load().sbi_gemm_plan(B, K, N, _tuning(path, split_k, waves, depth, blocks, panels, layernorm, int8),
                                ctypes.byref(pl)), "sbi_gemm_plan")
    return pl.as_dict()


# ---------------------------------------------------------------------------------- device calls
def new_workspace(nbytes, device="cuda"):
    """A zero-filled workspace tensor (the counters in it must start at zero)."""
    import torch
    return torch.zeros(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def layout_weights(W):
    """W: fp16 [K,N] CUDA tensor -> laid-out uint8 CUDA tensor (header + tiles)."""
    import torch
    assert W.is_cuda and W.dtype == torch.float16 and W.dim() == 2 and W.is_contiguous()
    K, N = W.shape
    out = torch.empty(layout_bytes(K, N), dtype=torch.uint8, device=W.device)
    _check(load().sbi_gemm_layout_weights(_ptr(W), K, N, _ptr(out), out.numel(), _stream()),
           "sbi_gemm_layout_weights")
    return out


def unlayout_weights(Wl, K, N):
    import torch
    out = torch.empty((K, N), dtype=torch.float16, device=Wl.device)
    _check(load().sbi_gemm_unlayout_weights(_ptr(Wl), K, N, _ptr(out), _stream()), "sbi_gemm_unlayout_weights")
    return out


def layout_check(Wl, K, N):
    """Status of the header check (0 = the buffer was laid out for exactly (K, N))."""
    return int(load().sbi_gemm_layout_check(_ptr(Wl), K, N, _stream()))


def i8_layout_bytes(K, N):
    return int(load().sbi_gemm_i8_layout_bytes(K, N))


def i8_workspace_bytes(B, K, N):
    return int(load().sbi_gemm_i8_workspace_bytes(B, K, N))


def i8_quantize_weights(W):
    """W: fp16 [K,N] CUDA tensor -> (codes int8 [K,N], scales float32 [N]), per output channel."""
    import torch
    K, N = W.shape
    _need(W, (K, N), "W")
    Wq = torch.empty((K, N), dtype=torch.int8, device=W.device)
    sw = torch.empty((N,), dtype=torch.float32, device=W.device)
    _check(load().sbi_gemm_i8_quantize_weights(_ptr(W), K, N, _ptr(Wq), _ptr(sw), _stream()),
           "sbi_gemm_i8_quantize_weights")
    return Wq, sw


def i8_layout_weights(Wq):
    """Wq: int8 [K,N] CUDA tensor of codes -> laid-out uint8 CUDA tensor (header + tiles)."""
    import torch
    assert Wq.is_cuda and Wq.dtype == torch.int8 and Wq.dim() == 2 and Wq.is_contiguous()
    K, N = Wq.shape
    out = torch.empty(i8_layout_bytes(K, N), dtype=torch.uint8, device=Wq.device)
    _check(load().sbi_gemm_i8_layout_weights(_ptr(Wq), K, N, _ptr(out), out.numel(), _stream()),
           "sbi_gemm_i8_layout_weights")
    return out


def i8_layout_check(Wl, K, N):
    return int(load().sbi_gemm_i8_layout_check(_ptr(Wl), K, N, _stream()))


def gemm_i8(Wl, sw, K, N, X, bias=None, residual=None, epilogue=EPI_NONE, out=None, workspace=None,
            path=PATH_AUTO, split_k=0, waves=0, depth=0, panels=0, layernorm=None):
    """Y = epilogue((quantize(X) @ Wq) * sx * sw + bias) through sbi_gemm_i8, or, with
    layernorm=(gamma, beta, eps), the same on the layer-normalised rows through sbi_gemm_i8_ln.
    Returns Y (fp16 [B,N])."""
    import torch
    assert X.is_cuda and X.dtype == torch.float16 and X.dim() == 2 and X.is_contiguous()
    B = X.shape[0]
    if isinstance(epilogue, str):
        epilogue = EPILOGUES[epilogue]
    if out is None:
        out = torch.empty((B, N), dtype=torch.float16, device=X.device)
    _need(X, (B, K), "X")
    _need(bias, (N,), "bias")
    _need(residual, (B, N), "residual")
    _need(out, (B, N), "out")
    _need_bytes(Wl, i8_layout_bytes(K, N), "laid-out int8 weights")
    if not (sw.is_cuda and sw.dtype == torch.float32 and sw.is_contiguous() and tuple(sw.shape) == (N,)):
        raise ValueError("w_scales: expected a contiguous CUDA float32 tensor of shape (N,)")
    tune = _tuning(path, split_k, waves, depth, panels=panels)
    if workspace is None:
        need = plan(B, K, N, path, split_k, waves, depth, panels=panels, int8=True,
                    layernorm=layernorm is not None)["workspace_bytes"]
        workspace = new_workspace(need, X.device) if need else None
    ws_len = workspace.numel() * workspace.element_size() if workspace is not None else 0
    if layernorm is not None:
        gamma, beta, eps = layernorm
        _need(gamma, (K,), "gamma")
        _need(beta, (K,), "beta")
        ln = LayerNorm(gamma.data_ptr(), beta.data_ptr(), float(eps), None)
        st = load().sbi_gemm_i8_ln(_ptr(Wl), _ptr(sw), K, N, _ptr(X), B, ctypes.byref(ln), _ptr(bias), _ptr(residual),
                                   int(epilogue), _ptr(out), _ptr(workspace), ws_len, _stream(), tune)
        _check(st, "sbi_gemm_i8_ln")
        return out
    st = load().sbi_gemm_i8(_ptr(Wl), _ptr(sw), K, N, _ptr(X), B, _ptr(bias), _ptr(residual), int(epilogue),
                            _ptr(out), _ptr(workspace), ws_len, _stream(), tune)
    _check(st, "sbi_gemm_i8")
    return out


def gemm(Wl, K, N, X, bias=None, residual=None, epilogue=EPI_NONE, out=None, workspace=None,
         path=PATH_AUTO, split_k=0, waves=0, depth=0, blocks=0, panels=0, layernorm=None, moments_in=None,
         moments_out=None):
    """Y = epilogue(X @ W + bias) through sbi_gemm / sbi_gemm_ex, or, with
    layernorm=(gamma, beta, eps), Y = epilogue(LN(X) @ W + bias) through sbi_gemm_ln.
    moments_out (float32 [B, ceil(N/64), 2]) receives the per-panel row moments of Y
    (sbi_gemm_moments); moments_in passes such moments of X to the layer-norm.
    Returns Y (fp16 [B,N])."""
    import torch
    assert X.is_cuda and X.dtype == torch.float16 and X.dim() == 2 and X.is_contiguous()
    B = X.shape[0]
    if isinstance(epilogue, str):
        epilogue = EPILOGUES[epilogue]
    if out is None:
        out = torch.empty((B, N), dtype=torch.float16, device=X.device)
    _need(X, (B, K), "X")
    _need(bias, (N,), "bias")
    _need(residual, (B, N), "residual")
    _need(out, (B, N), "out")
    _need_bytes(Wl, layout_bytes(K, N), "laid-out weights")
    if layernorm is not None:
        _need(layernorm[0], (K,), "gamma")
        _need(layernorm[1], (K,), "beta")
    tune = _tuning(path, split_k, waves, depth, blocks, panels)
    if workspace is None:
        if tune or layernorm is not None:
            need = plan(B, K, N, path, split_k, waves, depth, blocks, panels,
                        layernorm is not None)["workspace_bytes"]
        else:
            need = workspace_bytes(B, K, N)
        workspace = new_workspace(need, X.device) if need else None
    if workspace is not None:
        _need_bytes(workspace, 0, "workspace")
    ws_ptr = _ptr(workspace)
    ws_len = workspace.numel() * workspace.element_size() if workspace is not None else 0
    if moments_in is not None:
        if layernorm is None:
            raise ValueError("moments_in belongs to a layer-norm")
        if not (moments_in.is_cuda and moments_in.dtype == torch.float32 and moments_in.is_contiguous()
                and tuple(moments_in.shape) == (B, -(-K // 64), 2)):
            raise ValueError("moments_in: expected contiguous CUDA float32 [B, ceil(K/64), 2]")
    if moments_out is not None:
        if not (moments_out.is_cuda and moments_out.dtype == torch.float32 and moments_out.is_contiguous()
                and tuple(moments_out.shape) == (B, -(-N // 64), 2)):
            raise ValueError("moments_out: expected contiguous CUDA float32 [B, ceil(N/64), 2]")
    if layernorm is not None or moments_out is not None:
        ln = None
        if layernorm is not None:
            gamma, beta, eps = layernorm
            ln = LayerNorm(gamma.data_ptr(), beta.data_ptr(), float(eps),
                           moments_in.data_ptr() if moments_in is not None else None)
        lnp = ctypes.byref(ln) if ln is not None else None
        if moments_out is not None:
            st = load().sbi_gemm_moments(_ptr(Wl), K, N, _ptr(X), B, lnp, _ptr(bias), _ptr(residual),
                                         int(epilogue), _ptr(out), _ptr(moments_out), ws_ptr, ws_len, _stream(), tune)
            _check(st, "sbi_gemm_moments")
        else:
            st = load().sbi_gemm_ln(_ptr(Wl), K, N, _ptr(X), B, lnp, _ptr(bias), _ptr(residual),
                                    int(epilogue), _ptr(out), ws_ptr, ws_len, _stream(), tune)
            _check(st, "sbi_gemm_ln")
        return out
    if tune is None:
        st = load().sbi_gemm(_ptr(Wl), K, N, _ptr(X), B, _ptr(bias), _ptr(residual), int(epilogue),
                             _ptr(out), ws_ptr, ws_len, _stream())
    else:
        st = load().sbi_gemm_ex(_ptr(Wl), K, N, _ptr(X), B, _ptr(bias), _ptr(residual), int(epilogue),
                                _ptr(out), ws_ptr, ws_len, _stream(), tune)
    _check(st, "sbi_gemm")
    return out


STATIC_SCRATCH_BYTES = 16 << 20


def gemm_static(Wl, K, N, X, bias=None, residual=None, epilogue=EPI_NONE, out=None):
    """sbi_gemm_static: sbi_gemm with the workspace in the library's own device array.  `out` is
    allocated here only if the caller passes none; the library call itself allocates nothing."""
    import torch
    assert X.is_cuda and X.dtype == torch.float16 and X.dim() == 2 and X.is_contiguous()
    B = X.shape[0]
    if isinstance(epilogue, str):
        epilogue = EPILOGUES[epilogue]
    if out is None:
        out = torch.empty((B, N), dtype=torch.float16, device=X.device)
    _need(X, (B, K), "X")
    _need(bias, (N,), "bias")
    _need(residual, (B, N), "residual")
    _need(out, (B, N), "out")
    _need_bytes(Wl, layout_bytes(K, N), "laid-out weights")
    st = load().sbi_gemm_static(_ptr(Wl), K, N, _ptr(X), B, _ptr(bias), _ptr(residual), int(epilogue),
                                _ptr(out), _stream())
    _check(st, "sbi_gemm_static")
    return out


def make_layer(Wqkv, Wout, Wffn1, Wffn2, h, n_qkv, k_out, n_ffn1, k_ffn2,
               bqkv=None, bout=None, bffn1=None, bffn2=None, ffn1_gelu=True, ln1=None, ln2=None, ln_eps=1e-5,
               scales=None):
    """Fill an sbi_layer from laid-out weight tensors; keep the tensors alive yourself.
    scales = (sqkv, sout, sffn1, sffn2) float32 tensors makes it an INT8 layer (int8 laid-out weights)."""
    import torch
    for w, (K, N), name in ((Wqkv, (h, n_qkv), "Wqkv"), (Wout, (k_out, h), "Wout"),
                            (Wffn1, (h, n_ffn1), "Wffn1"), (Wffn2, (k_ffn2, h), "Wffn2")):
        _need_bytes(w, (i8_layout_bytes if scales is not None else layout_bytes)(K, N), name)
    if scales is not None:
        for sc, N in zip(scales, (n_qkv, h, n_ffn1, h)):
            if not (sc.is_cuda and sc.dtype == torch.float32 and sc.is_contiguous() and tuple(sc.shape) == (N,)):
                raise ValueError("scales: expected contiguous CUDA float32 tensors of shape (N,)")
    for b, N, name in ((bqkv, n_qkv, "bqkv"), (bout, h, "bout"), (bffn1, n_ffn1, "bffn1"), (bffn2, h, "bffn2")):
        _need(b, (N,), name)
    for ln, name in ((ln1, "ln1"), (ln2, "ln2")):
        if ln is not None:
            _need(ln[0], (h,), name + " gamma")
            _need(ln[1], (h,), name + " beta")
    L = Layer()
    L.Wqkv, L.Wout, L.Wffn1, L.Wffn2 = (w.data_ptr() for w in (Wqkv, Wout, Wffn1, Wffn2))
    L.bqkv, L.bout, L.bffn1, L.bffn2 = (None if b is None else b.data_ptr() for b in (bqkv, bout, bffn1, bffn2))
    L.h, L.n_qkv, L.k_out, L.n_ffn1, L.k_ffn2 = h, n_qkv, k_out, n_ffn1, k_ffn2
    L.ffn1_gelu = 1 if ffn1_gelu else 0
    if ln1 is not None:                       # (gamma, beta) tensors, fp16 [h]
        L.ln1_gamma, L.ln1_beta = ln1[0].data_ptr(), ln1[1].data_ptr()
    if ln2 is not None:
        L.ln2_gamma, L.ln2_beta = ln2[0].data_ptr(), ln2[1].data_ptr()
    L.ln_eps = float(ln_eps)
    if scales is not None:
        L.sqkv, L.sout, L.sffn1, L.sffn2 = (sc.data_ptr() for sc in scales)
    return L


def layer_workspace_bytes(layer, B):
    return int(load().sbi_layer_workspace_bytes(ctypes.byref(layer), B))


def layer_plan(layer, B, chained=False):
    """Per-GeMM plans of the grouped launch sbi_layer_gemms would make, and its total grid."""
    plans = (Plan * 4)()
    grid = ctypes.c_int32(0)
    _check(load().sbi_layer_plan(ctypes.byref(layer), B, 1 if chained else 0, plans, ctypes.byref(grid)),
           "sbi_layer_plan")
    return [p.as_dict() for p in plans][: 3 if chained else 4], grid.value


def layer_gemms(layer, B, Xqkv, Xout, Xffn1, Xffn2, residual, Yqkv, Yout, Yffn1, Yffn2, workspace):
    for t, cols, name in ((Xqkv, layer.h, "Xqkv"), (Xout, layer.k_out, "Xout"), (Xffn1, layer.h, "Xffn1"),
                          (Xffn2, layer.k_ffn2, "Xffn2"), (residual, layer.h, "residual"),
                          (Yqkv, layer.n_qkv, "Yqkv"), (Yout, layer.h, "Yout"), (Yffn1, layer.n_ffn1, "Yffn1"),
                          (Yffn2, layer.h, "Yffn2")):
        _need(t, (B, cols), name)
    ws_len = workspace.numel() * workspace.element_size() if workspace is not None else 0
    st = load().sbi_layer_gemms(ctypes.byref(layer), B, _ptr(Xqkv), _ptr(Xout), _ptr(Xffn1), _ptr(Xffn2),
                                _ptr(residual), _ptr(Yqkv), _ptr(Yout), _ptr(Yffn1), _ptr(Yffn2),
                                _ptr(workspace), ws_len, _stream())
    _check(st, "sbi_layer_gemms")


class TuneReport(ctypes.Structure):
    _fields_ = [("candidates", ctypes.c_int32), ("waves", ctypes.c_int32), ("depth", ctypes.c_int32),
                ("panels", ctypes.c_int32), ("block_ksteps", ctypes.c_int32), ("us_best", ctypes.c_float),
                ("us_model", ctypes.c_float)]

    def as_dict(self):
        return {k: getattr(self, k) for k, _ in self._fields_}


def layer_tune(layers, B, Xqkv, Xout, Xffn1, Xffn2, residual, Yqkv, Yout, Yffn1, Yffn2, workspace):
    """sbi_layer_tune over the weight sets `layers` (Layer structs of one shape): measures the
    candidate plans of the layer launch and makes the fastest the plan of later calls.  Returns the
    report as a dict."""
    layer = layers[0]
    for t, cols, name in ((Xqkv, layer.h, "Xqkv"), (Xout, layer.k_out, "Xout"), (Xffn1, layer.h, "Xffn1"),
                          (Xffn2, layer.k_ffn2, "Xffn2"), (residual, layer.h, "residual"),
                          (Yqkv, layer.n_qkv, "Yqkv"), (Yout, layer.h, "Yout"), (Yffn1, layer.n_ffn1, "Yffn1"),
                          (Yffn2, layer.h, "Yffn2")):
        _need(t, (B, cols), name)
    arr = (Layer * len(layers))(*layers)
    rep = TuneReport()
    ws_len = workspace.numel() * workspace.element_size() if workspace is not None else 0
    st = load().sbi_layer_tune(arr, len(layers), B, _ptr(Xqkv), _ptr(Xout), _ptr(Xffn1), _ptr(Xffn2), _ptr(residual),
                               _ptr(Yqkv), _ptr(Yout), _ptr(Yffn1), _ptr(Yffn2), _ptr(workspace), ws_len, _stream(),
                               ctypes.byref(rep))
    _check(st, "sbi_layer_tune")
    return rep.as_dict()


FLAVOURS = {"fp16": 0, "fp16_ln": 1, "int8": 2, "int8_codes": 3}


def kernel_registers(B, waves, depth, panels=1, flavour="fp16"):
    """(allocated, assumed) vector registers per lane of one GeMM kernel variant, or None if the
    library has no such variant."""
    a, m = ctypes.c_int32(0), ctypes.c_int32(0)
    st = load().sbi_kernel_registers(int(B), int(waves), int(depth), int(panels), FLAVOURS[flavour],
                                     ctypes.byref(a), ctypes.byref(m))
    if st == 10:                      # SBI_ERR_TUNING: no such variant
        return None
    _check(st, "sbi_kernel_registers")
    return a.value, m.value


def gemm_tune(Wls, K, N, X, bias=None, residual=None, epilogue=EPI_NONE, out=None, workspace=None):
    """sbi_gemm_tune over the laid-out weight copies `Wls` (one shape).  Returns the report as a dict."""
    import torch
    B = X.shape[0]
    if isinstance(epilogue, str):
        epilogue = EPILOGUES[epilogue]
    if out is None:
        out = torch.empty((B, N), dtype=torch.float16, device=X.device)
    _need(X, (B, K), "X")
    _need(bias, (N,), "bias")
    _need(residual, (B, N), "residual")
    _need(out, (B, N), "out")
    for w in Wls:
        _need_bytes(w, layout_bytes(K, N), "laid-out weights")
    ptrs = (ctypes.c_void_p * len(Wls))(*[w.data_ptr() for w in Wls])
    rep = TuneReport()
    ws_len = workspace.numel() * workspace.element_size() if workspace is not None else 0
    st = load().sbi_gemm_tune(ptrs, len(Wls), K, N, _ptr(X), B, _ptr(bias), _ptr(residual), int(epilogue), _ptr(out),
                              _ptr(workspace), ws_len, _stream(), ctypes.byref(rep))
    _check(st, "sbi_gemm_tune")
    return rep.as_dict()


def attn_workspace_bytes(B, heads, head_dim, max_seq):
    return int(load().sbi_attn_decode_workspace_bytes(B, heads, head_dim, max_seq))


def attn_decode(qkv, k_cache, v_cache, pos, scale=0.0, out=None, workspace=None):
    """Single-token attention with a KV cache (sbi_attn_decode).  qkv fp16 [B,3,H,d]; caches fp16
    [B,H,S,d], updated in place at position pos.  Returns out fp16 [B, H*d]."""
    import torch
    B, three, H, d = qkv.shape
    S = k_cache.shape[2]
    _need(qkv, (B, 3, H, d), "qkv")
    _need(k_cache, (B, H, S, d), "k_cache")
    _need(v_cache, (B, H, S, d), "v_cache")
    if out is None:
        out = torch.empty((B, H * d), dtype=torch.float16, device=qkv.device)
    _need(out, (B, H * d), "out")
    need = attn_workspace_bytes(B, H, d, S)
    if workspace is None and need:
        workspace = new_workspace(need, qkv.device)
    if need:
        _need_bytes(workspace, need, "workspace")
    ws_len = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(load().sbi_attn_decode(_ptr(qkv), _ptr(k_cache), _ptr(v_cache), B, H, d, S, int(pos), float(scale),
                                  _ptr(out), _ptr(workspace), ws_len, _stream()), "sbi_attn_decode")
    return out


def attn_decode_ragged(qkv, k_cache, v_cache, pos, pos_bound, scale=0.0, out=None, workspace=None):
    """sbi_attn_decode_ragged: as attn_decode, with one position per sequence (pos: int32 device
    tensor [B]) and the host-side bound pos_bound >= every entry."""
    import torch
    B, three, H, d = qkv.shape
    S = k_cache.shape[2]
    _need(qkv, (B, 3, H, d), "qkv")
    _need(k_cache, (B, H, S, d), "k_cache")
    _need(v_cache, (B, H, S, d), "v_cache")
    if pos.dtype != torch.int32 or tuple(pos.shape) != (B,) or not pos.is_contiguous() or pos.device != qkv.device:
        raise ValueError("pos: expected a contiguous int32 tensor [B] on the inputs' device")
    if out is None:
        out = torch.empty((B, H * d), dtype=torch.float16, device=qkv.device)
    _need(out, (B, H * d), "out")
    need = attn_workspace_bytes(B, H, d, S)
    if workspace is None and need:
        workspace = new_workspace(need, qkv.device)
    if need:
        _need_bytes(workspace, need, "workspace")
    ws_len = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(load().sbi_attn_decode_ragged(_ptr(qkv), _ptr(k_cache), _ptr(v_cache), B, H, d, S, _ptr(pos),
                                         int(pos_bound), float(scale), _ptr(out), _ptr(workspace), ws_len, _stream()),
           "sbi_attn_decode_ragged")
    return out


# ---------------------------------------------------------------------------------- measurement helpers
def calib_read(src, sink, blocks, waves=8, depth=4, nontemporal=True):
    """Stream the whole uint8 tensor `src` (numel a multiple of 4096) with the GeMM's access shape."""
    _check(load().sbi_calib_read(_ptr(src), src.numel(), _ptr(sink), sink.numel() * sink.element_size(),
                                 int(blocks), int(waves), int(depth), 1 if nontemporal else 0, _stream()),
           "sbi_calib_read")


def calib_copy(src, dst):
    _check(load().sbi_calib_copy(_ptr(src), _ptr(dst), src.numel() * src.element_size(), _stream()),
           "sbi_calib_copy")
