"""Python face of the CPU oracle (TEST INFRASTRUCTURE ONLY).

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this
module.  It loads oracle/libsbi_oracle.so (plain C, fp64) and adds two numpy-only pieces:

* layout_weights / unlayout_weights - the weight pre-layout written as a reshape/transpose
  from the layout's published definition (the paper, Sec. III-C "Leveraging Full
  Cache-line", only fixes the idea: re-tile W once at initialisation so that each thread
  reads several consecutive input-dimension elements of a column in one access);
* ulp16 / check_close - the acceptance rule |gpu - oracle| <= max(2 ulp16(oracle), 1e-3).

Nothing here imports the GPU package; inputs are numpy arrays of fp16 (or their uint16 bits).
"""
import ctypes
import os

import numpy as np

from . import build as _build

EPI_BIAS = 1
EPI_GELU = 2
EPI_RES = 4

# layout constants, restated here from the layout's definition (not imported from the GPU side)
CHUNK_K = 8      # consecutive k of one column held by one lane (16 bytes)
TILE_N = 16      # columns per tile
TILE_K = 32      # k per tile  = 4 lane groups x CHUNK_K
PANEL_TILES = 4  # tiles per panel -> a panel is 64 columns wide
PANEL_N = TILE_N * PANEL_TILES
STEP_GROUP = 8   # k-steps per panel are padded to a multiple of this
HEADER_BYTES = 256

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.build()
        L = ctypes.CDLL(path)
        L.sbi_oracle_half_to_double.restype = ctypes.c_double
        L.sbi_oracle_half_to_double.argtypes = [ctypes.c_uint16]
        L.sbi_oracle_double_to_half.restype = ctypes.c_uint16
        L.sbi_oracle_double_to_half.argtypes = [ctypes.c_double]
        L.sbi_oracle_gelu.restype = ctypes.c_double
        L.sbi_oracle_gelu.argtypes = [ctypes.c_double]
        L.sbi_oracle_half_to_double_array.restype = None
        L.sbi_oracle_half_to_double_array.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64]
        L.sbi_oracle_double_to_half_array.restype = None
        L.sbi_oracle_double_to_half_array.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64]
        L.sbi_oracle_layernorm.restype = ctypes.c_int
        L.sbi_oracle_layernorm.argtypes = [ctypes.c_void_p] * 3 + [ctypes.c_double, ctypes.c_int64, ctypes.c_int64,
                                           ctypes.c_void_p, ctypes.c_void_p]
        vp, i64 = ctypes.c_void_p, ctypes.c_int64
        L.sbi_oracle_quantize_rows.restype = ctypes.c_int
        L.sbi_oracle_quantize_rows.argtypes = [vp, i64, i64, vp, vp]
        L.sbi_oracle_quantize_columns.restype = ctypes.c_int
        L.sbi_oracle_quantize_columns.argtypes = [vp, i64, i64, vp, vp]
        L.sbi_oracle_gemm_i8.restype = ctypes.c_int
        L.sbi_oracle_gemm_i8.argtypes = [vp] * 6 + [ctypes.c_int, i64, i64, i64, vp, vp]
        L.sbi_oracle_attn_decode.restype = ctypes.c_int
        L.sbi_oracle_attn_decode.argtypes = [vp, vp, vp, i64, i64, i64, i64, i64, ctypes.c_double, vp, vp]
        L.sbi_oracle_max_threads.restype = ctypes.c_int
        L.sbi_oracle_gemm.restype = ctypes.c_int
        L.sbi_oracle_gemm.argtypes = [ctypes.c_void_p] * 4 + [ctypes.c_int] + [ctypes.c_int64] * 3 + \
            [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int]
        _lib = L
    return _lib


def _bits(a, name):
    """fp16 array (or uint16 bit patterns) -> contiguous uint16 view."""
    a = np.asarray(a)
    if a.dtype == np.float16:
        a = a.view(np.uint16)
    if a.dtype != np.uint16:
        raise TypeError(f"{name}: expected float16 or uint16, got {a.dtype}")
    return np.ascontiguousarray(a)


def half_to_double(bits):
    b = _bits(bits, "bits")
    out = np.empty(b.shape, dtype=np.float64)
    lib().sbi_oracle_half_to_double_array(b.ctypes.data, out.ctypes.data, b.size)
    return out


def double_to_half(values):
    """fp64 array -> fp16 array, one round-to-nearest-even step (the oracle's own rounding)."""
    v = np.ascontiguousarray(np.asarray(values, dtype=np.float64))
    out = np.empty(v.shape, dtype=np.uint16)
    lib().sbi_oracle_double_to_half_array(v.ctypes.data, out.ctypes.data, v.size)
    return out.view(np.float16)


def gelu(v):
    return lib().sbi_oracle_gelu(float(v))


def max_threads():
    return int(lib().sbi_oracle_max_threads())


def gemm(X, W, bias=None, residual=None, epi=0, threads=0, return_pre=False):
    """Y = epilogue(X @ W + bias) per the oracle definition.  X [B,K], W [K,N] fp16.

    epi is a bit set of EPI_BIAS | EPI_GELU | EPI_RES.  Returns fp16 [B,N]
    (and the fp64 values before the final rounding when return_pre is set).
    """
    Xb, Wb = _bits(X, "X"), _bits(W, "W")
    if Xb.ndim != 2 or Wb.ndim != 2 or Xb.shape[1] != Wb.shape[0]:
        raise ValueError(f"shape mismatch X{Xb.shape} W{Wb.shape}")
    B, K = Xb.shape
    N = Wb.shape[1]
    bb = rb = None
    if epi & EPI_BIAS:
        bb = _bits(bias, "bias")
        if bb.shape != (N,):
            raise ValueError("bias shape")
    if epi & EPI_RES:
        rb = _bits(residual, "residual")
        if rb.shape != (B, N):
            raise ValueError("residual shape")
    Y = np.empty((B, N), dtype=np.uint16)
    pre = np.empty((B, N), dtype=np.float64) if return_pre else None
    rc = lib().sbi_oracle_gemm(Xb.ctypes.data, Wb.ctypes.data,
                               bb.ctypes.data if bb is not None else None,
                               rb.ctypes.data if rb is not None else None,
                               int(epi), B, K, N, Y.ctypes.data,
                               pre.ctypes.data if pre is not None else None, int(threads))
    if rc != 0:
        raise RuntimeError(f"sbi_oracle_gemm failed rc={rc}")
    Yh = Y.view(np.float16)
    return (Yh, pre) if return_pre else Yh


def layernorm(X, gamma, beta, eps, return_pre=False):
    """Row-wise layer normalisation of X [B,K] in fp64, rounded once to fp16 (it is the fp16
    operand of the GeMM that follows).  eps is taken at fp32 precision, as the C ABI passes it."""
    Xb, gb, bb = _bits(X, "X"), _bits(gamma, "gamma"), _bits(beta, "beta")
    if Xb.ndim != 2 or gb.shape != (Xb.shape[1],) or bb.shape != (Xb.shape[1],):
        raise ValueError("layernorm shapes")
    B, K = Xb.shape
    out = np.empty((B, K), dtype=np.uint16)
    pre = np.empty((B, K), dtype=np.float64) if return_pre else None
    rc = lib().sbi_oracle_layernorm(Xb.ctypes.data, gb.ctypes.data, bb.ctypes.data, float(np.float32(eps)),
                                    B, K, out.ctypes.data, pre.ctypes.data if pre is not None else None)
    if rc != 0:
        raise RuntimeError(f"sbi_oracle_layernorm failed rc={rc}")
    return (out.view(np.float16), pre) if return_pre else out.view(np.float16)


# --------------------------------------------------------------------------------------
# INT8 path: symmetric quantisation (binary32 decisions, see sbi_oracle.c) and the exact-integer GeMM.
# --------------------------------------------------------------------------------------
def quantize_rows(X):
    """X [B,K] fp16 -> (Xq int8 [B,K], sx float32 [B]): one scale per row (per token)."""
    Xb = _bits(X, "X")
    if Xb.ndim != 2:
        raise ValueError("quantize_rows wants [B,K]")
    B, K = Xb.shape
    q = np.empty((B, K), dtype=np.int8)
    s = np.empty(B, dtype=np.float32)
    if lib().sbi_oracle_quantize_rows(Xb.ctypes.data, B, K, q.ctypes.data, s.ctypes.data) != 0:
        raise RuntimeError("sbi_oracle_quantize_rows failed")
    return q, s


def quantize_columns(W):
    """W [K,N] fp16 -> (Wq int8 [K,N], sw float32 [N]): one scale per column (per output channel)."""
    Wb = _bits(W, "W")
    if Wb.ndim != 2:
        raise ValueError("quantize_columns wants [K,N]")
    K, N = Wb.shape
    q = np.empty((K, N), dtype=np.int8)
    s = np.empty(N, dtype=np.float32)
    if lib().sbi_oracle_quantize_columns(Wb.ctypes.data, K, N, q.ctypes.data, s.ctypes.data) != 0:
        raise RuntimeError("sbi_oracle_quantize_columns failed")
    return q, s


def gemm_i8(Xq, sx, Wq, sw, bias=None, residual=None, epi=0, return_pre=False):
    """Y = epilogue((Xq @ Wq) * sx[:,None] * sw[None,:] + bias): exact integer product, fp64 epilogue,
    one rounding to fp16.  Xq [B,K], Wq [K,N] int8; sx [B], sw [N] float32."""
    Xq = np.ascontiguousarray(Xq, dtype=np.int8)
    Wq = np.ascontiguousarray(Wq, dtype=np.int8)
    sx = np.ascontiguousarray(sx, dtype=np.float32)
    sw = np.ascontiguousarray(sw, dtype=np.float32)
    if Xq.ndim != 2 or Wq.ndim != 2 or Xq.shape[1] != Wq.shape[0] or sx.shape != (Xq.shape[0],) or \
            sw.shape != (Wq.shape[1],):
        raise ValueError("gemm_i8 shapes")
    B, K = Xq.shape
    N = Wq.shape[1]
    bb = rb = None
    if epi & EPI_BIAS:
        bb = _bits(bias, "bias")
        if bb.shape != (N,):
            raise ValueError("bias shape")
    if epi & EPI_RES:
        rb = _bits(residual, "residual")
        if rb.shape != (B, N):
            raise ValueError("residual shape")
    Y = np.empty((B, N), dtype=np.uint16)
    pre = np.empty((B, N), dtype=np.float64) if return_pre else None
    rc = lib().sbi_oracle_gemm_i8(Xq.ctypes.data, sx.ctypes.data, Wq.ctypes.data, sw.ctypes.data,
                                  bb.ctypes.data if bb is not None else None,
                                  rb.ctypes.data if rb is not None else None, int(epi), B, K, N,
                                  Y.ctypes.data, pre.ctypes.data if pre is not None else None)
    if rc != 0:
        raise RuntimeError(f"sbi_oracle_gemm_i8 failed rc={rc}")
    Yh = Y.view(np.float16)
    return (Yh, pre) if return_pre else Yh


def gemm_i8_from_fp16(X, Wq, sw, bias=None, residual=None, epi=0):
    """The whole INT8 path on fp16 activations: quantise the rows of X, then gemm_i8."""
    Xq, sx = quantize_rows(X)
    return gemm_i8(Xq, sx, Wq, sw, bias, residual, epi)


def gemm_i8_ln_from_fp16(X, gamma, beta, eps, Wq, sw, bias=None, residual=None, epi=0):
    """Layer-norm in front of the INT8 GeMM (the paper's fused regions start with the layer-norm
    whatever the GeMM's data type, Sec. III-D): the composition of the definitions above and
    nothing else - layernorm() in fp64 rounded once to fp16 (the GeMM's operand), those fp16
    values quantised per row by quantize_rows() (binary32 decisions), then gemm_i8()."""
    return gemm_i8_from_fp16(layernorm(X, gamma, beta, eps), Wq, sw, bias, residual, epi)


def attn_decode(qkv, Kc, Vc, pos, scale=None, return_pre=False):
    """Single-token attention with a KV cache.  qkv [B,3,H,d] fp16 (query, new key, new value of
    the token), Kc / Vc [B,H,S,d] fp16 caches with `pos` tokens in them.  Returns
    (out [B,H*d] fp16, Kc', Vc') where the caches now also hold the new token at position pos
    (the inputs are not modified); scale defaults to 1/sqrt(d)."""
    q = np.ascontiguousarray(_bits(qkv, "qkv"))
    K = np.array(_bits(Kc, "Kc"), copy=True)
    V = np.array(_bits(Vc, "Vc"), copy=True)
    if q.ndim != 4 or q.shape[1] != 3 or K.ndim != 4 or K.shape != V.shape or \
            K.shape[:2] != (q.shape[0], q.shape[2]) or K.shape[3] != q.shape[3]:
        raise ValueError("attn_decode shapes")
    B, _, H, d = q.shape
    S = K.shape[2]
    if scale is None:
        scale = 1.0 / np.sqrt(float(d))
    out = np.empty((B, H * d), dtype=np.uint16)
    pre = np.empty((B, H * d), dtype=np.float64) if return_pre else None
    rc = lib().sbi_oracle_attn_decode(q.ctypes.data, K.ctypes.data, V.ctypes.data, B, H, d, S, int(pos),
                                      float(scale), out.ctypes.data, pre.ctypes.data if pre is not None else None)
    if rc != 0:
        raise RuntimeError(f"sbi_oracle_attn_decode failed rc={rc}")
    res = (out.view(np.float16), K.view(np.float16), V.view(np.float16))
    return res + (pre,) if return_pre else res


I8_TILE_K = 64          # k per k-step of the int8 layout
I8_CHUNK_K = 16         # consecutive k one lane owns (16 bytes)


def layout_dims_i8(K, N):
    KS = -(-(-(-K // I8_TILE_K)) // STEP_GROUP) * STEP_GROUP
    return KS, -(-N // PANEL_N)


def layout_weights_i8(Wq):
    """Wq [K,N] int8 -> flat int8 array of P*KS*4*64*16 bytes (no header): the fp16 layout's
    structure with 64-k steps, lane (g, i) owning k = 16g..16g+15 of column i."""
    Wq = np.ascontiguousarray(Wq, dtype=np.int8)
    K, N = Wq.shape
    KS, P = layout_dims_i8(K, N)
    Wp = np.zeros((KS * I8_TILE_K, P * PANEL_N), dtype=np.int8)
    Wp[:K, :N] = Wq
    T = Wp.reshape(KS, 4, I8_CHUNK_K, P, PANEL_TILES, TILE_N)          # ks, g, e, p, t, i
    return np.ascontiguousarray(T.transpose(3, 0, 4, 1, 5, 2)).reshape(-1)   # p, ks, t, g, i, e


# --------------------------------------------------------------------------------------
# Weight pre-layout, from its definition.  W [K,N] is zero-padded to Kp = ceil256(K)
# (KS = Kp // 32 k-steps, a multiple of 8), Np = ceil64(N).  Element (k, n) lands at half-index
#     ((((p*KS + ks)*4 + t)*64 + lane)*8 + e)
# with p = n // 64, t = (n % 64) // 16, i = n % 16, ks = k // 32, g = (k % 32) // 8,
# e = k % 8, lane = g*16 + i, KS = Kp // 32 -- i.e. one lane of a 64-wide wavefront owns
# 8 consecutive k of one column (16 bytes), a wavefront load covers a 16-column x 32-k tile
# (1 KiB) and four such tiles (64 columns) of the same k range are adjacent.
# --------------------------------------------------------------------------------------
def layout_dims(K, N):
    KS = -(-(-(-K // TILE_K)) // STEP_GROUP) * STEP_GROUP
    P = -(-N // PANEL_N)
    return KS, P


def layout_weights(W):
    """W [K,N] fp16 -> flat uint16 array of P*KS*4*64*8 halfs (no header)."""
    Wb = _bits(W, "W")
    K, N = Wb.shape
    KS, P = layout_dims(K, N)
    Wp = np.zeros((KS * TILE_K, P * PANEL_N), dtype=np.uint16)
    Wp[:K, :N] = Wb
    # axes: ks, g, e, p, t, i
    T = Wp.reshape(KS, 4, CHUNK_K, P, PANEL_TILES, TILE_N)
    # target order: p, ks, t, g, i, e
    return np.ascontiguousarray(T.transpose(3, 0, 4, 1, 5, 2)).reshape(-1)


def unlayout_weights(flat, K, N):
    """Inverse of layout_weights: flat halfs -> W [K,N] uint16 bits (padding dropped)."""
    KS, P = layout_dims(K, N)
    T = np.asarray(flat, dtype=np.uint16).reshape(P, KS, PANEL_TILES, 4, TILE_N, CHUNK_K)
    Wp = T.transpose(1, 3, 5, 0, 2, 4).reshape(KS * TILE_K, P * PANEL_N)
    return np.ascontiguousarray(Wp[:K, :N])


# --------------------------------------------------------------------------------------
# Acceptance rule.
# --------------------------------------------------------------------------------------
def ulp16(v):
    """Spacing of fp16 numbers at |v| (2^-24 in the subnormal range)."""
    a = np.abs(np.asarray(v, dtype=np.float64))
    e = np.floor(np.log2(np.maximum(a, 2.0 ** -14)))
    return np.exp2(np.maximum(e, -14.0) - 10.0)


def check_close(got, want, ulps=2, abs_tol=1e-3):
    """Element-wise |got - want| <= max(ulps * ulp16(want), abs_tol); inf must match inf.

    Returns (ok, report dict with max abs error, max error in ulp16, number of failures).
    """
    g = np.asarray(got, dtype=np.float16).astype(np.float64)
    w = np.asarray(want, dtype=np.float16).astype(np.float64)
    if g.shape != w.shape:
        raise ValueError(f"shape mismatch {g.shape} vs {w.shape}")
    fin = np.isfinite(w)
    same_nonfinite = np.where(fin, True, (g == w) | (np.isnan(g) & np.isnan(w)))
    with np.errstate(invalid="ignore"):
        diff = np.where(fin, np.abs(g - w), 0.0)
    diff = np.where(np.isfinite(diff), diff, np.inf)
    tol = np.maximum(ulps * ulp16(np.where(fin, w, 1.0)), abs_tol)
    bad = (diff > tol) | ~same_nonfinite
    rep = {
        "max_abs": float(diff.max()) if diff.size else 0.0,
        "max_ulp": float((diff / ulp16(np.where(fin, w, 1.0))).max()) if diff.size else 0.0,
        "n_bad": int(bad.sum()),
        "n": int(bad.size),
    }
    if rep["n_bad"]:
        idx = np.argwhere(bad)[0]
        rep["first_bad"] = (tuple(int(i) for i in idx), float(g[tuple(idx)]), float(w[tuple(idx)]))
    return rep["n_bad"] == 0, rep
