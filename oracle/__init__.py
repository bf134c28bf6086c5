"""CPU oracle for the DGQ A8W4 linear layer (test infrastructure, not the product).

Thin numpy/ctypes front end over ``dgq_oracle.c``.  Only the tests, the smoke
check and the benchmark's ``cpu_baseline`` leg may import this package; it
imports nothing from the HIP path.

Each function cites the passage of the paper (arXiv 2310.04836) it follows.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dgq_oracle.c")
_LIB = os.path.join(_HERE, "libdgq_oracle.so")


def build(force: bool = False) -> str:
    """Compile dgq_oracle.c with gcc (-O2, OpenMP, no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-fno-fast-math",
             "-ffp-contract=off", "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _L():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.dgq_oracle_expand.restype = ctypes.c_long
        _lib.dgq_oracle_gemm_i32.restype = ctypes.c_long
        _lib.dgq_oracle_pack.restype = ctypes.c_long
        _lib.dgq_oracle_threads.restype = ctypes.c_int
        _lib.dgq_oracle_bmm_s8.restype = ctypes.c_long
        _lib.dgq_oracle_expand_zp.restype = ctypes.c_long
        _lib.dgq_oracle_pack_zp.restype = ctypes.c_long
        _lib.dgq_oracle_quant_act_static.argtypes = [ctypes.c_void_p, ctypes.c_long, ctypes.c_float, ctypes.c_void_p]
        _lib.dgq_oracle_smooth_scales.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_float, ctypes.c_void_p]
        _lib.dgq_oracle_rmsnorm.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_float, ctypes.c_void_p]
        _lib.dgq_oracle_quantize_grid_act.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int,
                                                      ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                                      ctypes.c_float, ctypes.c_void_p, ctypes.c_void_p,
                                                      ctypes.c_void_p, ctypes.c_void_p]
        _lib.dgq_oracle_quantize_grid.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                                  ctypes.c_int, ctypes.c_float, ctypes.c_void_p,
                                                  ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
    return _lib


def _p(a: np.ndarray):
    assert a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    return np.ascontiguousarray(a, dtype=dtype)


def threads() -> int:
    return int(_L().dgq_oracle_threads())


def quantize_weights_rtn(W, group: int):
    """RTN dual-grained quantizer (Table 1 "RTN"; Section 3.1 symmetric scale; Eq. 5 decoupling).

    W: fp16/fp32 [K, N].  Returns (w4 int8 [K,N], s2 uint8 [K/group,N], s1 float32 [N]).
    """
    Wf = _c(W, np.float32)
    K, N = Wf.shape
    assert K % group == 0
    w4 = np.empty((K, N), np.int8)
    s2 = np.empty((K // group, N), np.uint8)
    s1 = np.empty(N, np.float32)
    _L().dgq_oracle_quantize_rtn(_p(Wf), K, N, group, _p(w4), _p(s2), _p(s1))
    return w4, s2, s1


def quant_act(x):
    """Per-token dynamic symmetric INT8 quantizer (Section 3.1 symmetric case; Section 4.1).

    x: fp16/fp32 [M, K].  Returns (xq int8 [M,K], sx float32 [M]).
    """
    xf = _c(x, np.float32)
    M, K = xf.shape
    xq = np.empty((M, K), np.int8)
    sx = np.empty(M, np.float32)
    _L().dgq_oracle_quant_act(_p(xf), M, K, _p(xq), _p(sx))
    return xq, sx


def expand(w4, s2, group: int):
    """W_s8 = S2 * W4 (Eq. 2, second line).  Returns (ws8 int8 [K,N], n_out_of_int8)."""
    w4 = _c(w4, np.int8)
    s2 = _c(s2, np.uint8)
    K, N = w4.shape
    assert s2.shape == (K // group, N) and K % group == 0
    ws8 = np.empty((K, N), np.int8)
    bad = _L().dgq_oracle_expand(_p(w4), _p(s2), K, N, group, _p(ws8))
    return ws8, int(bad)


def gemm_i32(xq, ws8):
    """acc = Xq @ W_s8 in INT32, one reduction over all of K (Eq. 2, third line).

    Returns (acc int32 [M,N], n_outputs_that_would_wrap_int32).
    """
    xq = _c(xq, np.int8)
    ws8 = _c(ws8, np.int8)
    M, K = xq.shape
    K2, N = ws8.shape
    assert K == K2
    acc = np.empty((M, N), np.int32)
    wrapped = _L().dgq_oracle_gemm_i32(_p(xq), _p(ws8), M, N, K, _p(acc))
    return acc, int(wrapped)


def bmm_s8_acc(a, b):
    """Batched INT8 product for attention (Section 4.1 "Implementation"): acc[i] = a[i] @ b[i].T in INT32.

    a: int8 [B, M, K], b: int8 [B, N, K] (both with the reduction index last).
    Returns (acc int32 [B, M, N], n_outputs_that_would_wrap_int32)."""
    a = _c(a, np.int8)
    b = _c(b, np.int8)
    B, M, K = a.shape
    B2, N, K2 = b.shape
    assert B == B2 and K == K2
    acc = np.empty((B, M, N), np.int32)
    wrapped = _L().dgq_oracle_bmm_s8(_p(a), _p(b), B, M, N, K, _p(acc))
    return acc, int(wrapped)


def bmm_s8(a, b, sa, sb):
    """out[i][m][n] = fp16((sa[i][m] * sb[i][n]) * acc[i][m][n]): the batched product with the scale epilogue of
    Eq. 2, the second operand's per-token scale in the place of the channel scale.  Returns (out fp16, acc int32)."""
    acc, wrapped = bmm_s8_acc(a, b)
    if wrapped:
        raise OverflowError("%d INT32 accumulators would wrap" % wrapped)
    sa = _c(sa, np.float32)
    sb = _c(sb, np.float32)
    out = np.stack([epilogue(acc[i], sa[i], sb[i]) for i in range(acc.shape[0])])
    return out, acc


def epilogue(acc, sx, s1):
    """O = (s_X * s1) * acc, rounded once to fp16 (Eq. 2, first and third lines)."""
    acc = _c(acc, np.int32)
    sx = _c(sx, np.float32)
    s1 = _c(s1, np.float32)
    M, N = acc.shape
    assert sx.shape == (M,) and s1.shape == (N,)
    out32 = np.empty((M, N), np.float32)
    _L().dgq_oracle_epilogue(_p(acc), _p(sx), _p(s1), M, N, _p(out32))
    with np.errstate(over="ignore"):
        return out32.astype(np.float16)


def linear_a8w4(xq, sx, w4, s2, s1, group: int):
    """The A8W4 linear of Eq. 2 from already-quantized operands.

    Returns (out fp16 [M,N], acc int32 [M,N]).
    """
    ws8, bad = expand(w4, s2, group)
    if bad:
        raise ValueError("%d expanded weights fall outside INT8" % bad)
    acc, wrapped = gemm_i32(xq, ws8)
    if wrapped:
        raise OverflowError("%d INT32 accumulators would wrap" % wrapped)
    return epilogue(acc, sx, s1), acc


def forward(x, w4, s2, s1, group: int):
    """Whole hot path: per-token quantization of fp16 x, then linear_a8w4."""
    xq, sx = quant_act(x)
    out, acc = linear_a8w4(xq, sx, w4, s2, s1, group)
    return out, acc, xq, sx


def packed_sizes(K: int, N: int, group: int):
    ng = K // group
    return K * N // 2, (N // 16) * ((ng + 3) // 4) * 64


def pack(w4, s2, group: int):
    """Device weight format written from the layout text.  Returns (qweight u8, scales u8, n_bad)."""
    w4 = _c(w4, np.int8)
    s2 = _c(s2, np.uint8)
    K, N = w4.shape
    assert K % 128 == 0 and N % 16 == 0 and group in (64, 128)
    assert s2.shape == (K // group, N)
    qb, sb = packed_sizes(K, N, group)
    qweight = np.empty(qb, np.uint8)
    scales = np.empty(sb, np.uint8)
    bad = _L().dgq_oracle_pack(_p(w4), _p(s2), K, N, group, _p(qweight), _p(scales))
    return qweight, scales, int(bad)


def unpack(qweight, scales, K: int, N: int, group: int):
    """Inverse of pack.  Returns (w4 int8 [K,N], s2 uint8 [K/group,N])."""
    qweight = _c(qweight, np.uint8)
    scales = _c(scales, np.uint8)
    qb, sb = packed_sizes(K, N, group)
    assert qweight.size == qb and scales.size == sb
    w4 = np.empty((K, N), np.int8)
    s2 = np.empty((K // group, N), np.uint8)
    _L().dgq_oracle_unpack(_p(qweight), _p(scales), K, N, group, _p(w4), _p(s2))
    return w4, s2


# ---------------------------------------------------------------------------
# General operands: unsigned nibbles with per-group zero points (Section 3.2),
# the clip of Eq. 4 and the two-phase grid search of Section 3.3
# ---------------------------------------------------------------------------
def expand_zp(u4, s2, zp, group: int):
    """W_s8 = S2 * (W_u4 - ZP) (Eq. 2, second line; sign as in Eq. 1 / Appendix B).

    Returns (ws8 int8 [K,N], n_out_of_int8)."""
    u4 = _c(u4, np.uint8)
    s2 = _c(s2, np.uint8)
    zp = _c(zp, np.uint8)
    K, N = u4.shape
    assert K % group == 0 and s2.shape == (K // group, N) and zp.shape == s2.shape
    ws8 = np.empty((K, N), np.int8)
    bad = _L().dgq_oracle_expand_zp(_p(u4), _p(s2), _p(zp), K, N, group, _p(ws8))
    return ws8, int(bad)


def clip_interval(s2: int, zp: int):
    """Interval of stored nibbles that keeps S2 * (u - ZP) inside INT8 (Eq. 4).  Returns (lo, hi)."""
    lo, hi = ctypes.c_int(), ctypes.c_int()
    _L().dgq_oracle_clip_interval(int(s2), int(zp), ctypes.byref(lo), ctypes.byref(hi))
    return lo.value, hi.value


def quantize_weights_grid(W, group: int, n_alpha: int = 51, step: float = 0.01):
    """Two-phase grid search (Section 3.3, Eq. 3-5) with the weight-only objective.

    W: fp16/fp32 [K, N].  Returns (u4 uint8 [K,N], zp uint8 [K/group,N], s2 uint8 [K/group,N], s1 float32 [N]).
    """
    Wf = _c(W, np.float32)
    K, N = Wf.shape
    assert K % group == 0 and n_alpha >= 1
    u4 = np.empty((K, N), np.uint8)
    zp = np.empty((K // group, N), np.uint8)
    s2 = np.empty((K // group, N), np.uint8)
    s1 = np.empty(N, np.float32)
    _L().dgq_oracle_quantize_grid(_p(Wf), K, N, group, n_alpha, ctypes.c_float(step), _p(u4), _p(zp), _p(s2), _p(s1))
    return u4, zp, s2, s1


def dequant_act(x):
    """X^ of Eq. 3: the per-token INT8 quantization of x, dequantized (fp32 product sx * xq)."""
    xq, sx = quant_act(x)
    return (sx[:, None] * xq.astype(np.float32)).astype(np.float32)


def quantize_weights_grid_act(W, X, group: int, n_alpha: int = 51, step: float = 0.01, Xh=None):
    """Two-phase grid search with the activation-weighted objectives of Section 3.3 (Eq. 3; objective of Eq. 5) on
    calibration activations X [M, K]; Xh defaults to dequant_act(X).

    Returns (u4 uint8 [K,N], zp uint8 [K/group,N], s2 uint8 [K/group,N], s1 float32 [N])."""
    Wf, Xf = _c(W, np.float32), _c(X, np.float32)
    Xhf = dequant_act(X) if Xh is None else _c(Xh, np.float32)
    K, N = Wf.shape
    M = Xf.shape[0]
    assert K % group == 0 and n_alpha >= 1 and Xf.shape == (M, K) and Xhf.shape == (M, K)
    u4 = np.empty((K, N), np.uint8)
    zp = np.empty((K // group, N), np.uint8)
    s2 = np.empty((K // group, N), np.uint8)
    s1 = np.empty(N, np.float32)
    _L().dgq_oracle_quantize_grid_act(_p(Wf), _p(Xf), _p(Xhf), M, K, N, group, n_alpha, ctypes.c_float(step),
                                      _p(u4), _p(zp), _p(s2), _p(s1))
    return u4, zp, s2, s1


def packed_sizes_zp(K: int, N: int, group: int):
    ng = K // group
    return K * N // 2, (N // 16) * ((ng + 1) // 2) * 64


def pack_zp(u4, s2, zp, group: int):
    """Device format of the general operands.  Returns (qweight u8, scales_zp u8, n_bad)."""
    u4 = _c(u4, np.uint8)
    s2 = _c(s2, np.uint8)
    zp = _c(zp, np.uint8)
    K, N = u4.shape
    assert K % 128 == 0 and N % 16 == 0 and group in (64, 128)
    assert s2.shape == (K // group, N) and zp.shape == s2.shape
    qb, sb = packed_sizes_zp(K, N, group)
    qweight = np.empty(qb, np.uint8)
    scales = np.empty(sb, np.uint8)
    bad = _L().dgq_oracle_pack_zp(_p(u4), _p(s2), _p(zp), K, N, group, _p(qweight), _p(scales))
    return qweight, scales, int(bad)


def unpack_zp(qweight, scales_zp, K: int, N: int, group: int):
    """Inverse of pack_zp.  Returns (u4, s2, zp)."""
    qweight = _c(qweight, np.uint8)
    scales_zp = _c(scales_zp, np.uint8)
    qb, sb = packed_sizes_zp(K, N, group)
    assert qweight.size == qb and scales_zp.size == sb
    u4 = np.empty((K, N), np.uint8)
    s2 = np.empty((K // group, N), np.uint8)
    zp = np.empty((K // group, N), np.uint8)
    _L().dgq_oracle_unpack_zp(_p(qweight), _p(scales_zp), K, N, group, _p(u4), _p(s2), _p(zp))
    return u4, s2, zp


def linear_a8w4_zp(xq, sx, u4, s2, zp, s1, group: int):
    """Eq. 2 from quantized operands with per-group zero points.  Returns (out fp16, acc int32)."""
    ws8, bad = expand_zp(u4, s2, zp, group)
    if bad:
        raise ValueError("%d expanded weights fall outside INT8" % bad)
    acc, wrapped = gemm_i32(xq, ws8)
    if wrapped:
        raise OverflowError("%d INT32 accumulators would wrap" % wrapped)
    return epilogue(acc, sx, s1), acc


def quant_act_static(x, scale: float):
    """Static tensor-wise INT8 activation quantizer ("S" scheme of Section 4.1 / Table 5; Eq. 1, symmetric).

    x: fp16/fp32 [M, K], scale > 0.  Returns (xq int8 [M,K], sx float32 [M] filled with the scale)."""
    xf = _c(x, np.float32)
    M, K = xf.shape
    assert scale > 0
    xq = np.empty((M, K), np.int8)
    _L().dgq_oracle_quant_act_static(_p(xf), M * K, ctypes.c_float(scale), _p(xq))
    return xq, np.full(M, np.float32(scale), np.float32)


def smooth_scales(X, pct: float = 0.005):
    """Percentile clipping smoothing scale k [K] (Section 3.4, Eq. 6) from calibration activations X [M, K]."""
    Xf = _c(X, np.float32)
    M, K = Xf.shape
    k = np.empty(K, np.float32)
    _L().dgq_oracle_smooth_scales(_p(Xf), M, K, ctypes.c_float(pct), _p(k))
    return k


def smooth_apply(W, X, k):
    """Moves the scale from activations to weights: returns (fp16(diag(k) W), fp16(X / k)) (Section 3.4)."""
    Wf, Xf, kf = _c(W, np.float32), _c(X, np.float32), _c(k, np.float32)
    K, N = Wf.shape
    M = Xf.shape[0]
    assert Xf.shape[1] == K and kf.shape == (K,)
    Wo, Xo = np.empty_like(Wf), np.empty_like(Xf)
    _L().dgq_oracle_smooth_apply(_p(Wf), _p(Xf), _p(kf), M, K, N, _p(Wo), _p(Xo))
    with np.errstate(over="ignore"):
        return Wo.astype(np.float16), Xo.astype(np.float16)


def silu_mul(GU):
    """h = fp16(float(silu(gate) * up)) of a gated MLP (gate columns first, then up), silu and product in fp64.

    GU: fp16/fp32 [M, 2*I].  Returns h float16 [M, I]."""
    G = _c(GU, np.float32)
    M, I2 = G.shape
    assert I2 % 2 == 0
    h = np.empty((M, I2 // 2), np.float32)
    _L().dgq_oracle_silu_mul(_p(G), M, I2 // 2, _p(h))
    h16 = h.astype(np.float16)
    assert np.array_equal(h16.astype(np.float32), h) or not np.isfinite(h).all()   # already fp16 values
    return h16


def silu_mul_quant_act(GU):
    """The fused producer + per-token quantizer.  Returns (xq int8 [M,I], sx float32 [M], h float16 [M,I])."""
    h = silu_mul(GU)
    xq, sx = quant_act(h)
    return xq, sx, h


def rmsnorm(x, gamma, eps: float):
    """y = fp16(float(x / sqrt(mean x^2 + eps) * gamma)), evaluated in fp64.  Returns float16 [M, K]."""
    xf, gf = _c(x, np.float32), _c(gamma, np.float32)
    M, K = xf.shape
    assert gf.shape == (K,)
    y = np.empty((M, K), np.float32)
    _L().dgq_oracle_rmsnorm(_p(xf), _p(gf), M, K, ctypes.c_float(eps), _p(y))
    return y.astype(np.float16)


def rmsnorm_quant_act(x, gamma, eps: float):
    """RMSNorm fused with the per-token quantizer.  Returns (xq int8, sx float32, y float16)."""
    y = rmsnorm(x, gamma, eps)
    xq, sx = quant_act(y)
    return xq, sx, y
