"""MI355X-native DGQ A8W4 linear layer (arXiv 2310.04836, Eq. 2): thin Python binding.

Every function here only marshals arguments for the C ABI declared in ``include/dgq.h``;
all arithmetic runs in the HIP kernels of ``libdgq.so``.  PyTorch is used for device
memory and the current stream, nothing else.  There is no CPU fallback: if the shared
library cannot be loaded the import of this package raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

from . import build as _build

__all__ = [
    "DGQError", "lib", "layout_version", "packed_sizes", "linear_workspace_bytes", "pack_weights",
    "unpack_weights", "quantize_weights_rtn", "quant_act", "linear_a8w4", "linear_a8w4_acc",
    "linear_acc_workspace_bytes", "linear_a8w4_noalloc", "bmm_s8", "bmm_s8_acc", "linear_plan", "probe_read", "probe_mfma", "packed_sizes_zp", "pack_weights_zp", "quantize_weights_grid", "quantize_weights_grid_act", "quant_act_static", "smooth_scales", "smooth_apply", "silu_mul_quant_act", "rmsnorm_quant_act", "PackedWeight", "STREAM_MAX_M",
]

STREAM_MAX_M = 64


class DGQError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib.dgq_status_string(status).decode()
        if status == -6:
            msg += " [hipError %d]" % lib.dgq_last_hip_error()
        super().__init__("%s: %s (status %d)" % (where, msg, status))


def _load() -> ctypes.CDLL:
    if not _build.is_built():
        _build.build()
    L = ctypes.CDLL(_build.LIB)
    vp, i, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    psz = ctypes.POINTER(ctypes.c_size_t)
    L.dgq_status_string.restype = ctypes.c_char_p
    L.dgq_status_string.argtypes = [i]
    L.dgq_last_hip_error.restype = i
    L.dgq_layout_version.restype = i
    L.dgq_packed_sizes.argtypes = [i, i, i, psz, psz]
    L.dgq_linear_workspace_bytes.argtypes = [i, i, i, i, psz]
    L.dgq_linear_acc_workspace_bytes.argtypes = [i, i, i, i, i, psz]
    L.dgq_linear_acc_workspace_bytes.restype = i
    L.dgq_pack_weights.argtypes = [vp, vp, i, i, i, vp, vp, vp, vp]
    L.dgq_unpack_weights.argtypes = [vp, vp, i, i, i, vp, vp]
    L.dgq_quantize_weights_rtn.argtypes = [vp, i, i, i, vp, vp, vp, vp]
    L.dgq_quant_act.argtypes = [vp, i, i, vp, vp, vp]
    L.dgq_quant_act_static.argtypes = [vp, i, i, ctypes.c_float, vp, vp, vp]
    L.dgq_silu_mul_quant_act.argtypes = [vp, i, i, vp, vp, vp]
    L.dgq_rmsnorm_quant_act.argtypes = [vp, vp, i, i, ctypes.c_float, vp, vp, vp]
    L.dgq_smooth_scales.argtypes = [vp, i, i, ctypes.c_float, vp, vp, sz, vp]
    L.dgq_smooth_apply.argtypes = [vp, vp, vp, i, i, i, vp, vp, vp]
    L.dgq_linear_a8w4.argtypes = [vp, vp, vp, vp, vp, vp, i, i, i, i, vp, sz, vp]
    L.dgq_linear_a8w4_noalloc.argtypes = [vp, vp, vp, vp, vp, vp, i, i, i, i, vp]
    L.dgq_linear_a8w4_noalloc.restype = i
    L.dgq_linear_a8w4_acc.argtypes = [vp, vp, vp, vp, i, i, i, i, i, vp, sz, vp]
    L.dgq_quantize_weights_grid.argtypes = [vp, i, i, i, i, ctypes.c_float, vp, vp, vp, vp, vp, sz, vp]
    L.dgq_quantize_weights_grid_act.argtypes = [vp, vp, vp, vp, i, i, i, i, i, ctypes.c_float, vp, vp, vp, vp, vp, sz, vp]
    L.dgq_quantize_weights_grid_act.restype = i
    L.dgq_quantize_weights_grid_act_workspace_bytes.argtypes = [i, i, i, i, psz]
    L.dgq_quantize_weights_grid_act_workspace_bytes.restype = i
    L.dgq_packed_sizes_zp.argtypes = [i, i, i, psz, psz]
    L.dgq_pack_weights_zp.argtypes = [vp, vp, vp, i, i, i, vp, vp, vp, vp]
    L.dgq_unpack_weights_zp.argtypes = [vp, vp, i, i, i, vp, vp]
    L.dgq_linear_a8w4_zp.argtypes = [vp, vp, vp, vp, vp, vp, i, i, i, i, vp, sz, vp]
    L.dgq_linear_a8w4_zp_acc.argtypes = [vp, vp, vp, vp, i, i, i, i, i, vp, sz, vp]
    L.dgq_bmm_s8.argtypes = [vp, vp, vp, vp, vp, i, i, i, i, vp]
    L.dgq_bmm_s8.restype = i
    L.dgq_bmm_s8_acc.argtypes = [vp, vp, vp, i, i, i, i, vp]
    L.dgq_bmm_s8_acc.restype = i
    L.dgq_probe_read.argtypes = [vp, sz, vp, i, vp]
    L.dgq_probe_mfma.argtypes = [vp, sz, i, vp, i, vp]
    L.dgq_linear_plan.argtypes = [i, i, i, i, ctypes.c_char_p, sz]
    L.dgq_quant_linear_plan.argtypes = [i, i, i, i, ctypes.c_char_p, sz]
    L.dgq_quant_linear_workspace_bytes.argtypes = [i, i, i, i, psz]
    L.dgq_rmsnorm_quant_linear_workspace_bytes.argtypes = [i, i, i, i, psz]
    L.dgq_quant_linear_a8w4.argtypes = [vp, vp, vp, vp, vp, vp, i, i, i, i, vp, sz, vp]
    L.dgq_quant_linear_a8w4_zp.argtypes = [vp, vp, vp, vp, vp, vp, i, i, i, i, vp, sz, vp]
    L.dgq_rmsnorm_quant_linear_a8w4.argtypes = [vp, vp, ctypes.c_float, vp, vp, vp, vp, vp, i, i, i, i, vp, sz, vp]
    L.dgq_rmsnorm_quant_linear_a8w4_zp.argtypes = [vp, vp, ctypes.c_float, vp, vp, vp, vp, vp, i, i, i, i, vp, sz, vp]
    for name in ("dgq_quant_linear_plan", "dgq_quant_linear_workspace_bytes", "dgq_quant_linear_a8w4",
                 "dgq_quant_linear_a8w4_zp", "dgq_rmsnorm_quant_linear_a8w4", "dgq_rmsnorm_quant_linear_a8w4_zp",
                 "dgq_rmsnorm_quant_linear_workspace_bytes"):
        getattr(L, name).restype = i
    for name in ("dgq_packed_sizes", "dgq_linear_workspace_bytes", "dgq_pack_weights", "dgq_unpack_weights",
                 "dgq_quantize_weights_rtn", "dgq_quant_act", "dgq_linear_a8w4", "dgq_linear_a8w4_acc",
                 "dgq_probe_read", "dgq_probe_mfma", "dgq_linear_plan", "dgq_packed_sizes_zp", "dgq_pack_weights_zp",
                 "dgq_unpack_weights_zp", "dgq_linear_a8w4_zp", "dgq_linear_a8w4_zp_acc", "dgq_quantize_weights_grid", "dgq_quant_act_static", "dgq_smooth_scales", "dgq_smooth_apply", "dgq_silu_mul_quant_act", "dgq_rmsnorm_quant_act"):
        getattr(L, name).restype = i
    return L


lib = _load()


def _check(st: int, where: str) -> None:
    if st != 0:
        raise DGQError(st, where)


def _ptr(t):
    return None if t is None else t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


def _dev(t: torch.Tensor, dtype, name: str) -> torch.Tensor:
    if not (t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise TypeError("%s must be a contiguous CUDA tensor of %s" % (name, dtype))
    return t


def layout_version() -> int:
    return lib.dgq_layout_version()


def packed_sizes(K: int, N: int, group: int):
    q, s = ctypes.c_size_t(), ctypes.c_size_t()
    _check(lib.dgq_packed_sizes(K, N, group, ctypes.byref(q), ctypes.byref(s)), "dgq_packed_sizes")
    return q.value, s.value


def linear_workspace_bytes(M: int, N: int, K: int, group: int) -> int:
    b = ctypes.c_size_t()
    _check(lib.dgq_linear_workspace_bytes(M, N, K, group, ctypes.byref(b)), "dgq_linear_workspace_bytes")
    return b.value


class PackedWeight:
    """Device buffers of one packed layer: qweight, scales (both uint8), s1 (float32 [N]).

    zp_form False: signed nibbles, `scales` holds S2 bytes (dgq_pack_weights).  True: unsigned nibbles
    with per-group zero points, `scales` holds (S2, ZP) byte pairs (dgq_pack_weights_zp)."""

    def __init__(self, qweight, scales, s1, K, N, group, zp_form=False):
        self.qweight, self.scales, self.s1 = qweight, scales, s1
        self.K, self.N, self.group = K, N, group
        self.zp_form = zp_form
        self.layout = layout_version()

    @property
    def nbytes(self) -> int:
        return self.qweight.numel() + self.scales.numel() + 4 * self.s1.numel()


def pack_weights(w4: torch.Tensor, s2: torch.Tensor, s1: torch.Tensor, group: int, return_bad: bool = False):
    """dgq_pack_weights: w4 int8 [K,N], s2 uint8 [K/group,N], s1 float32 [N] -> PackedWeight."""
    _dev(w4, torch.int8, "w4"); _dev(s2, torch.uint8, "s2"); _dev(s1, torch.float32, "s1")
    K, N = w4.shape
    if tuple(s2.shape) != (K // group, N) or tuple(s1.shape) != (N,):
        raise ValueError("s2/s1 shapes do not match w4 and group")
    qb, sb = packed_sizes(K, N, group)
    qweight = torch.empty(qb, dtype=torch.uint8, device=w4.device)
    scales = torch.empty(sb, dtype=torch.uint8, device=w4.device)
    bad = torch.zeros(1, dtype=torch.int32, device=w4.device)
    _check(lib.dgq_pack_weights(_ptr(w4), _ptr(s2), K, N, group, _ptr(qweight), _ptr(scales), _ptr(bad),
                                _stream()), "dgq_pack_weights")
    pw = PackedWeight(qweight, scales, s1, K, N, group)
    if return_bad:
        return pw, int(bad.item())
    return pw


def packed_sizes_zp(K: int, N: int, group: int):
    q, s = ctypes.c_size_t(), ctypes.c_size_t()
    _check(lib.dgq_packed_sizes_zp(K, N, group, ctypes.byref(q), ctypes.byref(s)), "dgq_packed_sizes_zp")
    return q.value, s.value


def pack_weights_zp(u4: torch.Tensor, s2: torch.Tensor, zp: torch.Tensor, s1: torch.Tensor, group: int,
                    return_bad: bool = False):
    """dgq_pack_weights_zp: u4 uint8 [K,N], s2 and zp uint8 [K/group,N], s1 float32 [N] -> PackedWeight."""
    _dev(u4, torch.uint8, "u4"); _dev(s2, torch.uint8, "s2"); _dev(zp, torch.uint8, "zp"); _dev(s1, torch.float32, "s1")
    K, N = u4.shape
    if tuple(s2.shape) != (K // group, N) or tuple(zp.shape) != tuple(s2.shape) or tuple(s1.shape) != (N,):
        raise ValueError("s2/zp/s1 shapes do not match u4 and group")
    qb, sb = packed_sizes_zp(K, N, group)
    qweight = torch.empty(qb, dtype=torch.uint8, device=u4.device)
    scales = torch.empty(sb, dtype=torch.uint8, device=u4.device)
    bad = torch.zeros(1, dtype=torch.int32, device=u4.device)
    _check(lib.dgq_pack_weights_zp(_ptr(u4), _ptr(s2), _ptr(zp), K, N, group, _ptr(qweight), _ptr(scales),
                                   _ptr(bad), _stream()), "dgq_pack_weights_zp")
    pw = PackedWeight(qweight, scales, s1, K, N, group, zp_form=True)
    if return_bad:
        return pw, int(bad.item())
    return pw


def unpack_weights(pw: PackedWeight) -> torch.Tensor:
    """dgq_unpack_weights / dgq_unpack_weights_zp: W_s8 int8 [K,N]."""
    out = torch.empty((pw.K, pw.N), dtype=torch.int8, device=pw.qweight.device)
    fn = lib.dgq_unpack_weights_zp if pw.zp_form else lib.dgq_unpack_weights
    _check(fn(_ptr(pw.qweight), _ptr(pw.scales), pw.K, pw.N, pw.group, _ptr(out), _stream()), "dgq_unpack_weights")
    return out


def quantize_weights_rtn(W: torch.Tensor, group: int):
    """dgq_quantize_weights_rtn: fp16 [K,N] -> (w4 int8 [K,N], s2 uint8 [K/group,N], s1 float32 [N])."""
    _dev(W, torch.float16, "W")
    K, N = W.shape
    w4 = torch.empty((K, N), dtype=torch.int8, device=W.device)
    s2 = torch.empty((K // group if group else 0, N), dtype=torch.uint8, device=W.device)
    s1 = torch.empty(N, dtype=torch.float32, device=W.device)
    _check(lib.dgq_quantize_weights_rtn(_ptr(W), K, N, group, _ptr(w4), _ptr(s2), _ptr(s1), _stream()),
           "dgq_quantize_weights_rtn")
    return w4, s2, s1


def quantize_weights_grid(W: torch.Tensor, group: int, n_alpha: int = 51, step: float = 0.01):
    """dgq_quantize_weights_grid: fp16 [K,N] -> (u4 uint8 [K,N], zp uint8 [K/group,N], s2 uint8 [K/group,N],
    s1 float32 [N]) by the two-phase grid search of Section 3.3."""
    _dev(W, torch.float16, "W")
    K, N = W.shape
    u4 = torch.empty((K, N), dtype=torch.uint8, device=W.device)
    zp = torch.empty((K // group, N), dtype=torch.uint8, device=W.device)
    s2 = torch.empty((K // group, N), dtype=torch.uint8, device=W.device)
    s1 = torch.empty(N, dtype=torch.float32, device=W.device)
    ws = torch.empty((K // group) * N, dtype=torch.float32, device=W.device)
    _check(lib.dgq_quantize_weights_grid(_ptr(W), K, N, group, n_alpha, step, _ptr(u4), _ptr(zp), _ptr(s2), _ptr(s1),
                                         _ptr(ws), ws.numel() * 4, _stream()), "dgq_quantize_weights_grid")
    return u4, zp, s2, s1


def quantize_weights_grid_act(W: torch.Tensor, X: torch.Tensor, group: int, n_alpha: int = 51, step: float = 0.01):
    """dgq_quantize_weights_grid_act: the two-phase grid search with the activation-weighted objectives of Section 3.3
    on calibration activations X fp16 [M,K] (quantized here with dgq_quant_act).  Returns (u4, zp, s2, s1)."""
    _dev(W, torch.float16, "W"); _dev(X, torch.float16, "X")
    K, N = W.shape
    M = X.shape[0]
    if X.shape[1] != K:
        raise ValueError("X has K=%d but W has K=%d" % (X.shape[1], K))
    xq, sx = quant_act(X)
    u4 = torch.empty((K, N), dtype=torch.uint8, device=W.device)
    zp = torch.empty((K // group, N), dtype=torch.uint8, device=W.device)
    s2 = torch.empty((K // group, N), dtype=torch.uint8, device=W.device)
    s1 = torch.empty(N, dtype=torch.float32, device=W.device)
    nb = ctypes.c_size_t()
    _check(lib.dgq_quantize_weights_grid_act_workspace_bytes(M, K, N, group, ctypes.byref(nb)),
           "dgq_quantize_weights_grid_act_workspace_bytes")
    ws = torch.empty(nb.value, dtype=torch.uint8, device=W.device)
    _check(lib.dgq_quantize_weights_grid_act(_ptr(W), _ptr(X), _ptr(xq), _ptr(sx), M, K, N, group, n_alpha, step,
                                             _ptr(u4), _ptr(zp), _ptr(s2), _ptr(s1), _ptr(ws), nb.value, _stream()),
           "dgq_quantize_weights_grid_act")
    return u4, zp, s2, s1


def quant_act(x: torch.Tensor, xq: torch.Tensor = None, sx: torch.Tensor = None):
    """dgq_quant_act: fp16 [M,K] -> (xq int8 [M,K], sx float32 [M])."""
    _dev(x, torch.float16, "x")
    M, K = x.shape
    if xq is None:
        xq = torch.empty((M, K), dtype=torch.int8, device=x.device)
    if sx is None:
        sx = torch.empty(M, dtype=torch.float32, device=x.device)
    _check(lib.dgq_quant_act(_ptr(x), M, K, _ptr(xq), _ptr(sx), _stream()), "dgq_quant_act")
    return xq, sx


def _workspace(M, N, K, group, device):
    """Zero-filled scratch of the size the library asks for (None when it needs none)."""
    nbytes = linear_workspace_bytes(M, N, K, group)
    return torch.zeros(nbytes, dtype=torch.uint8, device=device) if nbytes else None


def smooth_scales(X: torch.Tensor, pct: float = 0.005) -> torch.Tensor:
    """dgq_smooth_scales: calibration activations fp16 [M,K] -> smoothing scale k float32 [K] (Eq. 6)."""
    _dev(X, torch.float16, "X")
    M, K = X.shape
    k = torch.empty(K, dtype=torch.float32, device=X.device)
    ws = torch.empty(K, dtype=torch.float32, device=X.device)
    _check(lib.dgq_smooth_scales(_ptr(X), M, K, pct, _ptr(k), _ptr(ws), K * 4, _stream()), "dgq_smooth_scales")
    return k


def smooth_apply(W: torch.Tensor, X: torch.Tensor, k: torch.Tensor):
    """dgq_smooth_apply: (fp16(diag(k) W), fp16(X / k)); either input may be None."""
    _dev(k, torch.float32, "k")
    K = k.numel()
    Wout = Xout = None
    M = N = 0
    if W is not None:
        _dev(W, torch.float16, "W"); N = W.shape[1]; Wout = torch.empty_like(W)
    if X is not None:
        _dev(X, torch.float16, "X"); M = X.shape[0]; Xout = torch.empty_like(X)
    _check(lib.dgq_smooth_apply(_ptr(W), _ptr(X), _ptr(k), M, K, N, _ptr(Wout), _ptr(Xout), _stream()), "dgq_smooth_apply")
    return Wout, Xout


def silu_mul_quant_act(gate_up: torch.Tensor, xq: torch.Tensor = None, sx: torch.Tensor = None):
    """dgq_silu_mul_quant_act: fp16 [M, 2I] (gate | up) -> per-token quantized silu(gate)*up: (xq int8 [M,I], sx [M])."""
    _dev(gate_up, torch.float16, "gate_up")
    M, I2 = gate_up.shape
    if xq is None:
        xq = torch.empty((M, I2 // 2), dtype=torch.int8, device=gate_up.device)
    if sx is None:
        sx = torch.empty(M, dtype=torch.float32, device=gate_up.device)
    _check(lib.dgq_silu_mul_quant_act(_ptr(gate_up), M, I2 // 2, _ptr(xq), _ptr(sx), _stream()), "dgq_silu_mul_quant_act")
    return xq, sx


def rmsnorm_quant_act(x: torch.Tensor, gamma: torch.Tensor, eps: float, xq: torch.Tensor = None, sx: torch.Tensor = None):
    """dgq_rmsnorm_quant_act: per-token quantized RMSNorm(x) * gamma: (xq int8 [M,K], sx float32 [M])."""
    _dev(x, torch.float16, "x"); _dev(gamma, torch.float16, "gamma")
    M, K = x.shape
    if xq is None:
        xq = torch.empty((M, K), dtype=torch.int8, device=x.device)
    if sx is None:
        sx = torch.empty(M, dtype=torch.float32, device=x.device)
    _check(lib.dgq_rmsnorm_quant_act(_ptr(x), _ptr(gamma), M, K, eps, _ptr(xq), _ptr(sx), _stream()), "dgq_rmsnorm_quant_act")
    return xq, sx


def quant_act_static(x: torch.Tensor, scale: float, xq: torch.Tensor = None, sx: torch.Tensor = None):
    """dgq_quant_act_static: fp16 [M,K] and one scale -> (xq int8 [M,K], sx float32 [M] = scale)."""
    _dev(x, torch.float16, "x")
    M, K = x.shape
    if xq is None:
        xq = torch.empty((M, K), dtype=torch.int8, device=x.device)
    if sx is None:
        sx = torch.empty(M, dtype=torch.float32, device=x.device)
    _check(lib.dgq_quant_act_static(_ptr(x), M, K, scale, _ptr(xq), _ptr(sx), _stream()), "dgq_quant_act_static")
    return xq, sx


def linear_a8w4(xq: torch.Tensor, sx: torch.Tensor, pw: PackedWeight, out: torch.Tensor = None,
                workspace: torch.Tensor = None) -> torch.Tensor:
    """dgq_linear_a8w4: fp16 [M,N] = (sx x s1) * (xq @ expand(qweight))."""
    _dev(xq, torch.int8, "xq"); _dev(sx, torch.float32, "sx")
    M, K = xq.shape
    if K != pw.K:
        raise ValueError("xq has K=%d but the packed weight has K=%d" % (K, pw.K))
    if out is None:
        out = torch.empty((M, pw.N), dtype=torch.float16, device=xq.device)
    if workspace is None:
        workspace = _workspace(M, pw.N, K, pw.group, xq.device)
    wsb = 0 if workspace is None else workspace.numel() * workspace.element_size()
    fn = lib.dgq_linear_a8w4_zp if pw.zp_form else lib.dgq_linear_a8w4
    _check(fn(_ptr(xq), _ptr(sx), _ptr(pw.qweight), _ptr(pw.scales), _ptr(pw.s1), _ptr(out),
              M, pw.N, K, pw.group, _ptr(workspace), wsb, _stream()), "dgq_linear_a8w4")
    return out


def linear_a8w4_noalloc(xq: torch.Tensor, sx: torch.Tensor, pw: PackedWeight, out: torch.Tensor) -> torch.Tensor:
    """dgq_linear_a8w4_noalloc: dgq_linear_a8w4 with the library's static scratch; `out` must exist (nothing is
    allocated here either).  Signed-nibble form only."""
    _dev(xq, torch.int8, "xq"); _dev(sx, torch.float32, "sx"); _dev(out, torch.float16, "out")
    M, K = xq.shape
    if K != pw.K or tuple(out.shape) != (M, pw.N) or pw.zp_form:
        raise ValueError("shapes or weight form do not match")
    _check(lib.dgq_linear_a8w4_noalloc(_ptr(xq), _ptr(sx), _ptr(pw.qweight), _ptr(pw.scales), _ptr(pw.s1), _ptr(out),
                                       M, pw.N, K, pw.group, _stream()), "dgq_linear_a8w4_noalloc")
    return out


def quant_linear_workspace_bytes(M: int, N: int, K: int, group: int) -> int:
    """dgq_quant_linear_workspace_bytes."""
    n = ctypes.c_size_t(0)
    _check(lib.dgq_quant_linear_workspace_bytes(M, N, K, group, ctypes.byref(n)), "dgq_quant_linear_workspace_bytes")
    return n.value


def quant_linear_a8w4(x: torch.Tensor, pw: PackedWeight, out: torch.Tensor = None, sx_out: torch.Tensor = None,
                      workspace: torch.Tensor = None) -> torch.Tensor:
    """dgq_quant_linear_a8w4: fp16 [M,N] = linear_a8w4(quant_act(x)) as one call (one kernel for small M)."""
    _dev(x, torch.float16, "x")
    if sx_out is not None:
        _dev(sx_out, torch.float32, "sx_out")
    M, K = x.shape
    if K != pw.K:
        raise ValueError("x has K=%d but the packed weight has K=%d" % (K, pw.K))
    if sx_out is not None and sx_out.numel() != M:
        raise ValueError("sx_out must hold M floats")
    if out is None:
        out = torch.empty((M, pw.N), dtype=torch.float16, device=x.device)
    if workspace is None:
        nbytes = quant_linear_workspace_bytes(M, pw.N, K, pw.group)
        workspace = torch.zeros(nbytes, dtype=torch.uint8, device=x.device) if nbytes else None
    wsb = 0 if workspace is None else workspace.numel() * workspace.element_size()
    fn = lib.dgq_quant_linear_a8w4_zp if pw.zp_form else lib.dgq_quant_linear_a8w4
    _check(fn(_ptr(x), _ptr(pw.qweight), _ptr(pw.scales), _ptr(pw.s1), _ptr(out), _ptr(sx_out),
              M, pw.N, K, pw.group, _ptr(workspace), wsb, _stream()), "dgq_quant_linear_a8w4")
    return out


def rmsnorm_quant_linear_workspace_bytes(M: int, N: int, K: int, group: int) -> int:
    """dgq_rmsnorm_quant_linear_workspace_bytes."""
    n = ctypes.c_size_t(0)
    _check(lib.dgq_rmsnorm_quant_linear_workspace_bytes(M, N, K, group, ctypes.byref(n)),
           "dgq_rmsnorm_quant_linear_workspace_bytes")
    return n.value


def rmsnorm_quant_linear_a8w4(x: torch.Tensor, gamma: torch.Tensor, eps: float, pw: PackedWeight,
                              out: torch.Tensor = None, sx_out: torch.Tensor = None,
                              workspace: torch.Tensor = None) -> torch.Tensor:
    """dgq_rmsnorm_quant_linear_a8w4: fp16 [M,N] = linear_a8w4(quant_act(rmsnorm(x) * gamma)) as one call."""
    _dev(x, torch.float16, "x"); _dev(gamma, torch.float16, "gamma")
    if sx_out is not None:
        _dev(sx_out, torch.float32, "sx_out")
    M, K = x.shape
    if K != pw.K or gamma.numel() != K:
        raise ValueError("x has K=%d, gamma %d elements, the packed weight K=%d" % (K, gamma.numel(), pw.K))
    if sx_out is not None and sx_out.numel() != M:
        raise ValueError("sx_out must hold M floats")
    if out is None:
        out = torch.empty((M, pw.N), dtype=torch.float16, device=x.device)
    if workspace is None:
        nbytes = rmsnorm_quant_linear_workspace_bytes(M, pw.N, K, pw.group)
        workspace = torch.zeros(nbytes, dtype=torch.uint8, device=x.device) if nbytes else None
    wsb = 0 if workspace is None else workspace.numel() * workspace.element_size()
    fn = lib.dgq_rmsnorm_quant_linear_a8w4_zp if pw.zp_form else lib.dgq_rmsnorm_quant_linear_a8w4
    _check(fn(_ptr(x), _ptr(gamma), eps, _ptr(pw.qweight), _ptr(pw.scales), _ptr(pw.s1), _ptr(out), _ptr(sx_out),
              M, pw.N, K, pw.group, _ptr(workspace), wsb, _stream()), "dgq_rmsnorm_quant_linear_a8w4")
    return out


def bmm_s8(a: torch.Tensor, b: torch.Tensor, sa: torch.Tensor = None, sb: torch.Tensor = None,
           out: torch.Tensor = None) -> torch.Tensor:
    """dgq_bmm_s8: fp16 [B,M,N] = (sa x sb) * (a @ b^T) per batch; a int8 [B,M,K], b int8 [B,N,K], scales float32."""
    _dev(a, torch.int8, "a"); _dev(b, torch.int8, "b")
    B, M, K = a.shape
    B2, N, K2 = b.shape
    if B != B2 or K != K2:
        raise ValueError("a is %s but b is %s" % (tuple(a.shape), tuple(b.shape)))
    for t, n, name in ((sa, M, "sa"), (sb, N, "sb")):
        if t is not None:
            _dev(t, torch.float32, name)
            if tuple(t.shape) != (B, n):
                raise ValueError("%s must be [batch, %d]" % (name, n))
    if out is None:
        out = torch.empty((B, M, N), dtype=torch.float16, device=a.device)
    _check(lib.dgq_bmm_s8(_ptr(a), _ptr(b), _ptr(sa), _ptr(sb), _ptr(out), B, M, N, K, _stream()), "dgq_bmm_s8")
    return out


def bmm_s8_acc(a: torch.Tensor, b: torch.Tensor) -> torch.Tensor:
    """dgq_bmm_s8_acc: raw INT32 sums [B,M,N] of the same kernel (test hook)."""
    _dev(a, torch.int8, "a"); _dev(b, torch.int8, "b")
    B, M, K = a.shape
    B2, N, K2 = b.shape
    if B != B2 or K != K2:
        raise ValueError("a is %s but b is %s" % (tuple(a.shape), tuple(b.shape)))
    acc = torch.empty((B, M, N), dtype=torch.int32, device=a.device)
    _check(lib.dgq_bmm_s8_acc(_ptr(a), _ptr(b), _ptr(acc), B, M, N, K, _stream()), "dgq_bmm_s8_acc")
    return acc


def quant_linear_plan(M: int, N: int, K: int, group: int) -> str:
    """dgq_quant_linear_plan: name of the GEMM kernel dgq_quant_linear_a8w4 would launch."""
    buf = ctypes.create_string_buffer(128)
    _check(lib.dgq_quant_linear_plan(M, N, K, group, buf, 128), "dgq_quant_linear_plan")
    return buf.value.decode()


def linear_plan(M: int, N: int, K: int, group: int) -> str:
    """dgq_linear_plan: name of the GEMM kernel dgq_linear_a8w4 would launch for this problem."""
    buf = ctypes.create_string_buffer(128)
    _check(lib.dgq_linear_plan(M, N, K, group, buf, 128), "dgq_linear_plan")
    return buf.value.decode()


def probe_read(buf: torch.Tensor, sink: torch.Tensor, workgroups: int = 256, nbytes: int = None) -> None:
    """dgq_probe_read: stream `nbytes` (default: all) of `buf` once; measurement aid."""
    n = buf.numel() * buf.element_size() if nbytes is None else nbytes
    _check(lib.dgq_probe_read(_ptr(buf), n, _ptr(sink), workgroups, _stream()), "dgq_probe_read")


def probe_mfma(operands: torch.Tensor, iters: int, sink: torch.Tensor, workgroups: int = 512) -> int:
    """dgq_probe_mfma: MFMA-only loop on operands from `operands`; returns the integer operations issued."""
    n = operands.numel() * operands.element_size()
    _check(lib.dgq_probe_mfma(_ptr(operands), n, iters, _ptr(sink), workgroups, _stream()), "dgq_probe_mfma")
    return 2 * 32 * 32 * 32 * 8 * iters * 4 * workgroups


def linear_acc_workspace_bytes(M: int, N: int, K: int, group: int, path: int = 0) -> int:
    """dgq_linear_acc_workspace_bytes."""
    b = ctypes.c_size_t()
    _check(lib.dgq_linear_acc_workspace_bytes(M, N, K, group, path, ctypes.byref(b)), "dgq_linear_acc_workspace_bytes")
    return b.value


def linear_a8w4_acc(xq: torch.Tensor, pw: PackedWeight, workspace: torch.Tensor = None, path: int = 0) -> torch.Tensor:
    """dgq_linear_a8w4_acc: raw INT32 sums [M,N] of the same kernels (test hook).  path: 0 = the kernel
    dgq_linear_a8w4 chooses, 1 = weight-streaming kernels, 2 = tiled kernel, 3 = the streaming kernel that
    re-reads activations every step."""
    _dev(xq, torch.int8, "xq")
    M, K = xq.shape
    if K != pw.K:
        raise ValueError("xq has K=%d but the packed weight has K=%d" % (K, pw.K))
    acc = torch.empty((M, pw.N), dtype=torch.int32, device=xq.device)
    if workspace is None:
        nbytes = linear_acc_workspace_bytes(M, pw.N, K, pw.group, path)
        workspace = torch.zeros(nbytes, dtype=torch.uint8, device=xq.device) if nbytes else None
    wsb = 0 if workspace is None else workspace.numel() * workspace.element_size()
    fn = lib.dgq_linear_a8w4_zp_acc if pw.zp_form else lib.dgq_linear_a8w4_acc
    _check(fn(_ptr(xq), _ptr(pw.qweight), _ptr(pw.scales), _ptr(acc), M, pw.N, K, pw.group, path,
              _ptr(workspace), wsb, _stream()), "dgq_linear_a8w4_acc")
    return acc
