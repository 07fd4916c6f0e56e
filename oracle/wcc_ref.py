"""numpy front end of the CPU oracle (oracle/wcc_ref.c).

TEST INFRASTRUCTURE ONLY.  Every function converts its arguments to contiguous
float64 / int64 arrays, calls the C routine of the same name and returns new
arrays; there is no arithmetic of the method on the Python side.
"""
from __future__ import annotations

import ctypes as C

import numpy as np

from .build import build

_lib = None

_pd = C.POINTER(C.c_double)
_pi = C.POINTER(C.c_int64)
_i64 = C.c_int64


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        L.wcc_ref_max_threads.restype = C.c_int
        L.wcc_ref_set_threads.argtypes = [C.c_int]
        L.wcc_ref_k.restype = _i64
        L.wcc_ref_k.argtypes = [_i64, _i64, _i64]
        L.wcc_ref_haar_fwd.restype = C.c_int
        L.wcc_ref_haar_fwd.argtypes = [_pd, _i64, _i64, _i64, C.c_int, _pd]
        L.wcc_ref_haar_inv.restype = C.c_int
        L.wcc_ref_haar_inv.argtypes = [_pd, _i64, _i64, _i64, C.c_int, _pd]
        L.wcc_ref_channel_norm.restype = None
        L.wcc_ref_channel_norm.argtypes = [_pd, _i64, _i64, _i64, _pd]
        L.wcc_ref_channel_norm_sq.restype = None
        L.wcc_ref_channel_norm_sq.argtypes = [_pd, _i64, _i64, _i64, _pd]
        L.wcc_ref_topk.restype = C.c_int
        L.wcc_ref_topk.argtypes = [_pd, _i64, _i64, _i64, _pi]
        L.wcc_ref_gather.restype = None
        L.wcc_ref_gather.argtypes = [_pd, _pi, _i64, _i64, _i64, _i64, _pd]
        L.wcc_ref_scatter.restype = None
        L.wcc_ref_scatter.argtypes = [_pd, _pi, _i64, _i64, _i64, _i64, _pd]
        L.wcc_ref_absmax.restype = C.c_double
        L.wcc_ref_absmax.argtypes = [_pd, _i64]
        L.wcc_ref_quant_codes.restype = None
        L.wcc_ref_quant_codes.argtypes = [_pd, _i64, C.c_double, C.c_int, _pd]
        L.wcc_ref_pointwise.restype = None
        L.wcc_ref_pointwise.argtypes = [_pd, _pd, _pd, _i64, _i64, _i64, _i64, _pd]
        L.wcc_ref_forward.restype = C.c_int
        L.wcc_ref_forward.argtypes = [_pd, _pd, _pd, _i64, _i64, _i64, _i64, _i64, C.c_int,
                                      _i64, _i64, C.c_int, C.c_double, _pd, _pi, _pd]
        L.wcc_ref_conv_mac.restype = _i64
        L.wcc_ref_depthwise3x3.argtypes = [_pd, _pd, _i64, _i64, _i64, _i64, _pd]
        L.wcc_ref_depthwise3x3.restype = C.c_int
        L.wcc_ref_conv_mac.argtypes = [_i64] * 8
        L.wcc_ref_conv_bops.restype = _i64
        L.wcc_ref_conv_bops.argtypes = [_i64] * 3
        L.wcc_ref_haar_bops.restype = _i64
        L.wcc_ref_haar_bops.argtypes = [_i64, _i64, _i64, C.c_int, _i64]
        _lib = L
    return _lib


def _d(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _p(a):
    return a.ctypes.data_as(_pd)


def _q(a):
    return a.ctypes.data_as(_pi)


def max_threads() -> int:
    return int(lib().wcc_ref_max_threads())


def set_threads(n: int) -> None:
    lib().wcc_ref_set_threads(int(n))


def k_of(N: int, num: int, den: int) -> int:
    return int(lib().wcc_ref_k(N, num, den))


def haar_fwd(x, levels: int):
    """x [..., H, W] -> coefficients [..., H*W] in concatenated band order."""
    x = _d(x)
    H, W = x.shape[-2:]
    y = np.empty(x.shape[:-2] + (H * W,), dtype=np.float64)
    planes = x.size // (H * W)
    if lib().wcc_ref_haar_fwd(_p(x), planes, H, W, levels, _p(y)):
        raise ValueError("bad shape / levels")
    return y


def haar_inv(y, H: int, W: int, levels: int):
    """coefficients [..., H*W] -> planes [..., H, W]."""
    y = _d(y)
    assert y.shape[-1] == H * W
    x = np.empty(y.shape[:-1] + (H, W), dtype=np.float64)
    planes = y.size // (H * W)
    if lib().wcc_ref_haar_inv(_p(y), planes, H, W, levels, _p(x)):
        raise ValueError("bad shape / levels")
    return x


def channel_norm(coef, norm: str = "l1"):
    """coef [B, C, N] -> [B, N]: sum over channels of |coef| ("l1") or of coef^2 ("l2")."""
    coef = _d(coef)
    B, Cc, N = coef.shape
    out = np.empty((B, N), dtype=np.float64)
    fn = {"l1": lib().wcc_ref_channel_norm, "l2": lib().wcc_ref_channel_norm_sq}[norm]
    fn(_p(coef), B, Cc, N, _p(out))
    return out


def topk(norm, k: int):
    """norm [B, N] -> idx [B, k] int64, ascending."""
    norm = _d(norm)
    B, N = norm.shape
    idx = np.empty((B, k), dtype=np.int64)
    if lib().wcc_ref_topk(_p(norm), B, N, k, _q(idx)):
        raise ValueError("bad k")
    return idx


def gather(coef, idx):
    coef = _d(coef)
    idx = np.ascontiguousarray(idx, dtype=np.int64)
    B, Cc, N = coef.shape
    k = idx.shape[1]
    out = np.empty((B, Cc, k), dtype=np.float64)
    lib().wcc_ref_gather(_p(coef), _q(idx), B, Cc, N, k, _p(out))
    return out


def scatter(yc, idx, N: int):
    yc = _d(yc)
    idx = np.ascontiguousarray(idx, dtype=np.int64)
    B, Cc, k = yc.shape
    out = np.empty((B, Cc, N), dtype=np.float64)
    lib().wcc_ref_scatter(_p(yc), _q(idx), B, Cc, N, k, _p(out))
    return out


def absmax(v) -> float:
    v = _d(v)
    return float(lib().wcc_ref_absmax(_p(v), v.size))


def quant_codes(v, alpha: float, bits: int = 8):
    v = _d(v)
    out = np.empty_like(v)
    lib().wcc_ref_quant_codes(_p(v), v.size, float(alpha), bits, _p(out))
    return out


def pointwise(w, out_scale, xc):
    """w [C_out, C_in], out_scale [C_out] or None, xc [B, C_in, k] -> [B, C_out, k]."""
    w = _d(w)
    xc = _d(xc)
    B, Ci, k = xc.shape
    Co = w.shape[0]
    assert w.shape == (Co, Ci)
    sc = None if out_scale is None else _d(out_scale)
    out = np.empty((B, Co, k), dtype=np.float64)
    lib().wcc_ref_pointwise(_p(w), None if sc is None else _p(sc), _p(xc), B, Ci, Co, k, _p(out))
    return out


def forward(x, w, w_scale, levels: int, keep_num: int, keep_den: int, act_bits: int = 0,
            alpha_in: float = 0.0, norm: str = "l1"):
    """Whole layer.  Returns (y [B,C_out,H,W], idx [B,k], alpha).  norm = "l2": the positions
    are ranked by the sum of squares over channels; the steps are then taken one by one."""
    x = _d(x)
    w = _d(w)
    B, Ci, H, W = x.shape
    if norm != "l1":
        coef = haar_fwd(x, levels).reshape(B, Ci, H * W)
        idx = topk(channel_norm(coef, norm), k_of(H * W, keep_num, keep_den))
        y, alpha = forward_with_list(x, w, w_scale, levels, idx, act_bits, alpha_in)
        return y, idx, alpha
    Co = w.shape[0]
    assert w.shape == (Co, Ci)
    sc = None if w_scale is None else _d(w_scale)
    k = k_of(H * W, keep_num, keep_den)
    y = np.empty((B, Co, H, W), dtype=np.float64)
    idx = np.empty((B, max(k, 1)), dtype=np.int64)
    alpha = C.c_double(0.0)
    rc = lib().wcc_ref_forward(_p(x), _p(w), None if sc is None else _p(sc), B, Ci, Co, H, W,
                               levels, keep_num, keep_den, act_bits, float(alpha_in), _p(y),
                               _q(idx), C.byref(alpha))
    if rc:
        raise ValueError("wcc_ref_forward: bad arguments or out of memory")
    return y, idx, float(alpha.value)


def forward_with_list(x, w, w_scale, levels: int, idx, act_bits: int = 0, alpha_in: float = 0.0):
    """The layer with the index set given instead of selected (the steps of Alg. 1 after the
    shrinkage's top-k; footnote of the section "Joint hard shrinkage").  idx [B, k] ascending.
    Returns (y [B,C_out,H,W], alpha)."""
    x = _d(x)
    w = _d(w)
    B, Ci, H, W = x.shape
    N = H * W
    idx = np.ascontiguousarray(idx, dtype=np.int64)
    coef = haar_fwd(x, levels).reshape(B, Ci, N)
    xc = gather(coef, idx)
    alpha, sx = 0.0, 1.0
    if act_bits:
        alpha = float(np.float32(alpha_in if alpha_in > 0 else absmax(xc)))
        xc = quant_codes(xc, alpha, act_bits)
        sx = alpha / float((1 << (act_bits - 1)) - 1)
    sw = np.ones(w.shape[0]) if w_scale is None else _d(w_scale)
    yc = pointwise(w, sx * sw, xc)
    return haar_inv(scatter(yc, idx, N), H, W, levels), alpha


def depthwise3x3(x, w):
    """K_dw of Eq. (inverted): x [B, C, H, W], w [C, 3, 3] -> [B, C, H, W] (zero padding 1)."""
    x = _d(x)
    w = _d(w)
    B, Cc, H, W = x.shape
    assert w.shape == (Cc, 3, 3)
    y = np.empty_like(x)
    if lib().wcc_ref_depthwise3x3(_p(x), _p(w), B * Cc, Cc, H, W, _p(y)):
        raise ValueError("wcc_ref_depthwise3x3: bad arguments")
    return y


def block_forward(x, w1, w1_scale, w_dw, w3, w3_scale, levels: int, keep_num: int, keep_den: int,
                  act_bits: int = 0, norm: str = "l1"):
    """The inverted residual block of Eq. (inverted) with both 1x1 convolutions as WCC layers
    (activations left out, as in the paper's timings):
    x + WCC(K3, K_dw(WCC(K1, x))).  Returns (y, t1, t2, idx1, idx3, alpha1, alpha3) where
    t1 = WCC(K1, x) and t2 = K_dw t1."""
    x = _d(x)
    t1, idx1, a1 = forward(x, w1, w1_scale, levels, keep_num, keep_den, act_bits, norm=norm)
    t2 = depthwise3x3(t1, w_dw)
    t3, idx3, a3 = forward(t2, w3, w3_scale, levels, keep_num, keep_den, act_bits, norm=norm)
    return x + t3, t1, t2, idx1, idx3, a1, a3


def conv_mac(C_in, C_out, N_W, N_H, K_W=1, K_H=1, S_W=1, S_H=1) -> int:
    return int(lib().wcc_ref_conv_mac(C_in, C_out, N_W, N_H, K_W, K_H, S_W, S_H))


def conv_bops(mac, b_w, b_a) -> int:
    return int(lib().wcc_ref_conv_bops(mac, b_w, b_a))


def haar_bops(Cc, N_W, N_H, L, b_a) -> int:
    return int(lib().wcc_ref_haar_bops(Cc, N_W, N_H, L, b_a))
