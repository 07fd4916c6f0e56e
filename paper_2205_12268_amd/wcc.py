"""ctypes binding of libwcc (argument marshalling only; every step runs in the HIP kernels).

torch is used for device memory and for the current HIP stream, nothing else.  There is no
CPU fallback: if ``csrc/libwcc.so`` is missing or does not load, importing the symbols below
raises.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "csrc", "libwcc.so")

F32, BF16, I8, I4 = 0, 1, 2, 3
STATIC_SCRATCH_BYTES = 64 << 20  # WCC_STATIC_SCRATCH_BYTES of wcc.h
NORM_L1, NORM_L2 = 0, 1
STAGES = ("haar_fwd", "norm_select", "gather", "pointwise", "scatter_ihaar", "event_pair",
          "depthwise")

EXPORTS = ("wcc_create", "wcc_destroy", "wcc_workspace_bytes", "wcc_set_workspace", "wcc_k",
           "wcc_status_string", "wcc_set_profiling", "wcc_stage_times", "wcc_haar_fwd",
           "wcc_joint_topk", "wcc_gather_quant", "wcc_pointwise", "wcc_scatter_ihaar",
           "wcc_forward", "wcc_forward_static", "wcc_forward_fixed", "wcc_block_workspace_bytes", "wcc_depthwise3x3", "wcc_block_forward",
           "wcc_set_block_profile_layer", "wcc_block_is_chained")


class Desc(C.Structure):
    """Mirror of ``wcc_desc``."""
    _fields_ = [("B", C.c_int32), ("C_in", C.c_int32), ("C_out", C.c_int32), ("H", C.c_int32),
                ("W", C.c_int32), ("levels", C.c_int32), ("keep_num", C.c_int64),
                ("keep_den", C.c_int64), ("w_dtype", C.c_int32), ("act_quant_bits", C.c_int32),
                ("act_dtype", C.c_int32), ("norm", C.c_int32)]


class BlockDesc(C.Structure):
    """Mirror of ``wcc_block_desc``."""
    _fields_ = [("B", C.c_int32), ("C", C.c_int32), ("expansion", C.c_int32), ("H", C.c_int32),
                ("W", C.c_int32), ("levels", C.c_int32), ("keep_num", C.c_int64),
                ("keep_den", C.c_int64), ("w_dtype", C.c_int32), ("act_quant_bits", C.c_int32),
                ("act_dtype", C.c_int32), ("norm", C.c_int32)]


class WccError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


_lib = None


def lib():
    """Loads libwcc.so (built by ``__graft_entry__.build()``); raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} not found: build it with `python -c 'import __graft_entry__ as g; g.build()'`")
        L = C.CDLL(LIB_PATH)
        vp, dp = C.c_void_p, C.POINTER(Desc)
        L.wcc_create.argtypes = [C.POINTER(vp), C.c_int]
        L.wcc_destroy.argtypes = [vp]
        L.wcc_workspace_bytes.argtypes = [dp, C.POINTER(C.c_size_t)]
        L.wcc_set_workspace.argtypes = [vp, vp, C.c_size_t]
        L.wcc_k.argtypes = [dp]
        L.wcc_k.restype = C.c_int64
        L.wcc_status_string.argtypes = [C.c_int]
        L.wcc_status_string.restype = C.c_char_p
        L.wcc_set_profiling.argtypes = [vp, C.c_int]
        L.wcc_stage_times.argtypes = [vp, C.POINTER(C.c_float)]
        L.wcc_haar_fwd.argtypes = [vp, dp, vp, vp, vp, vp]
        L.wcc_joint_topk.argtypes = [vp, dp, vp, vp, vp, vp]
        L.wcc_gather_quant.argtypes = [vp, dp, vp, vp, C.c_float, vp, vp, vp]
        L.wcc_pointwise.argtypes = [vp, dp, vp, vp, vp, vp, vp, vp]
        L.wcc_scatter_ihaar.argtypes = [vp, dp, vp, vp, vp, vp]
        L.wcc_forward.argtypes = [vp, dp, vp, vp, vp, C.c_float, vp, vp, vp, vp]
        L.wcc_forward_static.argtypes = [vp, dp, vp, vp, vp, C.c_float, vp, vp, vp, vp]
        L.wcc_forward_fixed.argtypes = [vp, dp, vp, vp, vp, C.c_float, vp, vp, vp, vp]
        bp = C.POINTER(BlockDesc)
        L.wcc_block_workspace_bytes.argtypes = [bp, C.POINTER(C.c_size_t)]
        L.wcc_depthwise3x3.argtypes = [vp, C.c_int32, C.c_int32, C.c_int32, C.c_int32, vp, vp, vp, vp]
        L.wcc_block_forward.argtypes = [vp, bp] + [vp] * 12
        L.wcc_set_block_profile_layer.argtypes = [vp, C.c_int]
        L.wcc_block_is_chained.argtypes = [bp]
        for name in EXPORTS:
            if name not in ("wcc_k", "wcc_status_string"):
                getattr(L, name).restype = C.c_int
        L.wcc_block_is_chained.restype = C.c_int32
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().wcc_status_string(int(status)).decode()


def _check(status: int, where: str) -> None:
    if status != 0:
        raise WccError(status, where)


def make_desc(B, C_in, C_out, H, W, levels, keep_num, keep_den, w_dtype, act_quant_bits,
              act_dtype=F32, norm=NORM_L1) -> Desc:
    return Desc(B, C_in, C_out, H, W, levels, keep_num, keep_den, w_dtype, act_quant_bits, act_dtype,
                norm)


def k_of(desc: Desc) -> int:
    return int(lib().wcc_k(C.byref(desc)))


def workspace_bytes(desc: Desc) -> int:
    out = C.c_size_t(0)
    _check(lib().wcc_workspace_bytes(C.byref(desc), C.byref(out)), "wcc_workspace_bytes")
    return int(out.value)


def make_block_desc(B, Cc, expansion, H, W, levels, keep_num, keep_den, w_dtype,
                    act_quant_bits, act_dtype=F32, norm=NORM_L1) -> BlockDesc:
    return BlockDesc(B, Cc, expansion, H, W, levels, keep_num, keep_den, w_dtype, act_quant_bits,
                     act_dtype, norm)


def block_is_chained(desc: BlockDesc) -> bool:
    """Whether wcc_block_forward without middle outputs chains the two layers of this block."""
    r = int(lib().wcc_block_is_chained(C.byref(desc)))
    if r < 0:
        raise ValueError("invalid block descriptor")
    return r == 1


def block_workspace_bytes(desc: BlockDesc) -> int:
    out = C.c_size_t(0)
    _check(lib().wcc_block_workspace_bytes(C.byref(desc), C.byref(out)), "wcc_block_workspace_bytes")
    return int(out.value)


def _ptr(t):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device tensors must be contiguous"
    return C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


class Context:
    """Owns a ``wcc_ctx`` and the torch tensor that backs its workspace."""

    def __init__(self, device: int = 0):
        self._h = C.c_void_p()
        self.device = device
        _check(lib().wcc_create(C.byref(self._h), device), "wcc_create")
        self._ws = None

    def close(self):
        if self._h:
            lib().wcc_destroy(self._h)
            self._h = C.c_void_p()
            self._ws = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def ensure_workspace(self, desc) -> int:
        need = block_workspace_bytes(desc) if isinstance(desc, BlockDesc) else workspace_bytes(desc)
        if self._ws is None or self._ws.numel() < need:
            self._ws = torch.empty(need, dtype=torch.uint8, device=f"cuda:{self.device}")
            _check(lib().wcc_set_workspace(self._h, _ptr(self._ws), self._ws.numel()),
                   "wcc_set_workspace")
        return need

    def set_workspace(self, tensor) -> None:
        self._ws = tensor
        _check(lib().wcc_set_workspace(self._h, _ptr(tensor), 0 if tensor is None else tensor.numel()),
               "wcc_set_workspace")

    def set_profiling(self, on: bool) -> None:
        _check(lib().wcc_set_profiling(self._h, int(bool(on))), "wcc_set_profiling")

    def stage_times(self) -> dict:
        ms = (C.c_float * len(STAGES))()
        _check(lib().wcc_stage_times(self._h, ms), "wcc_stage_times")
        return {n: float(ms[i]) for i, n in enumerate(STAGES)}

    # ---- the five stages and the fused call: same names as the C entry points ----
    def wcc_haar_fwd(self, desc, x, coef, norm=None):
        _check(lib().wcc_haar_fwd(self._h, C.byref(desc), _ptr(x), _ptr(coef), _ptr(norm), _stream()),
               "wcc_haar_fwd")

    def wcc_joint_topk(self, desc, coef, norm, idx):
        _check(lib().wcc_joint_topk(self._h, C.byref(desc), _ptr(coef), _ptr(norm), _ptr(idx),
                                    _stream()), "wcc_joint_topk")

    def wcc_gather_quant(self, desc, coef, idx, alpha_in, xc, alpha_dev):
        _check(lib().wcc_gather_quant(self._h, C.byref(desc), _ptr(coef), _ptr(idx),
                                      C.c_float(alpha_in), _ptr(xc), _ptr(alpha_dev), _stream()),
               "wcc_gather_quant")

    def wcc_pointwise(self, desc, w, w_scale, xc, alpha_dev, yc):
        _check(lib().wcc_pointwise(self._h, C.byref(desc), _ptr(w), _ptr(w_scale), _ptr(xc),
                                   _ptr(alpha_dev), _ptr(yc), _stream()), "wcc_pointwise")

    def wcc_scatter_ihaar(self, desc, yc, idx, y):
        _check(lib().wcc_scatter_ihaar(self._h, C.byref(desc), _ptr(yc), _ptr(idx), _ptr(y),
                                       _stream()), "wcc_scatter_ihaar")

    def wcc_forward(self, desc, x, w, w_scale, alpha_in, y, idx_out=None, alpha_out=None):
        _check(lib().wcc_forward(self._h, C.byref(desc), _ptr(x), _ptr(w), _ptr(w_scale),
                                 C.c_float(alpha_in), _ptr(y), _ptr(idx_out), _ptr(alpha_out),
                                 _stream()), "wcc_forward")

    def wcc_forward_static(self, desc, x, w, w_scale, alpha_in, y, idx_out=None, alpha_out=None):
        _check(lib().wcc_forward_static(self._h, C.byref(desc), _ptr(x), _ptr(w), _ptr(w_scale),
                                        C.c_float(alpha_in), _ptr(y), _ptr(idx_out), _ptr(alpha_out),
                                        _stream()), "wcc_forward_static")

    def wcc_forward_fixed(self, desc, x, w, w_scale, alpha_in, idx, y, alpha_out=None):
        _check(lib().wcc_forward_fixed(self._h, C.byref(desc), _ptr(x), _ptr(w), _ptr(w_scale),
                                       C.c_float(alpha_in), _ptr(idx), _ptr(y), _ptr(alpha_out),
                                       _stream()), "wcc_forward_fixed")

    # ---- the inverted residual block (next row) ----
    def wcc_depthwise3x3(self, x, w, y):
        B, Cc, H, W = x.shape
        _check(lib().wcc_depthwise3x3(self._h, B, Cc, H, W, _ptr(x), _ptr(w), _ptr(y), _stream()),
               "wcc_depthwise3x3")

    def wcc_block_forward(self, desc, x, w1, w1_scale, w_dw, w3, w3_scale, y, t1_out=None,
                          t2_out=None, idx1_out=None, idx3_out=None):
        _check(lib().wcc_block_forward(self._h, C.byref(desc), _ptr(x), _ptr(w1), _ptr(w1_scale),
                                       _ptr(w_dw), _ptr(w3), _ptr(w3_scale), _ptr(y), _ptr(t1_out),
                                       _ptr(t2_out), _ptr(idx1_out), _ptr(idx3_out), _stream()),
               "wcc_block_forward")

    def set_block_profile_layer(self, layer: int) -> None:
        _check(lib().wcc_set_block_profile_layer(self._h, int(layer)), "wcc_set_block_profile_layer")
