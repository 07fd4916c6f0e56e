"""ctypes binding of libwcc_probe.so: plain streaming kernels (read, write, copy) that bench.py
times beside the library's kernels.  A measurement aid; not part of libwcc."""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "csrc", "libwcc_probe.so")
EXPORTS = ("wcc_probe_stream",)

READ, WRITE, COPY, WRITE8 = 0, 1, 2, 3
_STATUS = {1: "required pointer is NULL", 2: "bad size, block count or alignment", 3: "unknown kind",
           7: "HIP runtime error"}


class ProbeError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__(f"wcc_probe_stream: {_STATUS.get(status, 'unknown status')} (status {status})")


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} not found: build it with `python -c 'import __graft_entry__ as g; g.build()'`")
        L = C.CDLL(LIB_PATH)
        L.wcc_probe_stream.argtypes = [C.c_int, C.c_void_p, C.c_void_p, C.c_size_t, C.c_int, C.c_int,
                                       C.c_void_p]
        L.wcc_probe_stream.restype = C.c_int
        _lib = L
    return _lib


def _ptr(t):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device tensors must be contiguous"
    return C.c_void_p(t.data_ptr())


def wcc_probe_stream(kind: int, src, dst, nbytes: int, nontemporal: bool = False, blocks: int = 0) -> None:
    st = lib().wcc_probe_stream(int(kind), _ptr(src), _ptr(dst), C.c_size_t(nbytes),
                                int(bool(nontemporal)), int(blocks),
                                C.c_void_p(torch.cuda.current_stream().cuda_stream))
    if st != 0:
        raise ProbeError(st)
