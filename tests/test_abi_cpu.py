"""The C-ABI library loads and exports every symbol the header declares; host-only entry
points (no kernel launch, no device needed) behave as documented."""
import ctypes as C
import os
import re

import pytest

from paper_2205_12268_amd import synth, wcc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions(header="wcc.h"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = set(re.findall(r"\b(wcc_[a-z_0-9]+)\s*\(", text))
    return sorted(names)


def test_header_and_binding_agree():
    names = declared_functions()
    assert set(names) == set(wcc.EXPORTS)
    for n in ("wcc_haar_fwd", "wcc_joint_topk", "wcc_gather_quant", "wcc_pointwise",
              "wcc_scatter_ihaar", "wcc_forward"):
        assert n in names and hasattr(wcc.Context, n)


def test_library_exports_every_declared_symbol():
    L = C.CDLL(wcc.LIB_PATH)
    for n in declared_functions():
        assert getattr(L, n) is not None, n


def test_probe_library_is_separate_and_exports_its_header():
    """The streaming probe is a measurement aid in a library of its own: libwcc exports none of
    it, and libwcc_probe.so exports what include/wcc_probe.h declares."""
    from paper_2205_12268_amd import probe
    names = declared_functions("wcc_probe.h")
    assert set(names) == set(probe.EXPORTS) == {"wcc_probe_stream"}
    P = C.CDLL(probe.LIB_PATH)
    for n in names:
        assert getattr(P, n) is not None, n
    assert not hasattr(C.CDLL(wcc.LIB_PATH), "wcc_probe_stream")
    assert "probe" not in open(os.path.join(ROOT, "include", "wcc.h")).read()


def test_k_and_workspace_are_pure_host_functions():
    for n, k in ((1, 2048), (2, 32768), (3, 65536), (4, 7680)):
        cfg = synth.config(n)
        d = wcc.make_desc(cfg.B, cfg.C_in, cfg.C_out, cfg.H, cfg.W, cfg.levels, cfg.keep_num,
                          cfg.keep_den, cfg.w_dtype, cfg.act_bits)
        assert wcc.k_of(d) == k == cfg.k
        ws = wcc.workspace_bytes(d)
        assert ws % 256 == 0
        N = cfg.H * cfg.W
        must_hold = 4 * cfg.B * (cfg.C_in * k + cfg.C_out * k + 2 * N)
        assert ws >= must_hold
    d = wcc.make_desc(1, 4, 4, 8, 8, 1, 1, 3, wcc.F32, 0)
    assert wcc.k_of(d) == 22  # ceil(64/3)


@pytest.mark.parametrize("kw,status", [
    (dict(H=12, levels=3), 2), (dict(levels=0), 2), (dict(levels=5), 2), (dict(B=0), 2),
    (dict(W=6, levels=2), 2), (dict(w_dtype=7), 3), (dict(act_quant_bits=4), 3),
    (dict(keep_num=0), 4), (dict(keep_num=3, keep_den=2), 4), (dict(keep_den=0), 4),
    (dict(norm=2), 3), (dict(norm=wcc.NORM_L2, act_dtype=wcc.BF16), 6),
])
def test_descriptor_errors(kw, status):
    base = dict(B=1, C_in=4, C_out=4, H=16, W=16, levels=2, keep_num=1, keep_den=4,
                w_dtype=wcc.F32, act_quant_bits=0)
    base.update(kw)
    d = wcc.make_desc(**base)
    assert wcc.k_of(d) == -1
    out = C.c_size_t(0)
    assert wcc.lib().wcc_workspace_bytes(C.byref(d), C.byref(out)) == status
    assert wcc.status_string(status) != "unknown status"


def test_null_arguments_are_reported_not_dereferenced():
    L = wcc.lib()
    d = wcc.make_desc(1, 4, 4, 16, 16, 2, 1, 4, wcc.F32, 0)
    assert L.wcc_workspace_bytes(C.byref(d), None) == 1
    assert L.wcc_workspace_bytes(None, C.byref(C.c_size_t(0))) == 1
    assert L.wcc_destroy(None) == 1
    assert L.wcc_set_workspace(None, None, 0) == 1
    assert L.wcc_haar_fwd(None, C.byref(d), None, None, None, None) == 1
    assert L.wcc_forward(None, C.byref(d), None, None, None, 0.0, None, None, None, None) == 1
    assert wcc.status_string(0) == "ok"


def test_which_blocks_are_chained():
    """Pure host function: chained when nobody asks for the middle tensors and W % 4 == 0,
    a row fits one wave row (W <= 256) or is exactly two or four of them, levels <= 3, at most a
    third of the coefficients kept."""
    def chained(H, W, levels, num, den):
        return wcc.block_is_chained(wcc.make_block_desc(2, 8, 4, H, W, levels, num, den, wcc.BF16, 8))
    assert chained(256, 256, 3, 1, 4) and chained(96, 96, 3, 1, 8) and chained(48, 64, 1, 1, 3)
    assert not chained(256, 256, 3, 1, 2)        # more than a third kept
    assert chained(512, 512, 3, 1, 4) and chained(64, 264, 3, 1, 4) and chained(64, 1024, 3, 1, 4)
    assert chained(64, 776, 2, 1, 4)             # 194 lanes: four wave rows
    assert not chained(64, 768, 3, 1, 4)         # three wave rows
    assert not chained(64, 1032, 3, 1, 4)        # five
    assert not chained(64, 64, 4, 1, 4)          # four levels
    assert not chained(16, 10, 1, 1, 4)          # W % 4 != 0
    with pytest.raises(ValueError):
        chained(60, 64, 3, 1, 4)                 # H not divisible by 8
