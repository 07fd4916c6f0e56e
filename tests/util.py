"""Shared helpers of the GPU parity tests (data movement and error norms only)."""
from __future__ import annotations

import numpy as np
import torch

from paper_2205_12268_amd import synth, wcc


def desc_of(cfg: synth.LayerCfg) -> wcc.Desc:
    return wcc.make_desc(cfg.B, cfg.C_in, cfg.C_out, cfg.H, cfg.W, cfg.levels, cfg.keep_num,
                         cfg.keep_den, cfg.w_dtype, cfg.act_bits)


def dev(a: np.ndarray) -> torch.Tensor:
    if a.dtype == np.uint16:  # bf16 bit patterns
        a = a.view(np.int16)
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def upload_weights(w: synth.Weights):
    return dev(w.stored), (None if w.scale is None else dev(w.scale))


def rel_l2(got, want) -> float:
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    den = np.linalg.norm(want.ravel())
    num = np.linalg.norm((got - want).ravel())
    return float(num / den) if den > 0 else float(num)


def tol_for(cfg: synth.LayerCfg) -> float:
    """1e-5 relative L2 for the fp32 path, 1e-2 for bf16 / int8 accumulation."""
    return 1e-5 if (cfg.w_dtype == synth.W_F32 and cfg.act_bits == 0) else 1e-2


def oracle_scale(ref, cfg, w, alpha):
    sx = alpha / 127.0 if cfg.act_bits else 1.0
    sw = np.ones(cfg.C_out) if w.scale is None else w.scale.astype(np.float64)
    return sx * sw
