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


def layer_with_index_set(ref, lcfg, w, x64, idx):
    """Alg. 1 on x64 with the index set given (the oracle's steps after the selection).
    Returns (y, channel norms of the wavelet vectors)."""
    N = lcfg.N
    coef = ref.haar_fwd(x64, lcfg.levels).reshape(lcfg.B, lcfg.C_in, N)
    norm = ref.channel_norm(coef)
    xc = ref.gather(coef, idx)
    if lcfg.act_bits:
        alpha = float(np.float32(ref.absmax(xc)))
        xhat = ref.quant_codes(xc, alpha, lcfg.act_bits)
    else:
        alpha, xhat = 0.0, xc
    yc = ref.pointwise(w.values, oracle_scale(ref, lcfg, w, alpha), xhat)
    y = ref.haar_inv(ref.scatter(yc, idx, N), lcfg.H, lcfg.W, lcfg.levels)
    return y, norm


def assert_valid_index_set(norm_b, sel, k, rel=1e-5):
    """sel is a correct answer to "the k positions with the largest norm" for norms known to a
    relative accuracy of `rel`: strictly ascending, inside the plane, every kept norm at least
    the k-th largest and every dropped norm at most it."""
    N = norm_b.shape[0]
    assert sel.shape == (k,) and np.all(np.diff(sel) > 0) and sel[0] >= 0 and sel[-1] < N
    kth = np.sort(norm_b)[::-1][k - 1]
    dropped = np.ones(N, dtype=bool)
    dropped[sel] = False
    assert norm_b[sel].min() >= kth * (1 - rel)
    if dropped.any():
        assert norm_b[dropped].max() <= kth * (1 + rel)


def check_block_without_middle_outputs(ref, ctx, cfg, d, xd, x_np, w1d, w1s, wdd, w3d, w3s, w3,
                                       g_t2, y_mat, idx3_mat, tol):
    """The block called without the test outputs: where the shape allows, the library then
    chains the two layers in the compressed domain (the middle tensors are never formed).  Its
    second index set must be valid for the fp64 norms of K_dw's output as the materialised call
    gave it (g_t2; the chained passes rebuild the same fp32 numbers), its output must match the
    oracle run on that set, and where the two calls chose the same set (same kept values, same
    alpha, same codes) the outputs must be equal bit for bit.  Returns whether the sets agreed."""
    y_p = torch.full_like(y_mat, float("nan"))
    idx3_p = torch.full_like(idx3_mat, -7)
    ctx.wcc_block_forward(d, xd, w1d, w1s, wdd, w3d, w3s, y_p, None, None, None, idx3_p)
    torch.cuda.synchronize()
    g_idx3 = idx3_p.cpu().numpy().astype(np.int64)
    want_branch, norm = layer_with_index_set(ref, cfg.layer(1), w3, g_t2.astype(np.float64), g_idx3)
    for b in range(cfg.B):
        assert_valid_index_set(norm[b], g_idx3[b], cfg.k)
    got = y_p.float().cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all()
    assert rel_l2(got - x_np, want_branch) <= tol
    same = bool(torch.equal(idx3_p, idx3_mat))
    if same:
        assert torch.equal(y_p, y_mat)
    return same
