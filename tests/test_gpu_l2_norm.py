"""Positions ranked by the sum of squares over channels (the Euclidean reading of the norm in
Alg. 1) instead of the sum of absolute values: HIP path vs CPU oracle through the C ABI.

Two kinds of input.  On a coarse dyadic grid every fp32 sum of squares is exact in any order,
so norms and index sets must match the oracle bit for bit.  On the ordinary inputs the sums
round, so the index set is checked for validity against the oracle's fp64 norms (everything
kept >= the k-th largest, everything dropped <= it, within 1e-5 relative) and the output is
compared with the oracle run on that index set.
"""
import numpy as np
import pytest
import torch

from paper_2205_12268_amd import synth, wcc
from tests.util import dev, rel_l2, tol_for, upload_weights

pytestmark = pytest.mark.gpu

F32, BF16, I8 = synth.W_F32, synth.W_BF16, synth.W_I8


def case(name, B, Ci, Co, H, W, d, num, den, wd, bits, base=2):
    return synth.small(synth.config(base), name=name, B=B, C_in=Ci, C_out=Co, H=H, W=W, levels=d,
                       keep_num=num, keep_den=den, w_dtype=wd, act_bits=bits,
                       seed=synth.SEED_BASE + 0x700 + sum(map(ord, name)))


def l2_desc(cfg, act_dtype=wcc.F32):
    return wcc.make_desc(cfg.B, cfg.C_in, cfg.C_out, cfg.H, cfg.W, cfg.levels, cfg.keep_num,
                         cfg.keep_den, cfg.w_dtype, cfg.act_bits, act_dtype, wcc.NORM_L2)


def coarse(x):
    """Multiples of 1/4 below 4: after d <= 3 levels the squares are multiples of 4^-(2+d) below
    4^(1+d), and sums over the channel counts used here stay below 2^24 units."""
    return np.minimum(np.floor(x * 4.0) / 4.0, 3.75).astype(np.float32)


@pytest.fixture(scope="module")
def ctx():
    c = wcc.Context(0)
    yield c
    c.close()


EXACT = [
    case("l2_d1", 2, 48, 16, 32, 64, 1, 1, 2, BF16, 8),          # one strip row per wave
    case("l2_d2_split", 1, 32, 24, 16, 32, 2, 1, 4, F32, 0),     # waves share a strip's channels
    case("l2_d3", 2, 8, 8, 64, 320, 3, 1, 8, I8, 8),             # two column segments
    case("l2_vec2", 1, 8, 8, 6, 10, 1, 1, 3, F32, 0),            # W % 4 != 0
    case("l2_groups", 1, 64, 8, 8, 16, 2, 1, 2, BF16, 0),        # few strips: several channel groups
]


@pytest.mark.parametrize("cfg", EXACT, ids=lambda c: c.name)
def test_exact_grid_matches_bit_for_bit(ref, ctx, cfg):
    print(f"case {cfg.name} seed {cfg.seed:#x}", flush=True)
    x, w = synth.make_inputs(cfg)
    x = coarse(x)
    N, k = cfg.N, cfg.k
    o_coef = ref.haar_fwd(x, cfg.levels).reshape(cfg.B, cfg.C_in, N)
    o_norm = ref.channel_norm(o_coef, "l2")
    assert o_norm.max() * 4.0 ** (2 + cfg.levels) < 2 ** 24          # the exactness budget holds
    o_y, o_idx, o_alpha = ref.forward(x, w.values, w.scale, cfg.levels, cfg.keep_num, cfg.keep_den,
                                      act_bits=cfg.act_bits, norm="l2")
    # the two norms must disagree somewhere, or the test shows nothing
    l1_idx = ref.topk(ref.channel_norm(o_coef, "l1"), k)
    d = l2_desc(cfg)
    ctx.ensure_workspace(d)
    xd = dev(x)
    wd, wsd = upload_weights(w)
    f32 = dict(dtype=torch.float32, device="cuda")

    coef = torch.full((cfg.B, cfg.C_in, N), float("nan"), **f32)
    norm = torch.full((cfg.B, N), float("nan"), **f32)
    ctx.wcc_haar_fwd(d, xd, coef, norm)
    np.testing.assert_array_equal(coef.cpu().numpy().astype(np.float64), o_coef)
    np.testing.assert_array_equal(norm.cpu().numpy().astype(np.float64), o_norm)

    idx = torch.full((cfg.B, k), -7, dtype=torch.int32, device="cuda")
    ctx.wcc_joint_topk(d, None, norm, idx)
    np.testing.assert_array_equal(idx.cpu().numpy().astype(np.int64), o_idx)
    idx2 = torch.full_like(idx, -7)
    ctx.wcc_joint_topk(d, coef, None, idx2)
    assert torch.equal(idx, idx2)

    y = torch.full((cfg.B, cfg.C_out, cfg.H, cfg.W), float("nan"), **f32)
    idxf = torch.full_like(idx, -7)
    af = torch.zeros(1, **f32)
    ctx.wcc_forward(d, xd, wd, wsd, 0.0, y, idxf, af)
    np.testing.assert_array_equal(idxf.cpu().numpy().astype(np.int64), o_idx)
    if cfg.act_bits:
        assert float(af.item()) == o_alpha
    err = rel_l2(y.cpu().numpy(), o_y)
    differs = not np.array_equal(l1_idx, o_idx)
    print(f"  rel-L2(y) = {err:.3e}; index set differs from the L1 one: {differs}", flush=True)
    assert err <= tol_for(cfg)
    if N >= 128:   # (a handful of positions can rank the same under both norms)
        assert differs


def check_valid(norm64, sel, k, rel=1e-5):
    N = norm64.shape[0]
    assert sel.shape == (k,) and np.all(np.diff(sel) > 0) and sel[0] >= 0 and sel[-1] < N
    kth = np.sort(norm64)[::-1][k - 1]
    dropped = np.ones(N, dtype=bool)
    dropped[sel] = False
    assert norm64[sel].min() >= kth * (1 - rel)
    if dropped.any():
        assert norm64[dropped].max() <= kth * (1 + rel)


ROUNDED = [
    case("l2r_bf16", 2, 24, 40, 48, 136, 3, 1, 8, BF16, 8),
    case("l2r_i8", 1, 32, 16, 64, 128, 2, 1, 4, I8, 8),
    case("l2r_f32", 2, 16, 16, 32, 32, 1, 1, 2, F32, 0),
    case("l2r_spiky", 1, 32, 32, 64, 128, 3, 1, 16, BF16, 8, base=3),
]


@pytest.mark.parametrize("cfg", ROUNDED, ids=lambda c: c.name)
def test_rounded_sums_give_a_valid_set_and_its_output(ref, ctx, cfg):
    print(f"case {cfg.name} seed {cfg.seed:#x}", flush=True)
    x, w = synth.make_inputs(cfg)
    N, k = cfg.N, cfg.k
    o_norm = ref.channel_norm(ref.haar_fwd(x, cfg.levels).reshape(cfg.B, cfg.C_in, N), "l2")
    d = l2_desc(cfg)
    ctx.ensure_workspace(d)
    wd, wsd = upload_weights(w)
    y = torch.full((cfg.B, cfg.C_out, cfg.H, cfg.W), float("nan"), dtype=torch.float32, device="cuda")
    idx = torch.full((cfg.B, k), -7, dtype=torch.int32, device="cuda")
    ctx.wcc_forward(d, dev(x), wd, wsd, 0.0, y, idx)
    g_idx = idx.cpu().numpy().astype(np.int64)
    for b in range(cfg.B):
        check_valid(o_norm[b], g_idx[b], k)
    want, _ = ref.forward_with_list(x, w.values, w.scale, cfg.levels, g_idx, cfg.act_bits)
    err = rel_l2(y.cpu().numpy(), want)
    # and against the oracle on its own: its index set may differ at the threshold only
    o_y, o_idx, _ = ref.forward(x, w.values, w.scale, cfg.levels, cfg.keep_num, cfg.keep_den,
                                act_bits=cfg.act_bits, norm="l2")
    moved = int((g_idx != o_idx).any(axis=1).sum())
    err_own = rel_l2(y.cpu().numpy(), o_y)
    print(f"  rel-L2(y) = {err:.3e}; against the oracle's own set {err_own:.3e} "
          f"({moved} of {cfg.B} samples keep a different set)", flush=True)
    assert err <= tol_for(cfg)
    assert err_own <= 3 * tol_for(cfg) + 1e-4


BLOCKS = [
    synth.BlockCfg("l2blk_bf16", 2, 16, 4, 32, 64, 2, 1, 4, BF16, 8, sigma=2.0, seed=synth.SEED_BASE + 0x720),
    synth.BlockCfg("l2blk_wide", 1, 8, 2, 16, 320, 2, 1, 4, I8, 8, sigma=2.0, seed=synth.SEED_BASE + 0x721),
    synth.BlockCfg("l2blk_f32_odd", 1, 4, 2, 8, 10, 1, 1, 2, F32, 0, sigma=1.0, seed=synth.SEED_BASE + 0x722),
]


@pytest.mark.parametrize("cfg", BLOCKS, ids=lambda c: c.name)
def test_block_layers_rank_by_l2(ref, ctx, cfg):
    """Both layers of the inverted residual block (the second one with K_dw folded into its
    transform passes): valid index sets for the tensors the GPU itself produced, and each
    layer's output for its set."""
    print(f"case {cfg.name} seed {cfg.seed:#x}", flush=True)
    x, w1, w_dw, w3 = synth.make_block_inputs(cfg)
    d = wcc.make_block_desc(cfg.B, cfg.C, cfg.expansion, cfg.H, cfg.W, cfg.levels, cfg.keep_num,
                            cfg.keep_den, cfg.w_dtype, cfg.act_bits, wcc.F32, wcc.NORM_L2)
    ctx.ensure_workspace(d)
    w1d, w1s = upload_weights(w1)
    w3d, w3s = upload_weights(w3)
    mid = (cfg.B, cfg.C_mid, cfg.H, cfg.W)
    t1 = torch.empty(mid, dtype=torch.float32, device="cuda")
    y = torch.empty(x.shape, dtype=torch.float32, device="cuda")
    idx1 = torch.empty((cfg.B, cfg.k), dtype=torch.int32, device="cuda")
    idx3 = torch.empty((cfg.B, cfg.k), dtype=torch.int32, device="cuda")
    ctx.wcc_block_forward(d, dev(x), w1d, w1s, dev(w_dw), w3d, w3s, y, t1, None, idx1, idx3)
    torch.cuda.synchronize()
    tol = 1e-5 if (cfg.w_dtype == F32 and cfg.act_bits == 0) else 1e-2
    N, k = cfg.N, cfg.k

    g_idx1 = idx1.cpu().numpy().astype(np.int64)
    n1 = ref.channel_norm(ref.haar_fwd(x, cfg.levels).reshape(cfg.B, cfg.C, N), "l2")
    for b in range(cfg.B):
        check_valid(n1[b], g_idx1[b], k)
    want1, _ = ref.forward_with_list(x, w1.values, w1.scale, cfg.levels, g_idx1, cfg.act_bits)
    g_t1 = t1.cpu().numpy()
    assert rel_l2(g_t1, want1) <= tol

    t2 = ref.depthwise3x3(g_t1, w_dw)
    g_idx3 = idx3.cpu().numpy().astype(np.int64)
    n3 = ref.channel_norm(ref.haar_fwd(t2, cfg.levels).reshape(cfg.B, cfg.C_mid, N), "l2")
    for b in range(cfg.B):
        check_valid(n3[b], g_idx3[b], k)
    want3, _ = ref.forward_with_list(t2, w3.values, w3.scale, cfg.levels, g_idx3, cfg.act_bits)
    err = rel_l2(y.cpu().numpy().astype(np.float64) - x.astype(np.float64), want3)
    print(f"  rel-L2(branch) = {err:.3e}", flush=True)
    assert err <= tol
