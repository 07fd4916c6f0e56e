"""The inverted residual block of Eq. (inverted), x + WCC(K3, K_dw(WCC(K1, x))), on the GPU
against the oracle, stage by stage and end to end.

The first layer sees dyadic inputs, so its index set is compared exactly.  The second layer
sees arbitrary fp32 numbers (the output of the first layer and of K_dw): there fp32 norms may
order two nearly equal positions differently from fp64 norms, so its index set is checked for
VALIDITY against the oracle's fp64 norms (every kept norm >= the k-th largest, every dropped
norm <= it, up to a relative 1e-5), and its output is compared with the oracle run on the
same index set.
"""
from __future__ import annotations

import numpy as np
import pytest
import torch

from paper_2205_12268_amd import synth, wcc
from tests.util import assert_valid_index_set, check_block_without_middle_outputs, layer_with_index_set, dev, oracle_scale, rel_l2, upload_weights

pytestmark = pytest.mark.gpu

F32, BF16, I8 = synth.W_F32, synth.W_BF16, synth.W_I8


@pytest.fixture(scope="module")
def ctx():
    c = wcc.Context(0)
    yield c
    c.close()


@pytest.mark.parametrize("shape", [(1, 3, 8, 8), (2, 5, 19, 36), (1, 2, 33, 520), (2, 3, 16, 1028),
                                   (1, 4, 7, 10), (1, 1, 1, 4), (1, 2, 5, 6)])
def test_depthwise_matches_oracle(ref, ctx, shape):
    """Widths that end inside a wave's 256-column segment, cross segments, are not multiples
    of 4; heights that are not multiples of the 8-row strips; arbitrary floats."""
    rng = np.random.default_rng(sum(shape))
    x = rng.standard_normal(shape).astype(np.float32)
    w = rng.standard_normal((shape[1], 3, 3)).astype(np.float32)
    y = torch.full(shape, float("nan"), dtype=torch.float32, device="cuda")
    ctx.wcc_depthwise3x3(dev(x), dev(w), y)
    want = ref.depthwise3x3(x, w)
    got = y.cpu().numpy()
    assert np.isfinite(got).all()
    assert rel_l2(got, want) <= 1e-6
    np.testing.assert_allclose(got, want, rtol=0, atol=2e-5)


CASES = [
    synth.BlockCfg("blk_bf16_d2", 2, 16, 4, 32, 64, 2, 1, 4, BF16, 8, sigma=2.0, seed=synth.SEED_BASE + 0x610),
    synth.BlockCfg("blk_i8_d3", 1, 32, 2, 64, 128, 3, 1, 8, I8, 8, sigma=3.0, seed=synth.SEED_BASE + 0x611),
    synth.BlockCfg("blk_f32_d1", 2, 8, 3, 16, 24, 1, 1, 2, F32, 0, sigma=1.0, seed=synth.SEED_BASE + 0x612),
    synth.BlockCfg("blk_bf16_big_plane", 1, 8, 6, 128, 256, 3, 1, 4, BF16, 8, sigma=3.0, seed=synth.SEED_BASE + 0x613),
    # rows wider than a wave: the folded K_dw reads its outside columns from memory
    synth.BlockCfg("blk_bf16_wide", 1, 8, 2, 16, 320, 2, 1, 4, BF16, 8, sigma=2.0, seed=synth.SEED_BASE + 0x614),
    synth.BlockCfg("blk_i8_wide_d1", 2, 16, 2, 8, 1024, 1, 1, 2, I8, 8, sigma=2.0, seed=synth.SEED_BASE + 0x615),
    # W % 4 != 0: K_dw stays a kernel of its own
    synth.BlockCfg("blk_f32_odd_width", 1, 4, 2, 8, 10, 1, 1, 2, F32, 0, sigma=1.0, seed=synth.SEED_BASE + 0x616),
]


@pytest.mark.parametrize("cfg", CASES, ids=lambda c: c.name)
def test_block_stage_by_stage_and_end_to_end(ref, ctx, cfg):
    x, w1, w_dw, w3 = synth.make_block_inputs(cfg)
    l0, l1 = cfg.layer(0), cfg.layer(1)
    d = wcc.make_block_desc(cfg.B, cfg.C, cfg.expansion, cfg.H, cfg.W, cfg.levels, cfg.keep_num,
                            cfg.keep_den, cfg.w_dtype, cfg.act_bits)
    ctx.ensure_workspace(d)
    xd = dev(x)
    w1d, w1s = upload_weights(w1)
    w3d, w3s = upload_weights(w3)
    mid = (cfg.B, cfg.C_mid, cfg.H, cfg.W)
    t1 = torch.empty(mid, dtype=torch.float32, device="cuda")
    t2 = torch.empty(mid, dtype=torch.float32, device="cuda")
    y = torch.empty(x.shape, dtype=torch.float32, device="cuda")
    idx1 = torch.empty((cfg.B, cfg.k), dtype=torch.int32, device="cuda")
    idx3 = torch.empty((cfg.B, cfg.k), dtype=torch.int32, device="cuda")
    ctx.wcc_block_forward(d, xd, w1d, w1s, dev(w_dw), w3d, w3s, y, t1, t2, idx1, idx3)
    torch.cuda.synchronize()
    tol = 1e-5 if (cfg.w_dtype == F32 and cfg.act_bits == 0) else 1e-2


    # layer 1 (dyadic input): exact index set, output within tolerance
    o_t1, o_idx1, _ = ref.forward(x, w1.values, w1.scale, cfg.levels, cfg.keep_num, cfg.keep_den,
                                  act_bits=cfg.act_bits)
    np.testing.assert_array_equal(idx1.cpu().numpy().astype(np.int64), o_idx1)
    g_t1 = t1.cpu().numpy()
    assert rel_l2(g_t1, o_t1) <= tol

    # K_dw on the GPU's own t1
    g_t2 = t2.cpu().numpy()
    assert rel_l2(g_t2, ref.depthwise3x3(g_t1, w_dw)) <= 1e-6

    # layer 3 on the GPU's own t2: a valid index set, then the output for that set
    g_idx3 = idx3.cpu().numpy().astype(np.int64)
    want_branch, norm = layer_with_index_set(ref, l1, w3, g_t2.astype(np.float64), g_idx3)
    for b in range(cfg.B):
        assert_valid_index_set(norm[b], g_idx3[b], cfg.k)
    g_branch = y.cpu().numpy().astype(np.float64) - x.astype(np.float64)
    assert rel_l2(g_branch, want_branch) <= tol

    # without the test outputs: chained in the compressed domain where the shape allows
    same = check_block_without_middle_outputs(ref, ctx, cfg, d, xd, x.astype(np.float64), w1d, w1s,
                                              dev(w_dw), w3d, w3s, w3, g_t2, y, idx3, tol)
    print(f"{cfg.name}: call without middle outputs chose {'the same' if same else 'another valid'} "
          f"second index set", flush=True)

    # End to end against the independent oracle chain (its own index sets throughout).  Where
    # the two second-layer sets agree the chain is held to the same bar; where fp32 and fp64
    # norms order two nearly equal positions differently both sets are correct, the outputs
    # belong to different sets, and the figure is printed only.
    o = ref.block_forward(x, w1.values, w1.scale, w_dw, w3.values, w3.scale, cfg.levels,
                          cfg.keep_num, cfg.keep_den, cfg.act_bits)
    err = rel_l2(g_branch, o[0] - x)
    same = np.array_equal(g_idx3, o[4])
    print(f"{cfg.name}: end-to-end rel-L2 of the branch = {err:.3e} (second index set "
          f"{'equal' if same else 'differs'})", flush=True)
    if same:
        assert err <= tol


def test_block_error_paths(ctx):
    d = wcc.make_block_desc(1, 8, 2, 16, 16, 2, 1, 4, wcc.BF16, 8)
    ctx.ensure_workspace(d)
    x = torch.zeros((1, 8, 16, 16), device="cuda")
    w = torch.zeros((16, 8), dtype=torch.int16, device="cuda")
    wd = torch.zeros((16, 3, 3), device="cuda")
    y = torch.empty_like(x)
    with pytest.raises(wcc.WccError) as e:
        ctx.wcc_block_forward(d, x, w, None, None, w, None, y)
    assert e.value.status == 1  # NULL depthwise kernel
    bad = wcc.make_block_desc(1, 8, 2, 12, 16, 3, 1, 4, wcc.BF16, 8)  # H not divisible by 8
    with pytest.raises(wcc.WccError) as e:
        wcc.block_workspace_bytes(bad)
    assert e.value.status == 2
    big = wcc.make_block_desc(1, 8, 9000, 16, 16, 2, 1, 4, wcc.BF16, 8)  # C * expansion too large
    with pytest.raises(wcc.WccError) as e:
        wcc.block_workspace_bytes(big)
    assert e.value.status == 2
    i8 = wcc.make_block_desc(1, 8, 2, 16, 16, 2, 1, 4, wcc.I8, 8)
    ctx.ensure_workspace(i8)
    with pytest.raises(wcc.WccError) as e:
        ctx.wcc_block_forward(i8, x, w, None, wd, w, None, y)
    assert e.value.status == 1  # int8 weights need their scales


@pytest.mark.parametrize("width,want_t2", [(16, True), (18, False)])
def test_block_refusal_enqueues_nothing(ctx, width, want_t2):
    """bf16 feature maps need K_dw folded into the transform (W % 4 == 0, no K_dw output asked
    for).  The refusal comes with the other argument checks: no kernel has run, so the output,
    the caller's middle tensor and the workspace are as they were."""
    d = wcc.make_block_desc(1, 8, 2, 16, width, 1, 1, 4, wcc.BF16, 8, wcc.BF16)
    need = ctx.ensure_workspace(d)
    x = torch.ones((1, 8, 16, width), dtype=torch.bfloat16, device="cuda")
    w = torch.zeros((16, 8), dtype=torch.int16, device="cuda")
    wd = torch.zeros((16, 3, 3), device="cuda")
    y = torch.full_like(x, 5.0)
    t1 = torch.full((1, 16, 16, width), 7.0, dtype=torch.bfloat16, device="cuda")
    t2 = torch.full((1, 16, 16, width), 9.0, dtype=torch.float32, device="cuda") if want_t2 else None
    ctx._ws.fill_(0x5A)
    torch.cuda.synchronize()
    with pytest.raises(wcc.WccError) as e:
        ctx.wcc_block_forward(d, x, w, None, wd, w, None, y, t1, t2)
    assert e.value.status == 6  # WCC_ERR_UNSUPPORTED
    torch.cuda.synchronize()
    assert bool((y == 5.0).all()) and bool((t1 == 7.0).all())
    assert t2 is None or bool((t2 == 9.0).all())
    assert bool((ctx._ws[:need] == 0x5A).all())
