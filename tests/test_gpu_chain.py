"""Compressed-domain chaining of the inverted residual block (appendix "Inference times",
paragraph on memory bandwidth and traffic) against the oracle and against the route that forms
the middle tensors (needs an MI355X).

wcc_block_forward chains the two layers when no middle output is asked for and the shape allows
(W % 4 == 0, d <= 3, W <= 256 or a row of exactly 2 or 4 wave rows): the project layer's transform passes rebuild the rows they need
from the expand layer's compressed output.  The shapes below walk through what that code
depends on: one, two and four strips a wave, planes of one strip (no row above or below), many
strips, rows that leave lanes idle, every level count, kept lists of 4, 8, 16 and 32 rows a wave,
strips that keep everything (the slot-by-slot route) and strips that keep nothing, no quantiser,
int8 weights, several samples and channel groups, and rows shared by two and by four waves (full
and ragged last segments, a last segment of one lane; empty strips beside full ones; every level count),
followed by 60 seeded random shapes (a sweep of such shapes is what found the one-lane case).
"""
import numpy as np
import pytest
import torch

from paper_2205_12268_amd import synth, wcc
from tests.util import (assert_valid_index_set, check_block_without_middle_outputs, dev,
                        layer_with_index_set, rel_l2, upload_weights)

pytestmark = pytest.mark.gpu

F32, BF16, I8 = synth.W_F32, synth.W_BF16, synth.W_I8


def blk(name, B, C, e, H, W, d, num, den, wd, bits, sigma=2.0):
    return synth.BlockCfg(name, B, C, e, H, W, d, num, den, wd, bits, sigma=sigma,
                          seed=synth.SEED_BASE + 0xC00 + sum(map(ord, name)))


CASES = [
    blk("full_wave_d3", 1, 8, 4, 64, 256, 3, 1, 8, BF16, 8, 3.0),      # W = 256: one strip a wave
    blk("two_strips_d3", 2, 8, 2, 48, 128, 3, 1, 4, BF16, 8),          # two strips a wave
    blk("idle_lanes_d3", 1, 4, 3, 40, 96, 3, 1, 4, BF16, 8),           # 24 of 32 lanes a row
    blk("four_strips_d2", 1, 8, 2, 36, 64, 2, 1, 4, I8, 8),            # four strips a wave, ragged last wave
    blk("one_strip_plane", 2, 4, 2, 8, 64, 3, 1, 4, BF16, 8),          # no row above or below
    blk("d1_tall", 1, 4, 2, 30, 32, 1, 1, 4, BF16, 8),                 # d = 1: every slot is a halo slot
    blk("d2_dense_top", 1, 8, 4, 64, 256, 2, 1, 4, BF16, 8),           # long lists (16 rows a wave) on top, empty strips below
    blk("d3_dense_top", 1, 4, 2, 32, 256, 3, 1, 4, BF16, 8),           # lists of more than 16 rows; empty strips
    blk("d3_all_on_top", 1, 4, 2, 32, 256, 3, 1, 4, BF16, 8),          # strips that keep everything: slot by slot
    blk("keep_few_d3", 1, 8, 2, 64, 256, 3, 1, 64, BF16, 8, 3.0),      # short lists, empty strips
    blk("f32_noquant_d2", 2, 4, 3, 16, 48, 2, 1, 3, F32, 0, 1.0),      # fp32 path, k % 4 != 0
    blk("ragged_k_d3", 1, 8, 2, 24, 40, 3, 2, 7, BF16, 8),             # k % 4 != 0 with the quantiser
    blk("many_channels", 2, 16, 8, 32, 64, 3, 1, 4, BF16, 8),          # 128 middle channels in groups
    blk("two_segments_d3", 2, 8, 2, 24, 512, 3, 1, 4, BF16, 8, 3.0),   # a row shared by two waves
    blk("two_segments_ragged", 1, 4, 3, 16, 328, 3, 1, 8, BF16, 8),    # 64 + 18 lanes a row
    blk("four_segments_d3", 1, 4, 2, 16, 1024, 3, 1, 8, BF16, 8, 3.0), # a row shared by four waves
    blk("four_segments_d2", 1, 8, 2, 12, 776, 2, 1, 4, I8, 8),         # 64 + 64 + 64 + 2 lanes a row
    blk("two_segments_d1", 1, 4, 2, 6, 384, 1, 1, 4, BF16, 8),         # d = 1, 64 + 32 lanes
    blk("two_segments_dense_top", 1, 4, 2, 32, 512, 3, 1, 4, BF16, 8), # packed, slot-by-slot and empty strips in one plane
    blk("two_segments_f32", 1, 4, 2, 16, 512, 2, 2, 7, F32, 0, 1.0),   # fp32 path through shared rows
    blk("two_segments_lone_lane", 1, 4, 2, 14, 260, 1, 1, 5, BF16, 8, 1.0),   # 64 + 1 lanes: the last lane is first and last of its segment
    blk("four_segments_lone_lane", 3, 16, 8, 14, 772, 1, 1, 5, I8, 8, 1.0),   # 64 + 64 + 64 + 1 lanes
    blk("two_segments_lone_lane_d2", 2, 4, 3, 16, 260, 2, 1, 4, BF16, 8),      # the same at d = 2 (W % 8 == 4: no d = 3)
    # enough kept coefficients in the project layer for the int8 route (clipping parameter known
    # before the second pass; the small cases above take the fp32 route)
    blk("codes_two_strips", 4, 64, 8, 64, 128, 3, 1, 4, BF16, 8),      # 512 middle channels, k = 2048
    blk("codes_idle_lanes", 4, 128, 8, 48, 96, 3, 1, 4, I8, 8),        # 1024 middle channels, 24 of 32 lanes
    blk("codes_two_segments", 2, 64, 8, 32, 512, 3, 1, 4, BF16, 8),    # shared rows, k = 4096
]
# Rows of the input from this fraction of the height on are zero, so that the kept positions of
# both layers crowd into the strips above: strips that keep a half or all of their positions at
# a keep ratio the chained route takes, and strips that keep nothing.
ZERO_BELOW = {"d2_dense_top": 0.5, "d3_dense_top": 0.5, "d3_all_on_top": 0.25,
              "two_segments_dense_top": 0.25}


def block_inputs(cfg):
    x, w1, w_dw, w3 = synth.make_block_inputs(cfg)
    if cfg.name in ZERO_BELOW:
        x[:, :, int(cfg.H * ZERO_BELOW[cfg.name]):, :] = 0.0
    return x, w1, w_dw, w3


@pytest.fixture(scope="module")
def ctx():
    c = wcc.Context(0)
    yield c
    c.close()


def draw_chained(seed: int) -> synth.BlockCfg:
    """A random block of a shape the chained route may take: every level count, widths of one,
    two and four wave rows with an accent on the ones around the seams (a last segment of one
    or two lanes, one lane short of full), 1-3 samples, every weight type."""
    rng = np.random.default_rng(9000 + seed)
    d = int(rng.choice([1, 2, 3, 3]))
    s = max(1 << d, 4)
    kind = int(rng.integers(0, 5))
    if kind == 0:
        W = int(rng.integers(2, 65)) * 4          # up to 256
    elif kind == 1:
        W = int(rng.integers(65, 129)) * 4        # two wave rows
    elif kind == 2:
        W = int(rng.integers(193, 257)) * 4       # four wave rows
    elif kind == 3:
        W = int(rng.choice([260, 264, 772, 776, 508, 1020, 252, 132, 36]))
    else:
        W = int(rng.choice([64, 96, 128, 256, 512, 1024]))
    W = max(s, (W // s) * s)
    H = int(rng.integers(1, 13)) * (1 << d)
    wd = int(rng.choice([F32, BF16, BF16, I8]))
    bits = 0 if (wd == F32 and rng.random() < 0.5) else 8
    return blk(f"rand{seed}", int(rng.integers(1, 4)), int(rng.choice([2, 4, 8, 16, 32])),
               int(rng.choice([2, 3, 4, 8])), H, W, d, 1, int(rng.choice([3, 4, 5, 8, 16, 40])), wd, bits,
               float(rng.choice([1.0, 2.0, 3.0])))


@pytest.mark.parametrize("cfg", CASES + [draw_chained(s) for s in range(60)], ids=lambda c: c.name)
def test_chained_block_matches_oracle_and_materialised_route(ref, ctx, cfg):
    print(f"{cfg}", flush=True)
    x, w1, w_dw, w3 = block_inputs(cfg)
    d = wcc.make_block_desc(cfg.B, cfg.C, cfg.expansion, cfg.H, cfg.W, cfg.levels, cfg.keep_num,
                            cfg.keep_den, cfg.w_dtype, cfg.act_bits)
    if cfg.name.startswith("rand") and not wcc.block_is_chained(d):
        pytest.skip("a random shape the chained route does not take (3 k > N, or three wave rows)")
    assert wcc.block_is_chained(d)
    ctx.ensure_workspace(d)
    xd = dev(x)
    w1d, w1s = upload_weights(w1)
    w3d, w3s = upload_weights(w3)
    wdd = dev(w_dw)
    mid = (cfg.B, cfg.C_mid, cfg.H, cfg.W)
    y = torch.full(x.shape, float("nan"), dtype=torch.float32, device="cuda")
    t1 = torch.full(mid, float("nan"), dtype=torch.float32, device="cuda")
    t2 = torch.full(mid, float("nan"), dtype=torch.float32, device="cuda")
    idx1 = torch.empty((cfg.B, cfg.k), dtype=torch.int32, device="cuda")
    idx3 = torch.empty((cfg.B, cfg.k), dtype=torch.int32, device="cuda")
    # the route that forms the middle tensors, held to the oracle first
    ctx.wcc_block_forward(d, xd, w1d, w1s, wdd, w3d, w3s, y, t1, t2, idx1, idx3)
    torch.cuda.synchronize()
    tol = 1e-5 if (cfg.w_dtype == F32 and cfg.act_bits == 0) else 1e-2
    o_t1, o_idx1, _ = ref.forward(x, w1.values, w1.scale, cfg.levels, cfg.keep_num, cfg.keep_den,
                                  act_bits=cfg.act_bits)
    np.testing.assert_array_equal(idx1.cpu().numpy().astype(np.int64), o_idx1)
    g_t1, g_t2 = t1.cpu().numpy(), t2.cpu().numpy()
    assert rel_l2(g_t1, o_t1) <= tol
    assert rel_l2(g_t2, ref.depthwise3x3(g_t1, w_dw)) <= 1e-6
    g_idx3 = idx3.cpu().numpy().astype(np.int64)
    want_branch, norm = layer_with_index_set(ref, cfg.layer(1), w3, g_t2.astype(np.float64), g_idx3)
    for b in range(cfg.B):
        assert_valid_index_set(norm[b], g_idx3[b], cfg.k)
    assert rel_l2(y.cpu().numpy().astype(np.float64) - x, want_branch) <= tol
    # the chained call: first index set exact, second one valid, output against the oracle
    idx1_c = torch.full_like(idx1, -7)
    y_c = torch.full_like(y, float("nan"))
    ctx.wcc_block_forward(d, xd, w1d, w1s, wdd, w3d, w3s, y_c, None, None, idx1_c, None)
    torch.cuda.synchronize()
    assert torch.equal(idx1_c, idx1)
    same = check_block_without_middle_outputs(ref, ctx, cfg, d, xd, x.astype(np.float64), w1d, w1s, wdd,
                                              w3d, w3s, w3, g_t2, y, idx3, tol)
    print(f"  second index set {'equal: outputs equal bit for bit' if same else 'differs: both valid'}",
          flush=True)
    # run to run: the chained call gives the same bits again
    y_c2 = torch.full_like(y, float("nan"))
    ctx.wcc_block_forward(d, xd, w1d, w1s, wdd, w3d, w3s, y_c2)
    torch.cuda.synchronize()
    assert torch.equal(y_c, y_c2)


@pytest.mark.parametrize("cfg", [CASES[0], CASES[1], CASES[3], CASES[6]], ids=lambda c: c.name)
def test_chained_block_with_bf16_maps(ctx, cfg):
    """x and y stored as bf16.  Chained, the middle tensors are never stored, so storage is all
    that differs from the chained call with fp32 maps on the same bf16-valued input: the same index
    sets, and that call's output rounded once to nearest even.  (The fp32 call is the one held
    to the oracle above.)"""
    x, w1, w_dw, w3 = block_inputs(cfg)
    x = synth.round_to_bf16(x)
    w1d, w1s = upload_weights(w1)
    w3d, w3s = upload_weights(w3)
    wdd = dev(w_dw)
    out = {}
    for act, tdt in ((wcc.F32, torch.float32), (wcc.BF16, torch.bfloat16)):
        d = wcc.make_block_desc(cfg.B, cfg.C, cfg.expansion, cfg.H, cfg.W, cfg.levels, cfg.keep_num,
                                cfg.keep_den, cfg.w_dtype, cfg.act_bits, act)
        ctx.ensure_workspace(d)
        xd = dev(x).to(tdt)
        y = torch.full(x.shape, float("nan"), dtype=tdt, device="cuda")
        idx1 = torch.full((cfg.B, cfg.k), -7, dtype=torch.int32, device="cuda")
        idx3 = torch.full((cfg.B, cfg.k), -7, dtype=torch.int32, device="cuda")
        ctx.wcc_block_forward(d, xd, w1d, w1s, wdd, w3d, w3s, y, None, None, idx1, idx3)
        torch.cuda.synchronize()
        out[act] = (y, idx1, idx3)
    y32, i1, i3 = out[wcc.F32]
    y16, j1, j3 = out[wcc.BF16]
    assert torch.equal(i1, j1) and torch.equal(i3, j3)
    want_bits = synth._round_to_bf16_bits(y32.cpu().numpy())
    np.testing.assert_array_equal(y16.view(torch.int16).cpu().numpy().view(np.uint16), want_bits)
