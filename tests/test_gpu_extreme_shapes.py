"""Shapes at the corners of what the descriptor allows, fused layer against the oracle: many
samples of a few pixels, thousands of channels on a tiny plane, planes one strip wide or one
strip tall, the smallest plane there is, k = 1 and k = N - 1 at four levels, widths that are
not a multiple of four, small planes with thousands of channels.  Index sets and alpha bit for bit, output to the usual tolerance.
"""
import numpy as np
import pytest
import torch

from paper_2205_12268_amd import synth, wcc
from tests.util import desc_of, dev, rel_l2, tol_for, upload_weights

pytestmark = pytest.mark.gpu

F32, BF16, I8, I4 = synth.W_F32, synth.W_BF16, synth.W_I8, synth.W_I4

SHAPES = [
    # B, C_in, C_out, H, W, levels, keep num, keep den, weights, activation bits
    (300, 4, 4, 8, 8, 1, 1, 2, BF16, 8),          # many samples
    (513, 8, 8, 4, 4, 1, 1, 4, F32, 0),
    (64, 16, 8, 16, 16, 2, 1, 4, I8, 8),
    (1, 2048, 8, 8, 16, 1, 1, 2, BF16, 8),        # many input channels
    (1, 8, 1500, 8, 16, 2, 1, 4, BF16, 8),        # many output channels
    (2, 1024, 1024, 8, 8, 3, 1, 4, I8, 8),        # the plane is one coarse coefficient
    (1, 4, 4, 2048, 8, 3, 1, 8, BF16, 8),         # tall and one strip wide
    (1, 4, 4, 8, 4096, 3, 1, 8, BF16, 8),         # one strip tall
    (1, 4, 4, 2, 2, 1, 1, 1, F32, 0),             # the smallest plane
    (1, 1, 1, 2, 2, 1, 1, 4, F32, 0),             # one channel, k = 1
    (1, 1, 1, 16, 16, 4, 1, 256, BF16, 8),        # k = 1 at four levels
    (2, 3, 5, 16, 16, 4, 255, 256, F32, 0),       # k = N - 1
    (1, 8, 8, 4096, 4, 2, 1, 2, I4, 8),           # one vector wide
    (3, 40, 72, 24, 24, 3, 2, 3, I4, 8),
    (1, 64, 64, 128, 1024, 1, 1, 2, BF16, 8),
    (1, 16, 16, 1024, 128, 4, 1, 16, I8, 8),
    (2, 8, 8, 16, 2048, 4, 1, 2, BF16, 8),
    (1, 8, 8, 6, 6, 1, 1, 3, BF16, 8),            # W % 4 != 0
    (1, 8, 8, 2, 1026, 1, 1, 2, BF16, 8),         # W % 4 != 0 over several segments
    (5, 8, 8, 2, 1026, 1, 2, 2, F32, 8),
    # small planes (one-workgroup selection) with millions of kept coefficients: the clipping
    # parameter is then found before the second pass (int8 codes through memory), unlike on the
    # small layers above
    (8, 512, 64, 64, 64, 3, 1, 4, BF16, 8),
    (2, 2048, 32, 96, 96, 3, 1, 2, I8, 8),        # partial planes combined before the selection
    (4, 1024, 16, 128, 128, 2, 1, 4, BF16, 8),    # the largest plane the one-workgroup selection takes
]


@pytest.fixture(scope="module")
def ctx():
    c = wcc.Context(0)
    yield c
    c.close()


@pytest.mark.parametrize("i", range(len(SHAPES)))
def test_extreme_shape(ref, ctx, i):
    B, Ci, Co, H, W, d, num, den, wd, bits = SHAPES[i]
    cfg = synth.LayerCfg(f"extreme{i}", B, Ci, Co, H, W, d, num, den, wd, bits, sigma=1.0,
                         clip_hi=8.0, seed=synth.SEED_BASE + 0xE00 + i)
    print(f"case {i}: {SHAPES[i]} k = {cfg.k} seed {cfg.seed:#x}", flush=True)
    x, w = synth.make_inputs(cfg, check=False)
    try:
        synth.assert_exact_budget(x, d)
    except AssertionError:
        # thousands of channels: a coarser grid keeps every L1 sum exact in fp32
        x = (np.floor(x * 4) / 4).astype(np.float32) * np.float32(0.25)
        synth.assert_exact_budget(x, d)
    dd = desc_of(cfg)
    ctx.ensure_workspace(dd)
    wdev, wsd = upload_weights(w)
    y = torch.full((B, Co, H, W), float("nan"), dtype=torch.float32, device="cuda")
    idx = torch.full((B, cfg.k), -7, dtype=torch.int32, device="cuda")
    alpha = torch.zeros(1, dtype=torch.float32, device="cuda")
    ctx.wcc_forward(dd, dev(x), wdev, wsd, 0.0, y, idx, alpha)
    want, o_idx, o_alpha = ref.forward(x, w.values, w.scale, d, num, den, act_bits=bits)
    np.testing.assert_array_equal(idx.cpu().numpy().astype(np.int64), o_idx)
    if bits:
        assert float(alpha.item()) == o_alpha
    err = rel_l2(y.cpu().numpy(), want)
    print(f"  rel-L2(y) = {err:.3e}", flush=True)
    assert err <= tol_for(cfg)
