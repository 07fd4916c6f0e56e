"""Seeded random small layers: every mix of level count, width class (narrow planes packed
several strips a wave, rows wider than a wave, widths that are not a multiple of 4), channel
counts that do and do not fit the matrix-core tiles, keep ratios from almost nothing to
everything, weight types and quantiser on/off -- each against the oracle through wcc_forward;
and a second family of wide planes at keep ratios around one half and above."""
from __future__ import annotations

import numpy as np
import pytest
import torch

from paper_2205_12268_amd import synth, wcc
from tests.util import assert_valid_index_set, check_block_without_middle_outputs, layer_with_index_set, desc_of, dev, rel_l2, tol_for, upload_weights

pytestmark = pytest.mark.gpu


def draw(seed: int) -> synth.LayerCfg:
    rng = np.random.default_rng(1000 + seed)
    d = int(rng.integers(1, 5))
    s = 1 << d
    H = s * int(rng.integers(1, max(2, 48 // s)))
    wide = rng.random() < 0.3
    W = s * int(rng.integers(1, (640 if wide else 160) // s + 1))
    if d == 1 and rng.random() < 0.5:
        W += 2 * int(rng.integers(0, 2))                      # W % 4 == 2 now and then
    dt = int(rng.choice([synth.W_F32, synth.W_BF16, synth.W_I8, synth.W_I4]))
    Ci = int(rng.choice([2, 6, 8, 16, 24, 32, 48, 64, 80]))
    Co = int(rng.choice([1, 3, 8, 20, 32, 64, 96, 130]))
    den = int(rng.choice([1, 2, 3, 4, 7, 8, 16, 50]))
    num = int(rng.integers(1, den + 1))
    bits = 0 if dt == synth.W_F32 and rng.random() < 0.5 else int(rng.choice([0, 8, 8]))
    return synth.LayerCfg(f"rand{seed}", int(rng.integers(1, 4)), Ci, Co, H, W, d, num, den, dt, bits,
                          sigma=float(rng.choice([0.0, 1.0, 2.5])), clip_hi=8.0,
                          seed=synth.SEED_BASE + 0x900 + seed)


@pytest.fixture(scope="module")
def ctx():
    c = wcc.Context(0)
    yield c
    c.close()


@pytest.mark.parametrize("seed", range(32))
def test_random_layer(ref, ctx, seed):
    cfg = draw(seed)
    print(f"{cfg}", flush=True)
    x, w = synth.make_inputs(cfg)
    d = desc_of(cfg)
    ctx.ensure_workspace(d)
    wd, wsd = upload_weights(w)
    y = torch.full((cfg.B, cfg.C_out, cfg.H, cfg.W), float("nan"), dtype=torch.float32, device="cuda")
    idx = torch.full((cfg.B, cfg.k), -7, dtype=torch.int32, device="cuda")
    alpha = torch.zeros(1, dtype=torch.float32, device="cuda")
    ctx.wcc_forward(d, dev(x), wd, wsd, 0.0, y, idx, alpha)
    want, o_idx, o_alpha = ref.forward(x, w.values, w.scale, cfg.levels, cfg.keep_num, cfg.keep_den,
                                       act_bits=cfg.act_bits)
    np.testing.assert_array_equal(idx.cpu().numpy().astype(np.int64), o_idx)
    if cfg.act_bits:
        assert float(alpha.item()) == o_alpha
    got = y.cpu().numpy()
    assert np.isfinite(got).all()
    assert rel_l2(got, want) <= tol_for(cfg)


def draw_dense(seed: int) -> synth.LayerCfg:
    """Wide planes at keep ratios around and above one half: strips near and beyond what the
    packed position lists of the keep pass and of the inverse hold."""
    rng = np.random.default_rng(5000 + seed)
    d = int(rng.choice([2, 3, 3]))
    s = 1 << d
    H = s * int(rng.integers(1, 5))
    W = (int(rng.choice([256, 264, 320, 512, 520, 768, 1024, 136, 72, 1032])) // s) * s
    num, den = [(1, 2), (5, 8), (3, 4), (7, 8), (1, 1), (3, 8), (1, 4), (9, 16), (17, 32),
                (15, 32)][int(rng.integers(0, 10))]
    dt = int(rng.choice([synth.W_F32, synth.W_BF16, synth.W_I8, synth.W_I4]))
    bits = 0 if dt == synth.W_F32 and rng.random() < 0.5 else int(rng.choice([0, 8, 8]))
    return synth.LayerCfg(f"dense{seed}", int(rng.integers(1, 3)), int(rng.choice([4, 8, 16])),
                          int(rng.choice([4, 8, 20])), H, W, d, num, den, dt, bits,
                          sigma=float(rng.choice([0.0, 1.0, 2.5])), clip_hi=8.0,
                          seed=synth.SEED_BASE + 0xB00 + seed)


@pytest.mark.parametrize("seed", range(24))
def test_random_dense_layer(ref, ctx, seed):
    cfg = draw_dense(seed)
    print(f"{cfg}", flush=True)
    x, w = synth.make_inputs(cfg)
    d = desc_of(cfg)
    ctx.ensure_workspace(d)
    wd, wsd = upload_weights(w)
    y = torch.full((cfg.B, cfg.C_out, cfg.H, cfg.W), float("nan"), dtype=torch.float32, device="cuda")
    idx = torch.full((cfg.B, cfg.k), -7, dtype=torch.int32, device="cuda")
    alpha = torch.zeros(1, dtype=torch.float32, device="cuda")
    a_in = 3.0 if (cfg.act_bits and seed % 3 == 0) else 0.0   # every third one with a caller's alpha
    ctx.wcc_forward(d, dev(x), wd, wsd, a_in, y, idx, alpha)
    want, o_idx, o_alpha = ref.forward(x, w.values, w.scale, cfg.levels, cfg.keep_num, cfg.keep_den,
                                       act_bits=cfg.act_bits, alpha_in=a_in)
    np.testing.assert_array_equal(idx.cpu().numpy().astype(np.int64), o_idx)
    if cfg.act_bits:
        assert float(alpha.item()) == o_alpha
    assert rel_l2(y.cpu().numpy(), want) <= tol_for(cfg)


def draw_block(seed: int) -> synth.BlockCfg:
    rng = np.random.default_rng(2000 + seed)
    d = int(rng.integers(1, 4))
    s = 1 << d
    H = s * int(rng.integers(1, max(2, 40 // s)))
    W = s * int(rng.integers(1, (560 if rng.random() < 0.4 else 128) // s + 1))
    dt = int(rng.choice([synth.W_F32, synth.W_BF16, synth.W_I8, synth.W_I4]))
    den = int(rng.choice([1, 2, 4, 8, 5]))
    bits = 0 if dt == synth.W_F32 else 8
    return synth.BlockCfg(f"randblk{seed}", int(rng.integers(1, 3)), int(rng.choice([2, 4, 8, 16])),
                          int(rng.integers(1, 5)), H, W, d, int(rng.integers(1, den + 1)), den, dt, bits,
                          sigma=float(rng.choice([1.0, 2.0])), seed=synth.SEED_BASE + 0xA00 + seed)


@pytest.mark.parametrize("seed", range(12))
def test_random_block(ref, ctx, seed):
    """x + WCC(K3, K_dw(WCC(K1, x))) on a random block.  The first layer sees dyadic inputs: its
    index set is the oracle's, bit for bit, and its output is within the tolerance.  The second
    layer's input is not dyadic, so fp32 and fp64 norms may order two nearly equal positions
    differently and several index sets are correct: the GPU's set is checked for validity
    against the oracle's fp64 norms of the GPU's own K_dw output, and the block's output is
    held to the tolerance against the oracle run on that set.  The independent oracle chain
    (its own sets throughout) is printed as a diagnostic and asserted where the sets agree."""
    cfg = draw_block(seed)
    print(f"{cfg}", flush=True)
    x, w1, w_dw, w3 = synth.make_block_inputs(cfg)
    d = wcc.make_block_desc(cfg.B, cfg.C, cfg.expansion, cfg.H, cfg.W, cfg.levels, cfg.keep_num,
                            cfg.keep_den, cfg.w_dtype, cfg.act_bits)
    ctx.ensure_workspace(d)
    w1d, w1s = upload_weights(w1)
    w3d, w3s = upload_weights(w3)
    mid = (cfg.B, cfg.C_mid, cfg.H, cfg.W)
    y = torch.full(x.shape, float("nan"), dtype=torch.float32, device="cuda")
    t1 = torch.full(mid, float("nan"), dtype=torch.float32, device="cuda")
    t2 = torch.full(mid, float("nan"), dtype=torch.float32, device="cuda")
    idx1 = torch.empty((cfg.B, cfg.k), dtype=torch.int32, device="cuda")
    idx3 = torch.empty((cfg.B, cfg.k), dtype=torch.int32, device="cuda")
    ctx.wcc_block_forward(d, dev(x), w1d, w1s, dev(w_dw), w3d, w3s, y, t1, t2, idx1, idx3)
    torch.cuda.synchronize()
    tol = 1e-5 if (cfg.w_dtype == synth.W_F32 and cfg.act_bits == 0) else 1e-2
    o = ref.block_forward(x, w1.values, w1.scale, w_dw, w3.values, w3.scale, cfg.levels,
                          cfg.keep_num, cfg.keep_den, cfg.act_bits)
    np.testing.assert_array_equal(idx1.cpu().numpy().astype(np.int64), o[3])
    g_t1, g_t2 = t1.cpu().numpy(), t2.cpu().numpy()
    assert rel_l2(g_t1, o[1]) <= tol
    assert rel_l2(g_t2, ref.depthwise3x3(g_t1, w_dw)) <= 1e-6
    g_idx3 = idx3.cpu().numpy().astype(np.int64)
    want_branch, norm = layer_with_index_set(ref, cfg.layer(1), w3, g_t2.astype(np.float64), g_idx3)
    for b in range(cfg.B):
        assert_valid_index_set(norm[b], g_idx3[b], cfg.k)
    got = y.cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all()
    assert rel_l2(got - x, want_branch) <= tol
    err = rel_l2(got - x, o[0] - x)
    same = np.array_equal(g_idx3, o[4])
    print(f"  end-to-end rel-L2 of the branch = {err:.3e} (second index set "
          f"{'equal' if same else 'differs'})", flush=True)
    if same:
        assert err <= tol
    # the same block without the test outputs (chained in the compressed domain where the shape
    # allows, else K_dw folded into the transform or a kernel of its own)
    check_block_without_middle_outputs(ref, ctx, cfg, d, dev(x), x.astype(np.float64), w1d, w1s,
                                       dev(w_dw), w3d, w3s, w3, g_t2, y, idx3, tol)
