"""Feature maps stored as bf16 (act_dtype = WCC_BF16): read exactly, written rounded to nearest
even, arithmetic unchanged.  Checked two ways: against the oracle on the same (bf16-valued)
input, and bit for bit against the fp32-output run of the same layer rounded on the host."""
from __future__ import annotations

import numpy as np
import pytest
import torch

from paper_2205_12268_amd import synth, wcc
from tests.test_gpu_parity import SMALL
from tests.util import dev, rel_l2, upload_weights

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    c = wcc.Context(0)
    yield c
    c.close()


def desc(cfg, act):
    return wcc.make_desc(cfg.B, cfg.C_in, cfg.C_out, cfg.H, cfg.W, cfg.levels, cfg.keep_num,
                         cfg.keep_den, cfg.w_dtype, cfg.act_bits, act)


@pytest.mark.parametrize("cfg", SMALL, ids=lambda c: c.name)
def test_bf16_feature_maps(ref, ctx, cfg):
    x, w = synth.make_inputs(cfg)
    x = synth.round_to_bf16(x)               # what a bf16 tensor can hold
    wd, wsd = upload_weights(w)
    shape = (cfg.B, cfg.C_out, cfg.H, cfg.W)
    # fp32 storage
    d32 = desc(cfg, wcc.F32)
    ctx.ensure_workspace(d32)
    y32 = torch.empty(shape, dtype=torch.float32, device="cuda")
    i32 = torch.empty((cfg.B, cfg.k), dtype=torch.int32, device="cuda")
    ctx.wcc_forward(d32, dev(x), wd, wsd, 0.0, y32, i32)
    # bf16 storage of the same numbers
    d16 = desc(cfg, wcc.BF16)
    ctx.ensure_workspace(d16)
    xb = torch.from_numpy(x).cuda().to(torch.bfloat16)
    assert torch.equal(xb.float().cpu(), torch.from_numpy(x))
    y16 = torch.full(shape, float("nan"), dtype=torch.bfloat16, device="cuda")
    i16 = torch.empty((cfg.B, cfg.k), dtype=torch.int32, device="cuda")
    a16 = torch.zeros(1, dtype=torch.float32, device="cuda")
    ctx.wcc_forward(d16, xb, wd, wsd, 0.0, y16, i16, a16)
    torch.cuda.synchronize()
    assert torch.equal(i16, i32)
    want_bits = synth._round_to_bf16_bits(y32.cpu().numpy())          # host rounding, RNE
    got_bits = y16.view(torch.int16).cpu().numpy().view(np.uint16)
    np.testing.assert_array_equal(got_bits, want_bits)
    # and the oracle on the same input
    o_y, o_idx, o_alpha = ref.forward(x, w.values, w.scale, cfg.levels, cfg.keep_num, cfg.keep_den,
                                      act_bits=cfg.act_bits)
    np.testing.assert_array_equal(i16.cpu().numpy().astype(np.int64), o_idx)
    if cfg.act_bits:
        assert float(a16.item()) == o_alpha
    assert rel_l2(y16.float().cpu().numpy(), o_y) <= 1e-2
    # the variants that share the kernels
    y16b = torch.full(shape, float("nan"), dtype=torch.bfloat16, device="cuda")
    ctx.wcc_forward_fixed(d16, xb, wd, wsd, 0.0, i16, y16b)
    assert torch.equal(y16b.view(torch.int16), y16.view(torch.int16))


def test_stage_calls_refuse_bf16(ctx):
    d = wcc.make_desc(1, 8, 8, 16, 16, 2, 1, 4, wcc.BF16, 8, wcc.BF16)
    ctx.ensure_workspace(d)
    x = torch.zeros((1, 8, 16, 16), dtype=torch.bfloat16, device="cuda")
    coef = torch.zeros((1, 8, 256), device="cuda")
    with pytest.raises(wcc.WccError) as e:
        ctx.wcc_haar_fwd(d, x, coef)
    assert e.value.status == 6
    with pytest.raises(wcc.WccError) as e:
        wcc.workspace_bytes(wcc.make_desc(1, 8, 8, 16, 16, 2, 1, 4, wcc.BF16, 8, 2))
    assert e.value.status == 3


@pytest.mark.parametrize("cfg", [
    synth.BlockCfg("blk16_d2", 2, 16, 4, 32, 64, 2, 1, 4, synth.W_BF16, 8, sigma=2.0, seed=synth.SEED_BASE + 0xB10),
    synth.BlockCfg("blk16_wide_d1", 1, 8, 2, 8, 1024, 1, 1, 2, synth.W_I8, 8, sigma=2.0, seed=synth.SEED_BASE + 0xB11),
    synth.BlockCfg("blk16_d3", 1, 8, 3, 64, 256, 3, 1, 8, synth.W_BF16, 8, sigma=3.0, seed=synth.SEED_BASE + 0xB12),
], ids=lambda c: c.name)
def test_bf16_block(ref, ctx, cfg):
    """The block with x, y and the middle tensor in bf16.  Stage by stage on the GPU's own
    middle tensor (the oracle rounds nothing: it is fed what the GPU stored)."""
    x, w1, w_dw, w3 = synth.make_block_inputs(cfg)
    x = synth.round_to_bf16(x)
    l0, l1 = cfg.layer(0), cfg.layer(1)
    d = wcc.make_block_desc(cfg.B, cfg.C, cfg.expansion, cfg.H, cfg.W, cfg.levels, cfg.keep_num,
                            cfg.keep_den, cfg.w_dtype, cfg.act_bits, wcc.BF16)
    ctx.ensure_workspace(d)
    w1d, w1s = upload_weights(w1)
    w3d, w3s = upload_weights(w3)
    xb = torch.from_numpy(x).cuda().to(torch.bfloat16)
    t1 = torch.empty((cfg.B, cfg.C_mid, cfg.H, cfg.W), dtype=torch.bfloat16, device="cuda")
    y = torch.full(x.shape, float("nan"), dtype=torch.bfloat16, device="cuda")
    idx1 = torch.empty((cfg.B, cfg.k), dtype=torch.int32, device="cuda")
    idx3 = torch.empty((cfg.B, cfg.k), dtype=torch.int32, device="cuda")
    ctx.wcc_block_forward(d, xb, w1d, w1s, dev(w_dw), w3d, w3s, y, t1, None, idx1, idx3)
    torch.cuda.synchronize()
    o_t1, o_idx1, _ = ref.forward(x, w1.values, w1.scale, cfg.levels, cfg.keep_num, cfg.keep_den,
                                  act_bits=cfg.act_bits)
    np.testing.assert_array_equal(idx1.cpu().numpy().astype(np.int64), o_idx1)
    g_t1 = t1.float().cpu().numpy()
    assert rel_l2(g_t1, o_t1) <= 1e-2
    # second layer on what the GPU stored: K_dw, a valid index set, the output for that set
    t2 = ref.depthwise3x3(g_t1, w_dw)
    g_idx3 = idx3.cpu().numpy().astype(np.int64)
    want, _ = ref.forward_with_list(t2, w3.values, w3.scale, cfg.levels, g_idx3, cfg.act_bits)
    coef = ref.haar_fwd(t2, cfg.levels).reshape(cfg.B, cfg.C_mid, cfg.N)
    norm = ref.channel_norm(coef)
    for b in range(cfg.B):
        kth = np.sort(norm[b])[::-1][cfg.k - 1]
        dropped = np.ones(cfg.N, dtype=bool)
        dropped[g_idx3[b]] = False
        assert norm[b][g_idx3[b]].min() >= kth * (1 - 1e-5)
        assert (not dropped.any()) or norm[b][dropped].max() <= kth * (1 + 1e-5)
    got = y.float().cpu().numpy().astype(np.float64)
    assert rel_l2(got, x + want) <= 1e-2
    with pytest.raises(wcc.WccError) as e:   # K_dw's output is not available in bf16
        ctx.wcc_block_forward(d, xb, w1d, w1s, dev(w_dw), w3d, w3s, y, t1,
                              torch.empty((cfg.B, cfg.C_mid, cfg.H, cfg.W), device="cuda"))
    assert e.value.status == 6
