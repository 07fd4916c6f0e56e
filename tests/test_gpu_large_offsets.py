"""Tensors of more than 2**31 elements (9.1 GB each): every element offset of the strip kernels,
the contraction and the staged calls has to be formed in 64 bits.

68 samples of 16 x 1024 x 2048.  The samples are independent once the clipping parameter is
handed in (Alg. 1 is per image; the quantiser then needs no maximum over the call), so the
oracle follows single samples: the first, the ones on either side of byte offset 2**32 and of
element offset 2**31, and the last.  Every sample is a channel rotation and a mirror image of
one generated base sample (exact operations, done with torch on the device and with numpy for
the oracle); a rotation of the channels leaves the exact L1 norms alone, so the index sets of
ALL samples are also checked against those of the four mirror classes.
"""
import numpy as np
import pytest
import torch

from paper_2205_12268_amd import synth, wcc
from tests.util import dev, rel_l2, upload_weights

pytestmark = pytest.mark.gpu

B, C, H, W, LEVELS = 68, 16, 1024, 2048, 3
KEEP = (1, 8)
ALPHA_IN = 3.0          # below the largest kept coefficient: clipping is live
SAMPLED = (0, 31, 32, 63, 64, 67)


def variant_np(base, b):
    v = np.roll(base, b % C, axis=0)
    if b & 1:
        v = v[:, ::-1, :]
    if b & 2:
        v = v[:, :, ::-1]
    return np.ascontiguousarray(v)


def variant_torch(base, b):
    v = torch.roll(base, b % C, 0)
    dims = [d for d, on in ((1, b & 1), (2, b & 2)) if on]
    return torch.flip(v, dims) if dims else v


def test_tensors_beyond_2_31_elements(ref):
    N = H * W
    cfg = synth.LayerCfg("large_offsets_base", 1, C, C, H, W, LEVELS, KEEP[0], KEEP[1],
                         synth.W_BF16, 8, sigma=3.0, clip_hi=8.0, seed=synth.SEED_BASE + 0xB10)
    k = cfg.k
    print("generating the base sample", flush=True)
    xb, w = synth.make_inputs(cfg)
    base_np = xb[0]
    assert variant_np(base_np, 5)[0, 0, 0] == base_np[(0 - 5) % C, H - 1, 0]  # rotation, then mirror
    base = dev(base_np)
    f32 = dict(dtype=torch.float32, device="cuda")
    x = torch.empty((B, C, H, W), **f32)
    for b in range(B):
        x[b] = variant_torch(base, b)
    assert x.numel() > 2 ** 31
    for b in (5, 66):  # the two recipes agree
        assert np.array_equal(x[b].cpu().numpy(), variant_np(base_np, b))

    d = wcc.make_desc(B, C, C, H, W, LEVELS, KEEP[0], KEEP[1], synth.W_BF16, 8)
    ctx = wcc.Context(0)
    ctx.ensure_workspace(d)
    wd, wsd = upload_weights(w)
    y = torch.full((B, C, H, W), float("nan"), **f32)
    idx = torch.full((B, k), -7, dtype=torch.int32, device="cuda")
    print("gpu forward", flush=True)
    ctx.wcc_forward(d, x, wd, wsd, ALPHA_IN, y, idx)
    torch.cuda.synchronize()

    print("gpu staged calls", flush=True)
    coef = torch.full((B, C, N), float("nan"), **f32)
    norm = torch.full((B, N), float("nan"), **f32)
    ctx.wcc_haar_fwd(d, x, coef, norm)
    idx_s = torch.full_like(idx, -7)
    ctx.wcc_joint_topk(d, None, norm, idx_s)
    assert torch.equal(idx_s, idx)
    xc = torch.zeros((B, C, k), dtype=torch.int8, device="cuda")
    alpha_dev = torch.zeros(1, **f32)
    ctx.wcc_gather_quant(d, coef, idx, ALPHA_IN, xc, alpha_dev)
    assert float(alpha_dev.item()) == ALPHA_IN
    yc = torch.full((B, C, k), float("nan"), **f32)
    ctx.wcc_pointwise(d, wd, wsd, xc, alpha_dev, yc)
    y_s = torch.full((B, C, H, W), float("nan"), **f32)
    ctx.wcc_scatter_ihaar(d, yc, idx, y_s)
    torch.cuda.synchronize()
    del yc, norm

    # all samples: a rotation of the channels changes no norm on the exact grid
    for b in range(4, B):
        assert torch.equal(idx[b], idx[b % 4]), b
    assert not torch.equal(idx[0], idx[1])  # (the mirror classes do differ)

    worst = 0.0
    for b in SAMPLED:
        print(f"oracle: sample {b}", flush=True)
        xs = variant_np(base_np, b)[None]
        o_y, o_idx, o_alpha = ref.forward(xs, w.values, w.scale, LEVELS, KEEP[0], KEEP[1],
                                          act_bits=8, alpha_in=ALPHA_IN)
        assert o_alpha == ALPHA_IN
        np.testing.assert_array_equal(idx[b].cpu().numpy().astype(np.int64), o_idx[0])
        o_coef = ref.haar_fwd(xs, LEVELS).reshape(C, N)
        np.testing.assert_array_equal(coef[b].cpu().numpy().astype(np.float64), o_coef)
        assert float(np.abs(o_coef[:, o_idx[0]]).max()) > ALPHA_IN       # some value does clip
        codes = ref.quant_codes(ref.gather(o_coef[None], o_idx), ALPHA_IN, 8)[0]
        np.testing.assert_array_equal(xc[b].cpu().numpy().astype(np.int64), codes.astype(np.int64))
        for got in (y[b], y_s[b]):
            err = rel_l2(got.cpu().numpy(), o_y[0])
            worst = max(worst, err)
            assert err <= 1e-2, (b, err)
    print(f"worst sample rel-L2 = {worst:.3e}", flush=True)
    ctx.close()


def test_block_with_middle_tensors_beyond_2_31_elements(ref):
    """The inverted residual block with 36 samples of 64 -> 256 -> 64 channels at 512 x 512:
    the two middle tensors hold 2.4e9 elements each, so the inverse of the first layer, the
    transform passes with K_dw folded in and the contraction over 256 channels form their
    offsets past 2**31.  No quantiser (with one, alpha would be a maximum over all samples):
    the samples are then independent and the oracle follows four of them."""
    Bb, Cb, E, Hb, Wb = 36, 64, 4, 512, 512
    sampled = (0, 16, 32, 35)
    cfg = synth.BlockCfg("large_offsets_block", 1, Cb, E, Hb, Wb, LEVELS, 1, 8, synth.W_BF16, 0,
                         sigma=3.0, seed=synth.SEED_BASE + 0xB20)
    k = cfg.k
    print("generating the base sample", flush=True)
    xb, w1, w_dw, w3 = synth.make_block_inputs(cfg)
    base_np = xb[0]

    def var_np(b):
        v = np.roll(base_np, b % Cb, axis=0)
        if b & 1:
            v = v[:, ::-1, :]
        if b & 2:
            v = v[:, :, ::-1]
        return np.ascontiguousarray(v)

    base = dev(base_np)
    f32 = dict(dtype=torch.float32, device="cuda")
    x = torch.empty((Bb, Cb, Hb, Wb), **f32)
    for b in range(Bb):
        v = torch.roll(base, b % Cb, 0)
        dims = [d for d, on in ((1, b & 1), (2, b & 2)) if on]
        x[b] = torch.flip(v, dims) if dims else v
    assert np.array_equal(x[35].cpu().numpy(), var_np(35))

    d = wcc.make_block_desc(Bb, Cb, E, Hb, Wb, LEVELS, 1, 8, synth.W_BF16, 0)
    ctx = wcc.Context(0)
    ctx.ensure_workspace(d)
    w1d, _ = upload_weights(w1)
    w3d, _ = upload_weights(w3)
    mid = (Bb, Cb * E, Hb, Wb)
    t1 = torch.full(mid, float("nan"), **f32)
    assert t1.numel() > 2 ** 31
    y = torch.full((Bb, Cb, Hb, Wb), float("nan"), **f32)
    idx1 = torch.full((Bb, k), -7, dtype=torch.int32, device="cuda")
    idx3 = torch.full((Bb, k), -7, dtype=torch.int32, device="cuda")
    print("gpu block forward", flush=True)
    ctx.wcc_block_forward(d, x, w1d, None, dev(w_dw), w3d, None, y, t1, None, idx1, idx3)
    torch.cuda.synchronize()
    for b in range(4, Bb):   # the first layer's norms do not see a rotation of the channels
        assert torch.equal(idx1[b], idx1[b % 4]), b

    worst = 0.0
    for b in sampled:
        print(f"oracle: sample {b}", flush=True)
        xs = var_np(b)[None]
        o_y, o_t1, _, o_idx1, o_idx3, _, _ = ref.block_forward(
            xs, w1.values, w1.scale, w_dw, w3.values, w3.scale, LEVELS, 1, 8, act_bits=0)
        np.testing.assert_array_equal(idx1[b].cpu().numpy().astype(np.int64), o_idx1[0])
        assert rel_l2(t1[b].cpu().numpy(), o_t1[0]) <= 1e-2
        # the second layer ranks norms of a tensor that carries fp32 rounding: a few positions
        # at the threshold may change places; the branch is compared as a whole
        moved = int(np.count_nonzero(idx3[b].cpu().numpy().astype(np.int64) != o_idx3[0]))
        err = rel_l2(y[b].cpu().numpy().astype(np.float64) - xs[0], o_y[0] - xs[0])
        worst = max(worst, err)
        print(f"  rel-L2(branch) = {err:.3e}; {moved} of {k} list entries differ", flush=True)
        assert err <= 1e-2
    print(f"worst sample rel-L2 = {worst:.3e}", flush=True)
    ctx.close()
