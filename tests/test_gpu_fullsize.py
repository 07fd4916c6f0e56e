"""The single-layer workloads at their full sizes, in the launch configuration bench.py times.

The oracle runs the cheap stages in full (transform, norms, selection, gather, quantiser,
contraction) so index sets and alpha are compared exactly, and the last stage (zero filling +
inverse transform) plane by plane in chunks, so the whole output is compared element by element.
"""
import numpy as np
import pytest
import torch

from paper_2205_12268_amd import synth, wcc
from tests.util import dev, oracle_scale, rel_l2, tol_for, upload_weights

pytestmark = pytest.mark.gpu


def _huge_plane():
    """More than 2**20 kept positions per sample: the packed (rank | cell) lists of the strip
    kernels do not apply, 4096 select workgroups per sample, a one-chunk contraction."""
    return synth.small(synth.config(2), name="huge_plane", B=1, C_in=8, C_out=16, H=2048, W=2048,
                       levels=2, keep_num=1, keep_den=2, seed=synth.SEED_BASE + 0x800)


@pytest.mark.parametrize("n,norm", [(2, "l1"), (3, "l1"), (4, "l1"), ("huge_plane", "l1"),
                                    (2, "l2"), (3, "l2"), (4, "l2")])
def test_full_size_forward(ref, n, norm):
    """norm = "l2" (bench.py --norm l2): sums of squares round in fp32, so the index sets are
    checked for validity against the oracle's fp64 norms and the oracle then follows the
    GPU's sets; with the L1 norm they are the oracle's own, bit for bit."""
    cfg = _huge_plane() if n == "huge_plane" else synth.config(n)
    n = 9 if n == "huge_plane" else n
    print(f"workload {cfg.name}, {norm} norm: generating inputs", flush=True)
    x, w = synth.make_inputs(cfg)
    d = wcc.make_desc(cfg.B, cfg.C_in, cfg.C_out, cfg.H, cfg.W, cfg.levels, cfg.keep_num,
                      cfg.keep_den, cfg.w_dtype, cfg.act_bits, wcc.F32,
                      wcc.NORM_L2 if norm == "l2" else wcc.NORM_L1)
    N, k = cfg.N, cfg.k
    ctx = wcc.Context(0)
    ctx.ensure_workspace(d)
    xd = dev(x)
    wd, wsd = upload_weights(w)
    y = torch.empty((cfg.B, cfg.C_out, cfg.H, cfg.W), dtype=torch.float32, device="cuda")
    idx = torch.full((cfg.B, k), -7, dtype=torch.int32, device="cuda")
    alpha = torch.zeros(1, dtype=torch.float32, device="cuda")
    print("  gpu forward", flush=True)
    ctx.wcc_forward(d, xd, wd, wsd, 0.0, y, idx, alpha)
    torch.cuda.synchronize()
    # run to run reproducibility of everything
    y2 = torch.empty_like(y)
    idx2 = torch.empty_like(idx)
    ctx.wcc_forward(d, xd, wd, wsd, 0.0, y2, idx2, None)
    assert torch.equal(idx, idx2) and torch.equal(y, y2)
    if cfg.act_bits:
        # the same alpha handed in by the caller: the keep pass decides the codes itself (int8
        # leaves the chip); same codes, so the same output bit for bit
        y2.fill_(float("nan"))
        ctx.wcc_forward(d, xd, wd, wsd, float(alpha.item()), y2, idx2, None)
        assert torch.equal(idx, idx2) and torch.equal(y, y2)
    # the selected list handed back in as a caller's list: the same kernels after the select,
    # so the same output bit for bit; and the first-k list against the same list given explicitly
    ctx.wcc_forward_fixed(d, xd, wd, wsd, 0.0, idx, y2, None)
    assert torch.equal(y, y2)
    if norm == "l1" and n != 9:
        y3 = torch.full_like(y, float("nan"))
        ctx.wcc_forward_fixed(d, xd, wd, wsd, 0.0, None, y2, None)
        first_k = torch.arange(k, dtype=torch.int32, device="cuda").repeat(cfg.B, 1).contiguous()
        ctx.wcc_forward_fixed(d, xd, wd, wsd, 0.0, first_k, y3, None)
        assert torch.equal(y2, y3) and not torch.equal(y2, y)
        del y3, first_k
    del y2, idx2

    print("  oracle: transform, norms, selection", flush=True)
    coef = ref.haar_fwd(x, cfg.levels).reshape(cfg.B, cfg.C_in, N)
    o_norm = ref.channel_norm(coef, norm)
    g_idx = idx.cpu().numpy().astype(np.int64)
    if norm == "l1":
        o_idx = ref.topk(o_norm, k)
        np.testing.assert_array_equal(g_idx, o_idx)
    else:
        for b in range(cfg.B):
            sel = g_idx[b]
            assert np.all(np.diff(sel) > 0) and sel[0] >= 0 and sel[-1] < N
            kth = np.sort(o_norm[b])[::-1][k - 1]
            dropped = np.ones(N, dtype=bool)
            dropped[sel] = False
            assert o_norm[b][sel].min() >= kth * (1 - 1e-5)
            assert o_norm[b][dropped].max() <= kth * (1 + 1e-5)
        o_idx = g_idx
    del o_norm
    xc = ref.gather(coef, o_idx)
    del coef
    o_alpha = float(np.float32(ref.absmax(xc)))
    assert float(alpha.item()) == o_alpha
    print("  oracle: quantiser, contraction", flush=True)
    xhat = ref.quant_codes(xc, o_alpha, 8)
    del xc
    yc = ref.pointwise(w.values, oracle_scale(ref, cfg, w, o_alpha), xhat)
    del xhat
    print("  oracle: zero filling + inverse transform of every plane", flush=True)
    # all B * C_out planes, a few hundred at a time (the oracle's fp64 planes of one chunk take
    # about 1 GB): the relative L2 error of the whole output, and of the worst single plane
    tol = tol_for(cfg)
    chunk = max(1, min(cfg.C_out, (64 << 20) // N))
    num = den = 0.0
    worst = 0.0
    for b in range(cfg.B):
        for o0 in range(0, cfg.C_out, chunk):
            o1 = min(cfg.C_out, o0 + chunk)
            z = ref.scatter(yc[b:b + 1, o0:o1], o_idx[b:b + 1], N)
            want = ref.haar_inv(z, cfg.H, cfg.W, cfg.levels)[0]
            del z
            diff = y[b, o0:o1].cpu().numpy().astype(np.float64) - want
            e2 = np.einsum("chw,chw->c", diff, diff)
            w2 = np.einsum("chw,chw->c", want, want)
            del diff, want
            num += float(e2.sum())
            den += float(w2.sum())
            ok = w2 > 0
            if ok.any():
                worst = max(worst, float(np.sqrt(e2[ok] / w2[ok]).max()))
            assert np.all(e2[~ok] == 0.0)
        print(f"    sample {b}: done", flush=True)
    err = float(np.sqrt(num / den))
    print(f"  whole-output rel-L2 = {err:.3e}, worst plane {worst:.3e} (tol {tol:g})", flush=True)
    assert err <= tol and worst <= tol
    # a property that holds at any size: Parseval, ||y[b,o]||_2 == ||yc[b,o,:]||_2
    en_gpu = torch.linalg.vector_norm(y.double(), dim=(2, 3)).cpu().numpy()
    en_ref = np.linalg.norm(yc, axis=2)
    assert rel_l2(en_gpu, en_ref) <= tol
    ctx.close()


@pytest.mark.parametrize("n", [2, 3, 4])
def test_full_size_bf16_maps(n):
    """The workloads with x and y stored as bf16, as bench.py --act bf16 times them (inputs
    beyond the memory-side cache take the streaming loads): the same index sets and alpha as the
    fp32-storage run on the same bf16-valued input, and bit for bit that run's output rounded
    to nearest even on the host.  The fp32-storage run is the one checked against the oracle in
    test_full_size_forward."""
    cfg = synth.config(n)
    print(f"workload {cfg.name}: generating inputs", flush=True)
    x, w = synth.make_inputs(cfg)
    x = synth.round_to_bf16(x)
    wd, wsd = upload_weights(w)
    ctx = wcc.Context(0)
    shape = (cfg.B, cfg.C_out, cfg.H, cfg.W)
    out = {}
    for act, tdt in ((wcc.F32, torch.float32), (wcc.BF16, torch.bfloat16)):
        d = wcc.make_desc(cfg.B, cfg.C_in, cfg.C_out, cfg.H, cfg.W, cfg.levels, cfg.keep_num,
                          cfg.keep_den, cfg.w_dtype, cfg.act_bits, act)
        ctx.ensure_workspace(d)
        xd = dev(x).to(tdt)
        y = torch.full(shape, float("nan"), dtype=tdt, device="cuda")
        idx = torch.full((cfg.B, cfg.k), -7, dtype=torch.int32, device="cuda")
        alpha = torch.zeros(1, dtype=torch.float32, device="cuda")
        print(f"  gpu forward, maps {tdt}", flush=True)
        ctx.wcc_forward(d, xd, wd, wsd, 0.0, y, idx, alpha)
        torch.cuda.synchronize()
        out[act] = (y, idx, float(alpha.item()))
        del xd
    y32, i32, a32 = out[wcc.F32]
    y16, i16, a16 = out[wcc.BF16]
    assert torch.equal(i16, i32) and a16 == a32
    want_bits = synth._round_to_bf16_bits(y32.cpu().numpy())
    got_bits = y16.view(torch.int16).cpu().numpy().view(np.uint16)
    np.testing.assert_array_equal(got_bits, want_bits)
    ctx.close()


@pytest.mark.parametrize("act,shape", [("f32", None), ("bf16", None), ("f32", (96, 1024, 4, 6)),
                                       ("f32", (512, 128, 6, 4))])
def test_full_size_block(ref, act, shape):
    """The block workload bench.py --config 6 times (256x256, c 256, expansion 4, batch 8,
    keep 1/4), with fp32 and with bf16 feature maps (--act bf16), and two more rows of the
    paper's timing table at the batch it prints (the smallest image with the most channels,
    chained; the largest image, whose middle tensors are formed), checked where the oracle can
    follow: the first layer's index sets in full, its output and K_dw on sampled planes, and
    the second layer on one sample (valid index set for the fp64 norms of K_dw applied to the
    GPU's own middle tensor, output for that index set).  With bf16 maps K_dw exists only
    folded into the second layer's transform, so its output is the oracle's."""
    bf16 = act == "bf16"
    cfg = synth.block_config(1, 4) if shape is None else synth.block_shape(shape[0], shape[0], *shape[1:], 1, 4)
    print(f"workload {cfg.name} ({act} maps): generating inputs", flush=True)
    x, w1, w_dw, w3 = synth.make_block_inputs(cfg)
    if bf16:
        x = synth.round_to_bf16(x)
    N, k = cfg.N, cfg.k
    d = wcc.make_block_desc(cfg.B, cfg.C, cfg.expansion, cfg.H, cfg.W, cfg.levels, cfg.keep_num,
                            cfg.keep_den, cfg.w_dtype, cfg.act_bits, wcc.BF16 if bf16 else wcc.F32)
    print(f"  route without middle outputs: {'chained' if wcc.block_is_chained(d) else 'middle tensors formed'}",
          flush=True)
    ctx = wcc.Context(0)
    ctx.ensure_workspace(d)
    tdt = torch.bfloat16 if bf16 else torch.float32
    xd = dev(x).to(tdt)
    assert torch.equal(xd.float().cpu(), torch.from_numpy(x))
    w1d, _ = upload_weights(w1)
    w3d, _ = upload_weights(w3)
    mid = (cfg.B, cfg.C_mid, cfg.H, cfg.W)
    t1 = torch.empty(mid, dtype=tdt, device="cuda")
    t2 = None if bf16 else torch.empty(mid, dtype=tdt, device="cuda")
    y = torch.empty(x.shape, dtype=tdt, device="cuda")
    idx1 = torch.empty((cfg.B, k), dtype=torch.int32, device="cuda")
    idx3 = torch.empty((cfg.B, k), dtype=torch.int32, device="cuda")
    print("  gpu block forward", flush=True)
    ctx.wcc_block_forward(d, xd, w1d, None, dev(w_dw), w3d, None, y, t1, t2, idx1, idx3)
    torch.cuda.synchronize()
    # The call bench.py times: no middle outputs, so the two layers are chained in the compressed
    # domain (the expanded tensors are never formed).  With fp32 maps the chained passes rebuild
    # the same numbers: where both calls choose the same second index set the outputs are equal
    # bit for bit, else this call's set is checked for validity further down.  With bf16 maps the
    # materialised middle tensor is rounded to bf16 and the chained one is not, so the two
    # outputs agree to the tolerance only.
    y2 = torch.empty_like(y)
    idx3_2 = torch.empty_like(idx3)
    ctx.wcc_block_forward(d, xd, w1d, None, dev(w_dw), w3d, None, y2, None, None, None, idx3_2)
    torch.cuda.synchronize()
    same3 = bool(torch.equal(idx3, idx3_2))
    print(f"  call without middle outputs: second index set {'equal' if same3 else 'differs'}", flush=True)
    if bf16:
        # storage is all that differs from the chained call with fp32 maps on the same (bf16-valued)
        # input: the same index sets, and that call's output rounded once to nearest even
        d32 = wcc.make_block_desc(cfg.B, cfg.C, cfg.expansion, cfg.H, cfg.W, cfg.levels, cfg.keep_num,
                                  cfg.keep_den, cfg.w_dtype, cfg.act_bits, wcc.F32)
        ctx.ensure_workspace(d32)
        y32 = torch.empty(x.shape, dtype=torch.float32, device="cuda")
        idx3_32 = torch.empty_like(idx3)
        ctx.wcc_block_forward(d32, xd.float(), w1d, None, dev(w_dw), w3d, None, y32, None, None, None, idx3_32)
        torch.cuda.synchronize()
        assert torch.equal(idx3_2, idx3_32)
        want_bits = synth._round_to_bf16_bits(y32.cpu().numpy())
        np.testing.assert_array_equal(y2.view(torch.int16).cpu().numpy().view(np.uint16), want_bits)
        del y32, idx3_32, want_bits
        ctx.ensure_workspace(d)
        print(f"  rel-L2 between the chained and the materialised output: "
              f"{rel_l2(y2.float().cpu().numpy(), y.float().cpu().numpy()):.3e}", flush=True)
    else:
        if same3:
            assert torch.equal(y, y2)
        assert rel_l2(y2.cpu().numpy(), y.cpu().numpy()) <= 1e-2
    g_idx3_2 = idx3_2.cpu().numpy().astype(np.int64)
    del y2, idx3_2

    print("  oracle: first layer's selection", flush=True)
    coef = ref.haar_fwd(x, cfg.levels).reshape(cfg.B, cfg.C, N)
    o_idx1 = ref.topk(ref.channel_norm(coef), k)
    np.testing.assert_array_equal(idx1.cpu().numpy().astype(np.int64), o_idx1)
    xc = ref.gather(coef, o_idx1)
    del coef
    a1 = float(np.float32(ref.absmax(xc)))
    print("  oracle: first layer's output on sampled planes", flush=True)
    xhat = ref.quant_codes(xc, a1, 8)
    del xc
    rng = np.random.default_rng(6)
    planes = {(0, 0), (cfg.B - 1, cfg.C_mid - 1)}
    while len(planes) < 5:
        planes.add((int(rng.integers(cfg.B)), int(rng.integers(cfg.C_mid))))
    for (b, o) in sorted(planes):
        yc = ref.pointwise(w1.values[o:o + 1], np.array([a1 / 127.0]), xhat[b:b + 1])
        want = ref.haar_inv(ref.scatter(yc, o_idx1[b:b + 1], N), cfg.H, cfg.W, cfg.levels)[0, 0]
        got_t1 = t1[b, o].float().cpu().numpy()
        assert rel_l2(got_t1, want) <= 1e-2, (b, o)
        if not bf16:
            # K_dw on the GPU's own plane
            want2 = ref.depthwise3x3(got_t1[None, None], w_dw[o:o + 1])[0, 0]
            assert rel_l2(t2[b, o].cpu().numpy(), want2) <= 1e-6, (b, o)
    del xhat

    print("  oracle: second layer's alpha over all samples, selection and output on sample 0", flush=True)
    g_idx3 = idx3.cpu().numpy().astype(np.int64)
    a3, keep0 = 0.0, None
    for b in range(cfg.B):
        if bf16:
            t2b = ref.depthwise3x3(t1[b:b + 1].float().cpu().numpy().astype(np.float64), w_dw)
        else:
            t2b = t2[b:b + 1].cpu().numpy().astype(np.float64)
        cb = ref.haar_fwd(t2b, cfg.levels).reshape(1, cfg.C_mid, N)
        del t2b
        xcb = ref.gather(cb, g_idx3[b:b + 1])
        a3 = max(a3, ref.absmax(xcb))
        if b == 0:
            norm0 = ref.channel_norm(cb)[0]
            keep0 = xcb
        del cb
    a3 = float(np.float32(a3))
    sel = g_idx3[0]
    assert np.all(np.diff(sel) > 0) and sel[0] >= 0 and sel[-1] < N
    kth = np.sort(norm0)[::-1][k - 1]
    dropped = np.ones(N, dtype=bool)
    dropped[sel] = False
    assert norm0[sel].min() >= kth * (1 - 1e-5) and norm0[dropped].max() <= kth * (1 + 1e-5)
    if not bf16:  # the chained call's own set, against the same fp64 norms
        sel2 = g_idx3_2[0]
        assert np.all(np.diff(sel2) > 0) and sel2[0] >= 0 and sel2[-1] < N
        dropped2 = np.ones(N, dtype=bool)
        dropped2[sel2] = False
        assert norm0[sel2].min() >= kth * (1 - 1e-5) and norm0[dropped2].max() <= kth * (1 + 1e-5)
    yc = ref.pointwise(w3.values, np.full(cfg.C, a3 / 127.0), ref.quant_codes(keep0, a3, 8))
    want = ref.haar_inv(ref.scatter(yc, g_idx3[0:1], N), cfg.H, cfg.W, cfg.levels)[0]
    got = y[0].float().cpu().numpy().astype(np.float64) - x[0].astype(np.float64)
    err = rel_l2(got, want)
    print(f"  sample 0 branch rel-L2 = {err:.3e}", flush=True)
    if bf16:
        # y = x + branch is rounded to 8 significant bits as a whole: the tolerance applies to
        # y, the block's output; the branch alone, smaller than x, carries that rounding several
        # times enlarged and is printed above for information
        err_y = rel_l2(y[0].float().cpu().numpy(), x[0].astype(np.float64) + want)
        print(f"  sample 0 output rel-L2 = {err_y:.3e}", flush=True)
        assert err_y <= 1e-2
    else:
        assert err <= 1e-2
    ctx.close()
