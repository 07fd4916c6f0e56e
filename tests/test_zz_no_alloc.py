"""wcc_forward_static (the entry point for callers that cannot allocate) against wcc_forward,
through the C ABI (needs an MI355X).

Both entry points run the same kernels, one on the caller's workspace, the other on the array
inside the library's device image, so every output is compared bit for bit; the oracle checks
the first call as well.  Two calls in a row, the second on a smaller layer: the array keeps the
first call's contents, and the second must not be disturbed by them.
"""
import numpy as np
import pytest
import torch

from paper_2205_12268_amd import synth, wcc
from tests.util import desc_of, dev, rel_l2, tol_for, upload_weights

pytestmark = pytest.mark.gpu

BF16, I8 = synth.W_BF16, synth.W_I8


def layer(name, B, Ci, Co, H, W, d, num, den, wd, bits, base=2):
    return synth.small(synth.config(base), name=name, B=B, C_in=Ci, C_out=Co, H=H, W=W, levels=d,
                       keep_num=num, keep_den=den, w_dtype=wd, act_bits=bits,
                       seed=synth.SEED_BASE + 0x900 + sum(map(ord, name)))


def run(ctx, cfg, entry, poison_ws=False):
    x, w = synth.make_inputs(cfg)
    d = desc_of(cfg)
    xd = dev(x)
    wd, wsd = upload_weights(w)
    y = torch.full((cfg.B, cfg.C_out, cfg.H, cfg.W), float("nan"), dtype=torch.float32, device="cuda")
    idx = torch.full((cfg.B, cfg.k), -7, dtype=torch.int32, device="cuda")
    alpha = torch.full((1,), -1.0, dtype=torch.float32, device="cuda")
    if entry == "static":
        ctx.wcc_forward_static(d, xd, wd, wsd, 0.0, y, idx, alpha)
    else:
        ctx.ensure_workspace(d)
        ctx.wcc_forward(d, xd, wd, wsd, 0.0, y, idx, alpha)
    torch.cuda.synchronize()
    return x, w, y.cpu().numpy(), idx.cpu().numpy(), float(alpha.item())


def test_static_entry_matches_workspace_entry_on_two_calls_in_a_row(ref):
    big = layer("static_big", 2, 64, 96, 128, 256, 3, 1, 4, BF16, 8)       # four-launch select
    small = layer("static_small", 1, 32, 16, 32, 64, 2, 1, 8, I8, 8)       # one-workgroup select
    ctx_s, ctx_w = wcc.Context(0), wcc.Context(0)
    try:
        assert wcc.workspace_bytes(desc_of(big)) <= wcc.STATIC_SCRATCH_BYTES
        # the static entry point first, back to back, with no workspace attached to its context
        got = []
        for cfg in (big, small):
            print(f"static call {cfg.name} seed {cfg.seed:#x}", flush=True)
            got.append(run(ctx_s, cfg, "static"))
        for cfg, (x, w, y_s, idx_s, a_s) in zip((big, small), got):
            print(f"workspace call {cfg.name}", flush=True)
            _, _, y_w, idx_w, a_w = run(ctx_w, cfg, "workspace")
            assert np.array_equal(idx_s, idx_w), cfg.name
            assert a_s == a_w, cfg.name
            assert np.array_equal(y_s.view(np.uint32), y_w.view(np.uint32)), cfg.name
            y_ref, idx_ref, a_ref = ref.forward(x, w.values, w.scale, cfg.levels, cfg.keep_num,
                                                cfg.keep_den, act_bits=cfg.act_bits)
            assert np.array_equal(idx_s.astype(np.int64), idx_ref), cfg.name
            assert np.float32(a_ref) == np.float32(a_s), cfg.name
            assert rel_l2(y_s, y_ref) <= tol_for(cfg), cfg.name
    finally:
        ctx_s.close()
        ctx_w.close()


def test_static_entry_rejects_layers_beyond_its_scratch():
    cfg = synth.config(3)  # 2.6 GB of workspace
    d = desc_of(cfg)
    assert wcc.workspace_bytes(d) > wcc.STATIC_SCRATCH_BYTES
    ctx = wcc.Context(0)
    try:
        x = torch.zeros(16, dtype=torch.float32, device="cuda")  # never read: the check comes first
        with pytest.raises(wcc.WccError) as e:
            ctx.wcc_forward_static(d, x, x, None, 0.0, x)
        assert e.value.status == 5  # WCC_ERR_WORKSPACE
    finally:
        ctx.close()
