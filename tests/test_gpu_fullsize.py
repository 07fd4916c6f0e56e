"""The single-layer workloads at their full sizes, in the launch configuration bench.py times.

The oracle runs the cheap stages in full (transform, norms, selection, gather, quantiser,
contraction) so index sets and alpha are compared exactly; the last stage (zero filling +
inverse transform) is evaluated by the oracle on sampled (sample, channel) planes.
"""
import numpy as np
import pytest
import torch

from paper_2205_12268_amd import synth, wcc
from tests.util import desc_of, dev, oracle_scale, rel_l2, tol_for, upload_weights

pytestmark = pytest.mark.gpu


def _huge_plane():
    """More than 2**20 kept positions per sample: the packed (rank | cell) lists of the strip
    kernels do not apply, 4096 select workgroups per sample, a one-chunk contraction."""
    return synth.small(synth.config(2), name="huge_plane", B=1, C_in=8, C_out=16, H=2048, W=2048,
                       levels=2, keep_num=1, keep_den=2, seed=synth.SEED_BASE + 0x800)


@pytest.mark.parametrize("n", [2, 3, 4, "huge_plane"])
def test_full_size_forward(ref, n):
    cfg = _huge_plane() if n == "huge_plane" else synth.config(n)
    n = 9 if n == "huge_plane" else n
    print(f"workload {cfg.name}: generating inputs", flush=True)
    x, w = synth.make_inputs(cfg)
    d = desc_of(cfg)
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
    del y2, idx2

    print("  oracle: transform, norms, selection", flush=True)
    coef = ref.haar_fwd(x, cfg.levels).reshape(cfg.B, cfg.C_in, N)
    o_idx = ref.topk(ref.channel_norm(coef), k)
    np.testing.assert_array_equal(idx.cpu().numpy().astype(np.int64), o_idx)
    xc = ref.gather(coef, o_idx)
    del coef
    o_alpha = float(np.float32(ref.absmax(xc)))
    assert float(alpha.item()) == o_alpha
    print("  oracle: quantiser, contraction", flush=True)
    xhat = ref.quant_codes(xc, o_alpha, 8)
    del xc
    yc = ref.pointwise(w.values, oracle_scale(ref, cfg, w, o_alpha), xhat)
    del xhat
    print("  oracle: inverse on sampled planes", flush=True)
    rng = np.random.default_rng(n)
    planes = {(0, 0), (cfg.B - 1, cfg.C_out - 1)}
    while len(planes) < 6:
        planes.add((int(rng.integers(cfg.B)), int(rng.integers(cfg.C_out))))
    tol = tol_for(cfg)
    worst = 0.0
    for (b, o) in sorted(planes):
        z = ref.scatter(yc[b:b + 1, o:o + 1], o_idx[b:b + 1], N)
        want = ref.haar_inv(z, cfg.H, cfg.W, cfg.levels)[0, 0]
        err = rel_l2(y[b, o].cpu().numpy(), want)
        worst = max(worst, err)
        assert err <= tol, (b, o, err)
    print(f"  worst plane rel-L2 = {worst:.3e} (tol {tol:g})", flush=True)
    # a property that holds at any size: Parseval, ||y[b,o]||_2 == ||yc[b,o,:]||_2
    en_gpu = torch.linalg.vector_norm(y.double(), dim=(2, 3)).cpu().numpy()
    en_ref = np.linalg.norm(yc, axis=2)
    assert rel_l2(en_gpu, en_ref) <= tol
    ctx.close()
