"""wcc_forward recorded into a HIP graph: every replay must reproduce the eager result.

The entry point enqueues kernels only (no allocation, no synchronisation, no memset node), so
a caller may capture it.  The graph is replayed several times with eager work and
synchronisations in between, and with the input changed in place between replays.
"""
from __future__ import annotations

import numpy as np
import pytest
import torch

from paper_2205_12268_amd import synth, wcc
from tests.util import desc_of, dev, upload_weights

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("which", ["small_plane", "large_plane"])
def test_graph_replays_match_eager(which):
    base = synth.config(2)
    if which == "small_plane":   # one-workgroup select, 64x64 contraction tiles
        cfg = synth.small(base, name="graph_small", B=2, C_in=64, C_out=96, H=64, W=128, levels=2,
                          keep_num=1, keep_den=4, seed=synth.SEED_BASE + 0x700)
    else:                        # multi-kernel select, partial-norm groups
        cfg = synth.small(base, name="graph_large", B=1, C_in=32, C_out=32, H=128, W=256, levels=3,
                          keep_num=1, keep_den=8, seed=synth.SEED_BASE + 0x701)
    x1, w = synth.make_inputs(cfg)
    x2 = np.ascontiguousarray(x1[:, ::-1, :, ::-1])  # another input of the same shape
    d = desc_of(cfg)
    ctx = wcc.Context(0)
    try:
        ctx.ensure_workspace(d)
        wd, wsd = upload_weights(w)
        xs = [dev(x1), dev(x2)]
        shape = (cfg.B, cfg.C_out, cfg.H, cfg.W)

        def eager(xd):
            y = torch.empty(shape, dtype=torch.float32, device="cuda")
            idx = torch.empty((cfg.B, cfg.k), dtype=torch.int32, device="cuda")
            ctx.wcc_forward(d, xd, wd, wsd, 0.0, y, idx)
            torch.cuda.synchronize()
            return y.clone(), idx.clone()

        want = [eager(xd) for xd in xs]
        assert not torch.equal(want[0][0], want[1][0])

        x_in = xs[0].clone()
        y = torch.empty(shape, dtype=torch.float32, device="cuda")
        idx = torch.empty((cfg.B, cfg.k), dtype=torch.int32, device="cuda")
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            ctx.wcc_forward(d, x_in, wd, wsd, 0.0, y, idx)  # warm-up on the capture stream
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            ctx.wcc_forward(d, x_in, wd, wsd, 0.0, y, idx)

        for rep in range(5):
            sel = rep % 2
            x_in.copy_(xs[sel])          # eager work between the replays
            y.fill_(float("nan"))
            idx.fill_(-1)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(idx, want[sel][1]), f"replay {rep}: index list differs"
            assert torch.equal(y, want[sel][0]), f"replay {rep}: output differs"
    finally:
        ctx.close()
