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


@pytest.mark.parametrize("which", ["chained", "chained_shared_rows"])
def test_block_graph_replays_match_eager(which):
    """wcc_block_forward without middle outputs (the chained route: the expand layer stops at its
    compressed output, the project layer's passes rebuild what they need from it) recorded into
    a graph: every replay reproduces the eager call bit for bit, also after the input changed
    in place."""
    if which == "chained":
        cfg = synth.BlockCfg("graph_block", 2, 16, 4, 64, 128, 3, 1, 4, synth.W_BF16, 8,
                             seed=synth.SEED_BASE + 0x710)
    else:  # rows shared by the two waves of a workgroup
        cfg = synth.BlockCfg("graph_block_wide", 1, 8, 4, 32, 512, 3, 1, 8, synth.W_BF16, 8,
                             seed=synth.SEED_BASE + 0x711)
    x1, w1, w_dw, w3 = synth.make_block_inputs(cfg)
    x2 = np.ascontiguousarray(x1[:, ::-1, :, ::-1])
    d = wcc.make_block_desc(cfg.B, cfg.C, cfg.expansion, cfg.H, cfg.W, cfg.levels, cfg.keep_num,
                            cfg.keep_den, cfg.w_dtype, cfg.act_bits)
    assert wcc.block_is_chained(d)
    ctx = wcc.Context(0)
    try:
        ctx.ensure_workspace(d)
        w1d, _ = upload_weights(w1)
        w3d, _ = upload_weights(w3)
        wdd = dev(w_dw)
        xs = [dev(x1), dev(x2)]

        def eager(xd):
            y = torch.empty_like(xd)
            idx3 = torch.empty((cfg.B, cfg.k), dtype=torch.int32, device="cuda")
            ctx.wcc_block_forward(d, xd, w1d, None, wdd, w3d, None, y, None, None, None, idx3)
            torch.cuda.synchronize()
            return y.clone(), idx3.clone()

        want = [eager(xd) for xd in xs]
        assert not torch.equal(want[0][0], want[1][0])

        x_in = xs[0].clone()
        y = torch.empty_like(x_in)
        idx3 = torch.empty((cfg.B, cfg.k), dtype=torch.int32, device="cuda")
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            ctx.wcc_block_forward(d, x_in, w1d, None, wdd, w3d, None, y, None, None, None, idx3)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            ctx.wcc_block_forward(d, x_in, w1d, None, wdd, w3d, None, y, None, None, None, idx3)

        for rep in range(5):
            sel = rep % 2
            x_in.copy_(xs[sel])
            y.fill_(float("nan"))
            idx3.fill_(-1)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(idx3, want[sel][1]), f"replay {rep}: index list differs"
            assert torch.equal(y, want[sel][0]), f"replay {rep}: output differs"
    finally:
        ctx.close()
