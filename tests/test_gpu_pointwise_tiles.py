"""The contraction's arithmetic-bound variant (Eq. WCC: K_1x1 applied to the compressed signal;
hundreds of channels, a 128 x 128 tile a workgroup, two LDS stages) against the oracle, called
through wcc_pointwise on int8 codes drawn at random (needs an MI355X).

The shapes are chosen to reach that kernel (C_in >= 256, C_out >= 128, at least 256 workgroups,
not a wide expansion of few channels)
and to walk its edges: a last stage with fewer channels than a stage holds, output rows that
end inside the second and inside the third tile, a last column tile of four positions, both weight
types, one and several samples, and a shape whose tiles are all full.  A second list of shapes
takes the stream kernel with one workgroup walking all row tiles of its column tile.  With int8 weights the
sums are exact integers on both sides, so the comparison is to fp32 rounding of the scales;
with bf16 weights the products are exact and only the fp32 accumulation rounds.
"""
import numpy as np
import pytest
import torch

from paper_2205_12268_amd import synth, wcc
from tests.util import dev, rel_l2, upload_weights

pytestmark = pytest.mark.gpu

# name, B, C_in, C_out, H, W, keep_num, keep_den, weights
CASES = [
    ("bf16_ragged", 2, 264, 200, 128, 512, 4097, 16384, synth.W_BF16),   # k = 16388: 129 column tiles
    ("i8_ragged", 2, 272, 300, 64, 512, 2051, 8192, synth.W_I8),         # k = 8204, three row tiles
    ("bf16_full", 1, 1024, 512, 128, 512, 1, 4, synth.W_BF16),           # 32 stages, every tile full
    ("i8_many_samples", 5, 256, 128, 32, 512, 1, 2, synth.W_I8),         # one row tile, 64 x 5 tiles
    ("bf16_many_tiles", 4, 264, 300, 128, 512, 4097, 16384, synth.W_BF16),  # 1548 tiles in the natural order (small weights)
    ("i8_big_weights", 2, 1040, 1100, 64, 512, 2051, 8192, synth.W_I8),     # weights over 1 MB: tiles dealt to the dies in chunks, grid padded to a multiple of 8
]
# The stream kernel where one workgroup walks all row tiles of its column tile (512 column tiles
# or more; shapes that are not the kernel above's): one to five row tiles, a last row tile that is
# ragged, two to five chunks of channels, both weight types, an output that is streamed past the
# caches (over 512 MB).
WALK_CASES = [
    ("bf16_walk_4chunks", 4, 200, 384, 128, 512, 1, 4, synth.W_BF16),
    ("i8_walk_2chunks_ragged_rows", 8, 128, 300, 64, 512, 1, 4, synth.W_I8),
    ("bf16_walk_expansion_streamed", 9, 256, 1024, 128, 512, 1, 4, synth.W_BF16),   # 604 MB of output
    ("i8_walk_5chunks", 4, 272, 1100, 128, 512, 1, 4, synth.W_I8),
    ("bf16_walk_3chunks_two_tiles", 16, 136, 136, 64, 256, 1, 4, synth.W_BF16),
]


@pytest.mark.parametrize("case", CASES + WALK_CASES, ids=lambda c: c[0])
def test_arithmetic_bound_contraction_matches_oracle(ref, case):
    name, B, Ci, Co, H, W, num, den, wd_t = case
    cfg = synth.LayerCfg(name, B, Ci, Co, H, W, 3, num, den, wd_t, 8,
                         seed=synth.SEED_BASE + 0x900 + sum(map(ord, name)))
    k = cfg.k
    assert k % 4 == 0 and ((k + 127) // 128) * ((Co + 127) // 128) * B >= 256
    print(f"{cfg} k={k}", flush=True)
    w = synth.make_w(cfg)
    rng = np.random.default_rng(cfg.seed)
    codes = rng.integers(-127, 128, size=(B, Ci, k), dtype=np.int8)
    codes[:, :, -1] = 127                     # the last position of the ragged tile carries weight
    codes[0, Ci - 1, :] = -127                # and so does the last channel of the short stage
    alpha = np.float32(3.25)
    d = wcc.make_desc(B, Ci, Co, H, W, 3, num, den, wd_t, 8)
    ctx = wcc.Context(0)
    ctx.ensure_workspace(d)
    wdev, wsdev = upload_weights(w)
    # a dense output with a guard band behind it
    flat = torch.full((B * Co * k + 64,), float("nan"), dtype=torch.float32, device="cuda")
    yc = flat[:B * Co * k].view(B, Co, k)
    ctx.wcc_pointwise(d, wdev, wsdev, dev(codes), dev(np.array([alpha], dtype=np.float32)), yc)
    torch.cuda.synchronize()
    assert bool(torch.isnan(flat[B * Co * k:]).all())          # nothing written past the end
    got = yc.cpu().numpy()
    assert not np.isnan(got).any()
    scale = np.full(Co, float(alpha) / 127.0) if w.scale is None else float(alpha) / 127.0 * w.scale.astype(np.float64)
    want = ref.pointwise(w.values, scale, codes.astype(np.float64))
    err = rel_l2(got, want)
    print(f"  rel-L2 {err:.3e}", flush=True)
    assert err <= (2e-7 if wd_t == synth.W_I8 else 1e-5)
    # sampled entries one by one (rows at tile seams, the last positions)
    for (b, o, j) in [(0, 0, 0), (B - 1, Co - 1, k - 1), (0, min(127, Co - 1), k - 4), (B - 1, min(128, Co - 1), 129),
                      (0, Co // 2, k // 2)]:
        s = float(np.dot(w.values[o], codes[b, :, j].astype(np.float64))) * scale[o]
        assert abs(got[b, o, j] - s) <= 1e-5 * max(1.0, abs(s)), (b, o, j)
    ctx.close()
