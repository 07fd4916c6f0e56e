"""The synthetic-input recipes: determinism, the dyadic grid, the exactness budget."""
import numpy as np
import pytest

from paper_2205_12268_amd import synth


def test_configs_have_the_stated_sizes():
    ks = {1: 2048, 2: 32768, 3: 65536, 4: 7680}
    for n, k in ks.items():
        assert synth.config(n).k == k
    st = synth.stack_layers()
    assert len(st) == 16
    assert st[0].C_in == 16 and st[-1].C_out == 320
    macs = sum(l.C_in * l.C_out * l.H * l.W for l in st)
    assert abs(macs / 1e9 - 2.20) < 0.01  # GMAC per image at keep ratio 1


@pytest.mark.parametrize("n", [1, 2, 4])
def test_small_inputs_are_on_the_grid_and_seeded(n):
    cfg = synth.small(synth.config(n), B=1, C_in=8, C_out=8, H=32, W=64)
    x, w = synth.make_inputs(cfg)
    x2, w2 = synth.make_inputs(cfg)
    np.testing.assert_array_equal(x, x2)
    np.testing.assert_array_equal(w.stored, w2.stored)
    assert x.dtype == np.float32 and x.min() >= 0 and x.max() < cfg.clip_hi
    np.testing.assert_array_equal(np.rint(x * 64) / 64, x)
    assert (x == 0).mean() > 0.2          # ReLU leaves a large zero set
    assert synth.assert_exact_budget(x, cfg.levels) < 2 ** 24


def test_weight_storage_types():
    cfg = synth.small(synth.config(2), C_in=16, C_out=8)
    w = synth.make_w(cfg)
    assert w.stored.dtype == np.uint16 and w.scale is None
    np.testing.assert_array_equal(synth.bf16_bits_to_f32(w.stored).astype(np.float64), w.values)
    # bf16 rounding error is at most 2**-9 relative
    rng = np.random.default_rng(cfg.seed ^ 0xABCDEF)
    raw = rng.standard_normal((8, 16)) / 4.0
    assert np.abs(w.values - raw).max() <= np.abs(raw).max() * 2.0 ** -8
    cfg4 = synth.small(synth.config(4), C_in=16, C_out=8)
    w4 = synth.make_w(cfg4)
    assert w4.stored.dtype == np.int8 and w4.scale.shape == (8,)
    assert np.abs(w4.stored).max() == 127
    cfg1 = synth.config(1)
    w1 = synth.make_w(cfg1)
    np.testing.assert_array_equal(np.rint(w1.stored * 1024) / 1024, w1.stored)
    # 4-bit codes: two a byte, even channel in the low nibble, two's complement, -7..7
    cfg44 = synth.small(synth.config(4), C_in=16, C_out=8, w_dtype=synth.W_I4)
    w44 = synth.make_w(cfg44)
    assert w44.stored.dtype == np.uint8 and w44.stored.shape == (8, 8) and w44.scale.shape == (8,)
    lo = (w44.stored & 0x0F).astype(np.int16)
    hi = (w44.stored >> 4).astype(np.int16)
    lo[lo > 7] -= 16
    hi[hi > 7] -= 16
    np.testing.assert_array_equal(lo, w44.values[:, 0::2])
    np.testing.assert_array_equal(hi, w44.values[:, 1::2])
    assert np.abs(w44.values).max() == 7 and (w44.values < 0).any()


def test_budget_guard_trips():
    x = np.full((1, 4096, 8, 8), 7.0, dtype=np.float32)
    with pytest.raises(AssertionError):
        synth.assert_exact_budget(x, 3)
