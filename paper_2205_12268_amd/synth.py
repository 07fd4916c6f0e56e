"""Seeded synthetic inputs for the WCC forward path.

This module only *draws data*: activations shaped like the feature maps of
image-to-image CNN layers (piece-wise smooth, non-negative, so that their Haar
detail bands are sparse -- the property the section "Haar wavelet transform and
compression" relies on) and 1x1-convolution weights in their storage type.
It holds none of the method's arithmetic (no Haar step, no selection, no
activation quantiser, no contraction) and is the only code the CPU oracle's
tests and the HIP path's tests share.

Every activation lies on a dyadic grid (multiples of 2**-GRID_BITS, bounded) so
that Haar coefficients and channel-wise L1 sums are exact in fp32 in any
summation order; `assert_exact_budget` checks a sufficient bound for that with
integer arithmetic only.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Optional

import numpy as np
from scipy import ndimage

GRID_BITS = 6  # activations are multiples of 2**-6
SEED_BASE = 0x57434300

W_F32, W_BF16, W_I8, W_I4 = 0, 1, 2, 3


@dataclass(frozen=True)
class LayerCfg:
    """One WCC 1x1 layer workload (inputs of the explicit algorithm: feature
    map shape, kernel shape, level d, kept fraction gamma = keep_num/keep_den)."""

    name: str
    B: int
    C_in: int
    C_out: int
    H: int
    W: int
    levels: int
    keep_num: int
    keep_den: int
    w_dtype: int          # W_F32 | W_BF16 | W_I8
    act_bits: int         # 0 = no activation quantisation, 8 = signed 8 bit
    sigma: float = 0.0    # Gaussian blur radius in pixels (0: white noise)
    spike_p: float = 0.0  # Bernoulli probability of an additive spike
    spike_mag: float = 0.0
    clip_hi: float = 8.0  # activations clipped to [0, clip_hi - 2**-GRID_BITS]
    seed: int = SEED_BASE

    @property
    def N(self) -> int:
        return self.H * self.W

    @property
    def k(self) -> int:
        return (self.keep_num * self.N + self.keep_den - 1) // self.keep_den


def config(n: int) -> LayerCfg:
    """The four single-layer workloads (1-based numbering)."""
    if n == 1:
        return LayerCfg("cfg1_fp32_32x32_64x64", 1, 32, 32, 64, 64, 1, 1, 2, W_F32, 0,
                        sigma=0.0, clip_hi=8.0, seed=SEED_BASE + 1)
    if n == 2:
        return LayerCfg("cfg2_bf16_256x256_256x512", 1, 256, 256, 256, 512, 2, 1, 4, W_BF16, 8,
                        sigma=3.0, clip_hi=8.0, seed=SEED_BASE + 2)
    if n == 3:
        return LayerCfg("cfg3_bf16_64x256_512x1024", 4, 64, 256, 512, 1024, 3, 1, 8, W_BF16, 8,
                        sigma=4.0, spike_p=0.05, spike_mag=4.0, clip_hi=16.0, seed=SEED_BASE + 3)
    if n == 4:
        return LayerCfg("cfg4_i8_128x128_192x640", 8, 128, 128, 192, 640, 3, 1, 16, W_I8, 8,
                        sigma=2.0, clip_hi=8.0, seed=SEED_BASE + 4)
    raise ValueError("config number must be 1..4 (the layer stack is stack_layers())")


# (C_in, C_out, H, W, levels, sigma): eight expand/project pairs of an
# inverted-residual (expansion 6) backbone, shapes from the MobilenetV2 MAC
# table at half its resolution (512x1024 network input).
_STACK = [
    (16, 96, 256, 512, 3, 4.0), (96, 24, 128, 256, 3, 2.0),
    (24, 144, 128, 256, 3, 2.0), (144, 24, 128, 256, 3, 2.0),
    (24, 144, 128, 256, 3, 2.0), (144, 32, 64, 128, 2, 1.5),
    (32, 192, 64, 128, 2, 1.5), (192, 32, 64, 128, 2, 1.5),
    (32, 192, 64, 128, 2, 1.5), (192, 64, 32, 64, 1, 1.0),
    (64, 384, 32, 64, 1, 1.0), (384, 96, 32, 64, 1, 1.0),
    (96, 576, 32, 64, 1, 1.0), (576, 160, 32, 64, 1, 1.0),
    (160, 960, 32, 64, 1, 1.0), (960, 320, 32, 64, 1, 1.0),
]


def stack_layers(keep_num: int = 1, keep_den: int = 4, B: int = 4) -> list[LayerCfg]:
    """The 16 point-wise layers of the backbone stack, each with its own input."""
    out = []
    for i, (ci, co, h, w, d, sig) in enumerate(_STACK):
        out.append(LayerCfg(f"stack{i:02d}_{ci}to{co}_{h}x{w}", B, ci, co, h, w, d,
                            keep_num, keep_den, W_BF16, 8, sigma=sig, clip_hi=4.0,
                            seed=SEED_BASE + 0x500 + i))
    return out


def small(cfg: LayerCfg, **kw) -> LayerCfg:
    """A reduced copy of a workload (same recipe, other sizes)."""
    return replace(cfg, **kw)


# --------------------------------------------------------------------------- #
# activations
# --------------------------------------------------------------------------- #
def make_x(cfg: LayerCfg) -> np.ndarray:
    """Activations [B, C_in, H, W] float32 on the 2**-GRID_BITS grid."""
    rng = np.random.default_rng(cfg.seed)
    scale = float(1 << GRID_BITS)
    hi = cfg.clip_hi - 1.0 / scale
    x = np.empty((cfg.B, cfg.C_in, cfg.H, cfg.W), dtype=np.float32)
    for b in range(cfg.B):
        z = rng.standard_normal((cfg.C_in, cfg.H, cfg.W))
        if cfg.sigma > 0:
            z = ndimage.gaussian_filter(z, sigma=(0.0, cfg.sigma, cfg.sigma),
                                        mode="reflect", truncate=3.0)
            # a blur shrinks the standard deviation; bring each plane back to 1
            z /= z.std(axis=(1, 2), keepdims=True)
        np.maximum(z, 0.0, out=z)
        if cfg.spike_p > 0:
            z += cfg.spike_mag * (rng.random(z.shape) < cfg.spike_p)
        np.clip(z, 0.0, hi, out=z)
        x[b] = (np.rint(z * scale) / scale).astype(np.float32)
    return x


def assert_exact_budget(x: np.ndarray, levels: int) -> int:
    """Sufficient bound for exact fp32 coefficients and L1 channel sums.

    With x = m / 2**GRID_BITS (m integer), every level-l coefficient is an
    integer combination of the m's inside one 2**l x 2**l pixel block divided
    by 2**(GRID_BITS + l), so its numerator is at most the block sum of |m|,
    and a sum over channels of such magnitudes at most the channel sum of the
    block sums.  If that stays below 2**24 every partial sum is an exactly
    representable fp32 number.  Returns the bound that was checked.
    """
    m = np.rint(np.abs(x.astype(np.float64)) * (1 << GRID_BITS)).astype(np.int64)
    assert np.array_equal(m.astype(np.float64) / (1 << GRID_BITS), np.abs(x).astype(np.float64))
    B, C, H, W = m.shape
    s = 1 << levels
    blocks = m.reshape(B, C, H // s, s, W // s, s).sum(axis=(1, 3, 5))
    worst = int(blocks.max())
    assert worst < (1 << 24), f"exactness budget exceeded: {worst} >= 2**24"
    return worst


# --------------------------------------------------------------------------- #
# weights
# --------------------------------------------------------------------------- #
def _round_to_bf16_bits(w32: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns (uint16), round to nearest even."""
    u = w32.astype(np.float32).view(np.uint32).astype(np.uint64)
    u = u + 0x7FFF + ((u >> 16) & 1)
    return (u >> 16).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << 16).view(np.float32)


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """float32 array of the bf16-representable numbers nearest to `a` (ties to even): feature
    maps for layers whose activations are stored as bf16.  Dyadic inputs stay dyadic."""
    return bf16_bits_to_f32(_round_to_bf16_bits(np.asarray(a, dtype=np.float32)))


@dataclass
class Weights:
    """1x1 kernel [C_out, C_in] in its storage type.

    `stored`  what the library receives: float32 values, bf16 bit patterns
              (uint16), int8 codes, or 4-bit codes packed two a byte (uint8
              [C_out, C_in/2], even channel in the low nibble).
    `scale`   float32 [C_out] per-output-channel scale for int8 codes, else None.
    `values`  float64 [C_out, C_in]: the numbers the stored weights stand for
              (codes are *not* multiplied by `scale` here).
    """

    dtype: int
    stored: np.ndarray
    scale: Optional[np.ndarray]
    values: np.ndarray


def make_w(cfg: LayerCfg) -> Weights:
    rng = np.random.default_rng(cfg.seed ^ 0xABCDEF)
    w = rng.standard_normal((cfg.C_out, cfg.C_in)) / np.sqrt(cfg.C_in)
    if cfg.w_dtype == W_F32:
        w32 = (np.rint(w * 1024.0) / 1024.0).astype(np.float32)
        return Weights(W_F32, w32, None, w32.astype(np.float64))
    if cfg.w_dtype == W_BF16:
        bits = _round_to_bf16_bits(w.astype(np.float32))
        return Weights(W_BF16, bits, None, bf16_bits_to_f32(bits).astype(np.float64))
    if cfg.w_dtype == W_I8:
        s = (np.abs(w).max(axis=1) / 127.0).astype(np.float32)
        codes = np.clip(np.rint(w / s[:, None].astype(np.float64)), -127, 127).astype(np.int8)
        return Weights(W_I8, codes, s, codes.astype(np.float64))
    if cfg.w_dtype == W_I4:
        assert cfg.C_in % 2 == 0
        s = (np.abs(w).max(axis=1) / 7.0).astype(np.float32)
        codes = np.clip(np.rint(w / s[:, None].astype(np.float64)), -7, 7).astype(np.int8)
        nib = codes.astype(np.uint8) & 0x0F                      # two's complement nibbles
        packed = (nib[:, 0::2] | (nib[:, 1::2] << 4)).astype(np.uint8)
        return Weights(W_I4, np.ascontiguousarray(packed), s, codes.astype(np.float64))
    raise ValueError("unknown weight dtype")


def make_inputs(cfg: LayerCfg, check: bool = True):
    x = make_x(cfg)
    if check:
        assert_exact_budget(x, cfg.levels)
    return x, make_w(cfg)


# --------------------------------------------------------------------------- #
# the inverted residual block (the workload of the paper's timing table)
# --------------------------------------------------------------------------- #
@dataclass(frozen=True)
class BlockCfg:
    """x + K3(K_dw(K1 x)): C channels in and out, C * expansion in the middle; both 1x1
    convolutions are WCC layers with the same levels / keep ratio / quantiser."""

    name: str
    B: int
    C: int
    expansion: int
    H: int
    W: int
    levels: int
    keep_num: int
    keep_den: int
    w_dtype: int
    act_bits: int
    sigma: float = 3.0
    clip_hi: float = 8.0
    seed: int = SEED_BASE + 0x600

    @property
    def C_mid(self) -> int:
        return self.C * self.expansion

    @property
    def N(self) -> int:
        return self.H * self.W

    @property
    def k(self) -> int:
        return (self.keep_num * self.N + self.keep_den - 1) // self.keep_den

    def layer(self, which: int) -> LayerCfg:
        """Layer descriptor of the expand (0) or project (1) convolution."""
        ci, co = (self.C, self.C_mid) if which == 0 else (self.C_mid, self.C)
        return LayerCfg(f"{self.name}_l{which}", self.B, ci, co, self.H, self.W, self.levels,
                        self.keep_num, self.keep_den, self.w_dtype, self.act_bits, sigma=self.sigma,
                        clip_hi=self.clip_hi, seed=self.seed + 17 * which)


def block_shape(H: int, W: int, c: int, e: int, B: int, keep_num: int, keep_den: int,
                w_dtype: int = W_BF16) -> BlockCfg:
    """Any row of the paper's timing table: 3 levels, 8-bit codes, bf16 weights (or int8 codes
    with a scale per output channel, the paper's 8-bit weight setting)."""
    tag = "" if w_dtype == W_BF16 else "_w8"
    return BlockCfg(f"block_{H}x{W}_c{c}_e{e}_b{B}_keep{keep_num}of{keep_den}{tag}", B, c, e, H, W, 3,
                    keep_num, keep_den, w_dtype, 8)


def block_config(keep_num: int = 1, keep_den: int = 4, w_dtype: int = W_BF16) -> BlockCfg:
    """A row of the paper's timing table: 256x256 image, c_in 256, expansion 4, batch 8."""
    return block_shape(256, 256, 256, 4, 8, keep_num, keep_den, w_dtype)


def make_block_inputs(cfg: BlockCfg):
    """(x, w1, w_dw, w3): x as in the single-layer workloads (dyadic grid), the two 1x1 kernels
    in their storage type, the depthwise kernel fp32 [C_mid, 3, 3] (multiples of 2**-8, drawn
    from N(0, 1/9))."""
    l0, l1 = cfg.layer(0), cfg.layer(1)
    x = make_x(l0)
    assert_exact_budget(x, cfg.levels)
    rng = np.random.default_rng(cfg.seed ^ 0x5A5A5A)
    w_dw = (np.rint(rng.standard_normal((cfg.C_mid, 3, 3)) / 3.0 * 256.0) / 256.0).astype(np.float32)
    return x, make_w(l0), w_dw, make_w(l1)
