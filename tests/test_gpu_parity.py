"""HIP path vs CPU oracle, element by element, through the C ABI (needs an MI355X).

Bars: coefficients, norms, index sets and int8 codes bit-exact (inputs lie on a dyadic grid,
so fp32 sums are exact in any order); outputs within 1e-5 relative L2 for the fp32 path and
1e-2 for bf16 / int8 accumulation.
"""
import numpy as np
import pytest
import torch

from paper_2205_12268_amd import synth, wcc
from tests.util import desc_of, dev, oracle_scale, rel_l2, tol_for, upload_weights

pytestmark = pytest.mark.gpu

F32, BF16, I8, I4 = synth.W_F32, synth.W_BF16, synth.W_I8, synth.W_I4


def case(name, B, Ci, Co, H, W, d, num, den, wd, bits, base=2, **kw):
    return synth.small(synth.config(base), name=name, B=B, C_in=Ci, C_out=Co, H=H, W=W, levels=d,
                       keep_num=num, keep_den=den, w_dtype=wd, act_bits=bits,
                       seed=synth.SEED_BASE + 0x100 + sum(map(ord, name)), **kw)


SMALL = [
    synth.config(1),                                                   # the fp32 workload as is
    case("bf16_ragged", 2, 24, 40, 48, 136, 3, 1, 8, BF16, 8),         # masked lanes, M ragged, N % 4096 != 0
    case("i8_substrips", 1, 16, 16, 32, 24, 2, 1, 4, I8, 8),           # 8 strips per wave
    case("fma_fallback", 2, 20, 12, 16, 40, 1, 3, 7, BF16, 8),         # K % 8 != 0, k % 4 != 0
    case("vec2_path", 1, 8, 8, 6, 10, 1, 1, 2, F32, 0),                # W % 4 != 0
    case("four_levels", 1, 5, 7, 32, 64, 4, 1, 16, F32, 8),            # d = 4
    case("i8_two_segments", 3, 64, 32, 64, 320, 3, 1, 16, I8, 8),      # 2 column segments, 5 select blocks
    case("keep_all", 1, 8, 8, 16, 32, 2, 1, 1, BF16, 8),               # k = N
    case("keep_one", 1, 8, 8, 16, 32, 2, 1, 512, BF16, 8),             # k = 1
    case("bf16_noquant", 1, 16, 24, 32, 32, 2, 1, 4, BF16, 0),         # bf16 weights, fp32 activations
    case("i8w_noquant", 1, 16, 24, 32, 32, 2, 1, 4, I8, 0),
    case("f32w_quant", 1, 16, 24, 32, 32, 3, 1, 4, F32, 8),
    case("wide_k", 1, 96, 160, 64, 128, 2, 1, 2, BF16, 8),             # K > 64: two k tiles; M > 128
    case("i8_wide", 2, 192, 144, 32, 64, 1, 1, 4, I8, 8),
    case("spiky", 2, 32, 32, 64, 128, 3, 1, 8, BF16, 8, base=3),
    case("i4_weights", 2, 64, 48, 32, 64, 2, 1, 4, I4, 8),              # 4-bit codes, matrix-core path
    case("i4_ragged", 1, 22, 10, 16, 24, 1, 1, 3, I4, 8),               # C_in % 16 != 0: FMA path
    case("i4_noquant", 1, 16, 24, 32, 32, 2, 1, 4, I4, 0),
    # strips that keep 1025..1088 of their 2048 positions: one more list row than the dense keep
    # pass packs, so these strips must take the one-store-per-slot route
    case("d3_half_kept", 2, 8, 8, 24, 336, 3, 1, 2, BF16, 8),
]


@pytest.fixture(scope="module")
def ctx():
    c = wcc.Context(0)
    yield c
    c.close()


def oracle_stages(ref, cfg, x, w, alpha_in=0.0):
    """Alg. 1 stage by stage with the oracle; returns every intermediate."""
    N, k = cfg.N, cfg.k
    coef = ref.haar_fwd(x, cfg.levels).reshape(cfg.B, cfg.C_in, N)
    norm = ref.channel_norm(coef)
    idx = ref.topk(norm, k)
    xc = ref.gather(coef, idx)
    if cfg.act_bits:
        alpha = float(np.float32(alpha_in if alpha_in > 0 else ref.absmax(xc)))
        xhat = ref.quant_codes(xc, alpha, cfg.act_bits)
    else:
        alpha, xhat = 0.0, xc
    yc = ref.pointwise(w.values, oracle_scale(ref, cfg, w, alpha), xhat)
    y = ref.haar_inv(ref.scatter(yc, idx, N), cfg.H, cfg.W, cfg.levels)
    return dict(coef=coef, norm=norm, idx=idx, xc=xc, alpha=alpha, xhat=xhat, yc=yc, y=y)


@pytest.mark.parametrize("cfg", SMALL, ids=lambda c: c.name)
def test_stages_and_forward_match_oracle(ref, ctx, cfg):
    print(f"case {cfg.name} seed {cfg.seed:#x}", flush=True)
    x, w = synth.make_inputs(cfg)
    o = oracle_stages(ref, cfg, x, w)
    d = desc_of(cfg)
    N, k = cfg.N, cfg.k
    assert wcc.k_of(d) == k
    ctx.ensure_workspace(d)
    xd = dev(x)
    wd, wsd = upload_weights(w)
    f32 = dict(dtype=torch.float32, device="cuda")

    # A: transform + norm
    coef = torch.full((cfg.B, cfg.C_in, N), float("nan"), **f32)
    norm = torch.full((cfg.B, N), float("nan"), **f32)
    ctx.wcc_haar_fwd(d, xd, coef, norm)
    np.testing.assert_array_equal(coef.cpu().numpy().astype(np.float64), o["coef"])
    np.testing.assert_array_equal(norm.cpu().numpy().astype(np.float64), o["norm"])
    coef2 = torch.empty_like(coef)
    ctx.wcc_haar_fwd(d, xd, coef2, None)
    assert torch.equal(coef, coef2)

    # B: index set, from norms and from coefficients
    idx = torch.full((cfg.B, k), -7, dtype=torch.int32, device="cuda")
    ctx.wcc_joint_topk(d, None, norm, idx)
    np.testing.assert_array_equal(idx.cpu().numpy().astype(np.int64), o["idx"])
    idx2 = torch.full_like(idx, -7)
    ctx.wcc_joint_topk(d, coef, None, idx2)
    assert torch.equal(idx, idx2)

    # B': gather (+ quantise)
    alpha = torch.zeros(1, **f32)
    if cfg.act_bits:
        xc = torch.zeros((cfg.B, cfg.C_in, k), dtype=torch.int8, device="cuda")
        ctx.wcc_gather_quant(d, coef, idx, 0.0, xc, alpha)
        assert float(alpha.item()) == o["alpha"]
        np.testing.assert_array_equal(xc.cpu().numpy().astype(np.float64), o["xhat"])
    else:
        xc = torch.zeros((cfg.B, cfg.C_in, k), **f32)
        ctx.wcc_gather_quant(d, coef, idx, 0.0, xc, None)
        np.testing.assert_array_equal(xc.cpu().numpy().astype(np.float64), o["xc"])

    # C: contraction
    yc = torch.full((cfg.B, cfg.C_out, k), float("nan"), **f32)
    ctx.wcc_pointwise(d, wd, wsd, xc, alpha if cfg.act_bits else None, yc)
    tol = tol_for(cfg)
    assert rel_l2(yc.cpu().numpy(), o["yc"]) <= tol

    # D+E: scatter + inverse, fed the oracle's Yc so that the stage is judged alone
    y = torch.full((cfg.B, cfg.C_out, cfg.H, cfg.W), float("nan"), **f32)
    ctx.wcc_scatter_ihaar(d, dev(o["yc"].astype(np.float32)), idx, y)
    want = ref.haar_inv(ref.scatter(o["yc"].astype(np.float32), o["idx"], N), cfg.H, cfg.W, cfg.levels)
    assert rel_l2(y.cpu().numpy(), want) <= 1e-6

    # the whole layer
    yf = torch.full_like(y, float("nan"))
    idxf = torch.full_like(idx, -7)
    af = torch.zeros(1, **f32)
    ctx.wcc_forward(d, xd, wd, wsd, 0.0, yf, idxf, af)
    assert torch.equal(idxf, idx)
    if cfg.act_bits:
        assert float(af.item()) == o["alpha"]
    err = rel_l2(yf.cpu().numpy(), o["y"])
    print(f"  rel-L2(y) = {err:.3e} (tol {tol:g})", flush=True)
    assert err <= tol
    # same result without the optional outputs, and run to run
    yf2 = torch.full_like(y, float("nan"))
    ctx.wcc_forward(d, xd, wd, wsd, 0.0, yf2)
    assert torch.equal(yf, yf2)


def test_perfect_reconstruction_with_identity_index_list(ref, ctx):
    cfg = case("recon", 2, 6, 6, 32, 72, 3, 1, 1, F32, 0)
    x, _ = synth.make_inputs(cfg)
    d = desc_of(cfg)
    ctx.ensure_workspace(d)
    xd = dev(x)
    coef = torch.empty((cfg.B, cfg.C_in, cfg.N), dtype=torch.float32, device="cuda")
    ctx.wcc_haar_fwd(d, xd, coef, None)
    idx = torch.arange(cfg.N, dtype=torch.int32, device="cuda").repeat(cfg.B, 1).contiguous()
    y = torch.empty_like(xd)
    ctx.wcc_scatter_ihaar(d, coef, idx, y)
    assert torch.equal(y, xd)  # dyadic inputs: bit-exact


# W = 200: a plane small enough for the one-workgroup select; W = 520: the multi-kernel one
@pytest.mark.parametrize("W", [200, 520])
@pytest.mark.parametrize("kind", ["constant", "zeros", "two_tie_classes"])
def test_tie_heavy_selection(ref, ctx, kind, W):
    B, k = 2, 5000
    cfg = case("ties", B, 4, 4, 64, W, 1, 1, 1, F32, 0)
    assert cfg.N == 64 * W
    d = wcc.make_desc(B, 4, 4, 64, W, 1, k, cfg.N, wcc.F32, 0)
    assert wcc.k_of(d) == k
    ctx.ensure_workspace(d)
    rng = np.random.default_rng(77)
    if kind == "constant":
        norm = np.full((B, cfg.N), 1.5, dtype=np.float32)
    elif kind == "zeros":
        norm = np.zeros((B, cfg.N), dtype=np.float32)
    else:
        norm = np.zeros((B, cfg.N), dtype=np.float32)
        norm[:, rng.choice(cfg.N, 3000, replace=False)] = 2.0   # all taken
        free = np.flatnonzero(norm[0] == 0)
        norm[:, rng.choice(free, 4000, replace=False)] = 0.25   # the class that straddles k
    idx = torch.full((B, k), -7, dtype=torch.int32, device="cuda")
    ctx.wcc_joint_topk(d, None, dev(norm), idx)
    np.testing.assert_array_equal(idx.cpu().numpy().astype(np.int64), ref.topk(norm, k))


@pytest.mark.parametrize("W", [200, 520])
def test_random_norms_all_bit_patterns(ref, ctx, W):
    """Keys that differ only in low mantissa bits, denormals and large values."""
    B, H = 3, 64
    N, k = H * W, 4321
    d = wcc.make_desc(B, 4, 4, H, W, 1, k, N, wcc.F32, 0)
    ctx.ensure_workspace(d)
    rng = np.random.default_rng(99)
    bits = rng.integers(0, 0x7F000000, size=(B, N), dtype=np.int64).astype(np.uint32)
    bits[1] = (0x3F800000 + rng.integers(0, 64, N)).astype(np.uint32)   # a narrow band around 1.0
    bits[2, ::3] = rng.integers(0, 200, size=len(bits[2, ::3])).astype(np.uint32)  # denormals
    norm = bits.view(np.float32)
    idx = torch.full((B, k), -7, dtype=torch.int32, device="cuda")
    ctx.wcc_joint_topk(d, None, dev(norm), idx)
    np.testing.assert_array_equal(idx.cpu().numpy().astype(np.int64), ref.topk(norm, k))


# Planes of 512 x 1024 positions: with 2 samples a select workgroup takes 2048 keys (two 16-byte
# loads a thread), with 4 samples 4096 (four) -- the ordered compaction then runs one block scan
# per load on top of the totals of the loads before it.
@pytest.mark.parametrize("B", [2, 4])
@pytest.mark.parametrize("kind", ["constant", "two_tie_classes", "bit_patterns"])
def test_selection_with_several_loads_per_thread(ref, ctx, kind, B):
    H, W = 512, 1024
    N, k = H * W, 70001
    d = wcc.make_desc(B, 4, 4, H, W, 1, k, N, wcc.F32, 0)
    assert wcc.k_of(d) == k
    ctx.ensure_workspace(d)
    rng = np.random.default_rng(1234 + B)
    if kind == "constant":
        norm = np.full((B, N), 0.75, dtype=np.float32)
    elif kind == "two_tie_classes":
        norm = np.zeros((B, N), dtype=np.float32)
        norm[:, rng.choice(N, 40000, replace=False)] = 2.0   # all taken
        free = np.flatnonzero(norm[0] == 0)
        norm[:, rng.choice(free, 90000, replace=False)] = 0.25   # the class that straddles k
    else:
        bits = rng.integers(0, 0x7F000000, size=(B, N), dtype=np.int64).astype(np.uint32)
        bits[1] = (0x3F800000 + rng.integers(0, 64, N)).astype(np.uint32)   # a narrow band around 1.0
        bits[0, ::3] = rng.integers(0, 200, size=len(bits[0, ::3])).astype(np.uint32)  # denormals
        norm = bits.view(np.float32)
    idx = torch.full((B, k), -7, dtype=torch.int32, device="cuda")
    ctx.wcc_joint_topk(d, None, dev(norm), idx)
    np.testing.assert_array_equal(idx.cpu().numpy().astype(np.int64), ref.topk(norm, k))


def test_all_zero_input_gives_zero_alpha_and_output(ref, ctx):
    cfg = case("zero_in", 1, 8, 8, 16, 32, 2, 1, 4, BF16, 8)
    _, w = synth.make_inputs(cfg)
    d = desc_of(cfg)
    ctx.ensure_workspace(d)
    xd = torch.zeros((1, 8, 16, 32), dtype=torch.float32, device="cuda")
    wd, wsd = upload_weights(w)
    y = torch.full((1, 8, 16, 32), float("nan"), dtype=torch.float32, device="cuda")
    idx = torch.full((1, cfg.k), -7, dtype=torch.int32, device="cuda")
    a = torch.ones(1, dtype=torch.float32, device="cuda")
    ctx.wcc_forward(d, xd, wd, wsd, 0.0, y, idx, a)
    assert float(a.item()) == 0.0
    assert torch.count_nonzero(y).item() == 0
    np.testing.assert_array_equal(idx.cpu().numpy()[0], np.arange(cfg.k))


def test_caller_supplied_alpha_clips(ref, ctx):
    cfg = case("alpha_in", 2, 16, 16, 32, 64, 2, 1, 4, BF16, 8)
    x, w = synth.make_inputs(cfg)
    o0 = oracle_stages(ref, cfg, x, w)
    a_in = o0["alpha"] / 3.0
    o = oracle_stages(ref, cfg, x, w, alpha_in=a_in)
    assert np.abs(o["xhat"]).max() == 127 and (np.abs(o["xhat"]) == 127).sum() > 1
    d = desc_of(cfg)
    ctx.ensure_workspace(d)
    wd, wsd = upload_weights(w)
    y = torch.empty((cfg.B, cfg.C_out, cfg.H, cfg.W), dtype=torch.float32, device="cuda")
    a = torch.zeros(1, dtype=torch.float32, device="cuda")
    ctx.wcc_forward(d, dev(x), wd, wsd, a_in, y, None, a)
    assert float(a.item()) == o["alpha"]
    assert rel_l2(y.cpu().numpy(), o["y"]) <= 1e-2
    # the stage call gives the oracle's codes bit for bit
    coef = dev(o["coef"].astype(np.float32))
    idx = dev(o["idx"].astype(np.int32))
    xc = torch.zeros((cfg.B, cfg.C_in, cfg.k), dtype=torch.int8, device="cuda")
    ctx.wcc_gather_quant(d, coef, idx, a_in, xc, a)
    np.testing.assert_array_equal(xc.cpu().numpy().astype(np.float64), o["xhat"])


def test_rounding_ties_in_the_quantiser(ref, ctx):
    """Coefficients that land exactly on .5 code boundaries: alpha = 127 -> code = rne(c)."""
    cfg = case("rne", 1, 4, 4, 8, 8, 1, 1, 1, F32, 8)
    d = desc_of(cfg)
    ctx.ensure_workspace(d)
    coef = np.zeros((1, 4, 64), dtype=np.float32)
    coef[0, 0, :16] = np.arange(16) + 0.5
    coef[0, 1, :16] = -(np.arange(16) + 0.5)
    coef[0, 2, :8] = [0.25, 0.75, 1.25, 126.5, 127.0, 126.49, 63.5, 64.5]
    idx = torch.arange(64, dtype=torch.int32, device="cuda")[None].contiguous()
    xc = torch.zeros((1, 4, 64), dtype=torch.int8, device="cuda")
    a = torch.zeros(1, dtype=torch.float32, device="cuda")
    ctx.wcc_gather_quant(d, dev(coef), idx, 127.0, xc, a)
    np.testing.assert_array_equal(xc.cpu().numpy().astype(np.float64),
                                  ref.quant_codes(coef, 127.0, 8))


def test_error_paths_enqueue_nothing(ctx):
    cfg = case("errs", 1, 8, 8, 16, 32, 2, 1, 4, BF16, 8)
    d = desc_of(cfg)
    x = torch.zeros((1, 8, 16, 32), dtype=torch.float32, device="cuda")
    y = torch.full_like(x, 3.0)
    w = torch.zeros((8, 8), dtype=torch.int16, device="cuda")
    fresh = wcc.Context(0)
    with pytest.raises(wcc.WccError) as e:      # no workspace attached
        fresh.wcc_forward(d, x, w, None, 0.0, y)
    assert e.value.status == 5
    small = torch.empty(256, dtype=torch.uint8, device="cuda")
    fresh.set_workspace(small)
    with pytest.raises(wcc.WccError) as e:      # workspace too small
        fresh.wcc_forward(d, x, w, None, 0.0, y)
    assert e.value.status == 5
    fresh.ensure_workspace(d)
    with pytest.raises(wcc.WccError) as e:      # misaligned tensor
        fresh.wcc_forward(d, x.view(-1)[1:], w, None, 0.0, y)
    assert e.value.status == 8
    d8 = wcc.make_desc(1, 8, 8, 16, 32, 2, 1, 4, wcc.I8, 8)
    with pytest.raises(wcc.WccError) as e:      # int8 weights need their scale
        fresh.wcc_forward(d8, x, w, None, 0.0, y)
    assert e.value.status == 1
    torch.cuda.synchronize()
    assert torch.all(y == 3.0)
    fresh.close()


@pytest.mark.parametrize("alpha_bits", [0x40490FDB, 0x3F7FFFFF, 0x41B4A3D7, 0x3A83126F, 0x7F000000, 0x00800000])
def test_quantiser_codes_on_arbitrary_floats(ref, ctx, alpha_bits):
    """Non-dyadic coefficients and clipping parameters (including a significand of all ones and
    the ends of the exponent range): the codes must still be the oracle's, bit for bit."""
    alpha = float(np.array([alpha_bits], dtype=np.uint32).view(np.float32)[0])
    cfg = case("anyfloat", 1, 16, 16, 64, 64, 1, 1, 1, F32, 8)
    d = desc_of(cfg)
    ctx.ensure_workspace(d)
    rng = np.random.default_rng(alpha_bits & 0xFFFF)
    n = 16 * cfg.N
    v = (rng.uniform(-1.2, 1.2, n) * alpha).astype(np.float32)
    # values that sit next to code boundaries (j + 0.5) * alpha / 127
    j = rng.integers(-127, 127, n // 4)
    near = ((j + 0.5) * (np.float64(alpha) / 127.0)).astype(np.float32)
    v[: n // 4] = np.nextafter(near, np.float32(np.inf) * rng.choice([-1, 1], n // 4).astype(np.float32))
    v[n // 4: n // 2] = near
    v = np.where(np.isfinite(v), v, np.float32(0)).astype(np.float32)
    coef = v.reshape(1, 16, cfg.N)
    idx = torch.arange(cfg.N, dtype=torch.int32, device="cuda")[None].contiguous()
    xc = torch.zeros((1, 16, cfg.N), dtype=torch.int8, device="cuda")
    a = torch.zeros(1, dtype=torch.float32, device="cuda")
    ctx.wcc_gather_quant(d, dev(coef), idx, alpha, xc, a)
    assert float(a.item()) == alpha
    np.testing.assert_array_equal(xc.cpu().numpy().astype(np.float64), ref.quant_codes(coef, alpha, 8))


@pytest.mark.parametrize("alpha", [1e-10, 3e-3, 7.5e18])
def test_quantiser_clips_values_whose_quotient_overflows(ref, ctx, alpha):
    """Finite coefficients so far above a caller-supplied clipping parameter that v / alpha is
    beyond fp32: Eq. (quantweights) clips them to +-1, so the codes are +-127 with the sign of v
    (the reciprocal route of the kernel must not turn the overflow into another code)."""
    cfg = case("overflow", 1, 16, 16, 64, 64, 1, 1, 1, F32, 8)
    d = desc_of(cfg)
    ctx.ensure_workspace(d)
    rng = np.random.default_rng(11)
    n = 16 * cfg.N
    with np.errstate(over="ignore"):
        mag = np.float32(alpha) * np.exp2(rng.uniform(-4.0, 126.0, n)).astype(np.float32)
    mag = np.minimum(mag, np.float32(3.0e38))
    v = (mag * rng.choice([-1.0, 1.0], n).astype(np.float32)).astype(np.float32)
    v[:8] = np.array([3.4e38, -3.4e38, 3.0e28, -3.0e28, 1.0e30, -1.0e30, 2.0, -2.0], dtype=np.float32)
    coef = v.reshape(1, 16, cfg.N)
    idx = torch.arange(cfg.N, dtype=torch.int32, device="cuda")[None].contiguous()
    xc = torch.zeros((1, 16, cfg.N), dtype=torch.int8, device="cuda")
    a = torch.zeros(1, dtype=torch.float32, device="cuda")
    ctx.wcc_gather_quant(d, dev(coef), idx, float(np.float32(alpha)), xc, a)
    got = xc.cpu().numpy().astype(np.float64)
    want = ref.quant_codes(coef, float(np.float32(alpha)), 8)
    np.testing.assert_array_equal(got, want)
    big = np.abs(coef.astype(np.float64)) >= 2.0 * float(np.float32(alpha))
    assert big.sum() > n // 2
    np.testing.assert_array_equal(got[big], 127.0 * np.sign(coef[big]))


@pytest.mark.parametrize("cfg", [SMALL[0], SMALL[1], SMALL[6], SMALL[12]], ids=lambda c: c.name)
@pytest.mark.parametrize("kind", ["prefix", "given"])
def test_forward_with_a_fixed_index_list(ref, ctx, cfg, kind):
    """wcc_forward_fixed: the first k positions, or a caller's ascending list per sample."""
    x, w = synth.make_inputs(cfg)
    d = desc_of(cfg)
    ctx.ensure_workspace(d)
    N, k = cfg.N, cfg.k
    if kind == "prefix":
        idx = np.tile(np.arange(k, dtype=np.int64), (cfg.B, 1))
        idx_dev = None
    else:
        rng = np.random.default_rng(cfg.seed + 5)
        idx = np.stack([np.sort(rng.choice(N, k, replace=False)) for _ in range(cfg.B)]).astype(np.int64)
        idx_dev = dev(idx.astype(np.int32))
    wd, wsd = upload_weights(w)
    y = torch.full((cfg.B, cfg.C_out, cfg.H, cfg.W), float("nan"), dtype=torch.float32, device="cuda")
    alpha = torch.zeros(1, dtype=torch.float32, device="cuda")
    ctx.wcc_forward_fixed(d, dev(x), wd, wsd, 0.0, idx_dev, y, alpha)
    want, o_alpha = ref.forward_with_list(x, w.values, w.scale, cfg.levels, idx, cfg.act_bits)
    if cfg.act_bits:
        assert float(alpha.item()) == o_alpha
    assert rel_l2(y.cpu().numpy(), want) <= tol_for(cfg)


QUANT_CASES = [c for c in SMALL if c.act_bits == 8]


@pytest.mark.parametrize("cfg", QUANT_CASES, ids=lambda c: c.name)
@pytest.mark.parametrize("frac", [0.37, 1.0, 2.5])
def test_forward_with_the_callers_alpha(ref, ctx, cfg, frac):
    """alpha_in > 0 (a learned clipping parameter): the keep pass writes int8 codes itself.
    alpha below, at and above the largest kept coefficient; every shape of the small set."""
    x, w = synth.make_inputs(cfg)
    o0 = oracle_stages(ref, cfg, x, w)
    a_in = float(np.float32(o0["alpha"] * frac))
    want, idx, alpha = ref.forward(x, w.values, w.scale, cfg.levels, cfg.keep_num, cfg.keep_den,
                                   act_bits=8, alpha_in=a_in)
    d = desc_of(cfg)
    ctx.ensure_workspace(d)
    wd, wsd = upload_weights(w)
    y = torch.full((cfg.B, cfg.C_out, cfg.H, cfg.W), float("nan"), dtype=torch.float32, device="cuda")
    a = torch.zeros(1, dtype=torch.float32, device="cuda")
    gi = torch.empty((cfg.B, cfg.k), dtype=torch.int32, device="cuda")
    ctx.wcc_forward(d, dev(x), wd, wsd, a_in, y, gi, a)
    assert float(a.item()) == alpha == a_in
    np.testing.assert_array_equal(gi.cpu().numpy().astype(np.int64), idx)
    assert rel_l2(y.cpu().numpy(), want) <= 1e-2
