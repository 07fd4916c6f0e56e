"""Pins for the CPU oracle: what the paper and the mathematics fix about it.

None of these tests call the HIP library.  Each compares an oracle routine with
something that is not the oracle: a library convolution fed the kernels of
Eq. (HaarKernel), explicit matrices, closed forms, brute force, or numbers the
paper prints.
"""
import itertools
import os

import numpy as np
import pytest
import torch

from paper_2205_12268_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")

# The weight tensor of Eq. (HaarKernel), typed from the paper: four 2x2 kernels, factor 1/2.
HAAR_W = 0.5 * torch.tensor(
    [[[1.0, 1.0], [1.0, 1.0]],
     [[1.0, -1.0], [1.0, -1.0]],
     [[1.0, 1.0], [-1.0, -1.0]],
     [[1.0, -1.0], [-1.0, 1.0]]], dtype=torch.float64).unsqueeze(1)  # [4,1,2,2]


def lib_hwt(x2d: np.ndarray, levels: int) -> np.ndarray:
    """Multi-level transform with torch's stride-2 convolution as the one-level
    step, bands concatenated as Eq. (wavelet_transform) prescribes."""
    cur = torch.from_numpy(np.ascontiguousarray(x2d, dtype=np.float64))[None, None]
    details = []
    for _ in range(levels):
        y = torch.nn.functional.conv2d(cur, HAAR_W, stride=2)[0]  # [4,h/2,w/2]
        details.append([y[1], y[2], y[3]])
        cur = y[0][None, None]
    parts = [cur[0, 0].reshape(-1)]
    for lvl in reversed(range(levels)):
        parts += [b.reshape(-1) for b in details[lvl]]
    return torch.cat(parts).numpy()


def lib_ihwt(y: np.ndarray, H: int, W: int, levels: int) -> np.ndarray:
    """Inverse with torch's transposed convolution, levels in opposite order."""
    h, w = H >> levels, W >> levels
    y = torch.from_numpy(np.ascontiguousarray(y, dtype=np.float64))
    ll = y[: h * w].reshape(h, w)
    off = h * w
    for _ in range(levels):
        n = h * w
        bands = torch.stack([ll] + [y[off + j * n: off + (j + 1) * n].reshape(h, w)
                                    for j in range(3)])[None]
        ll = torch.nn.functional.conv_transpose2d(bands, HAAR_W, stride=2)[0, 0]
        off += 3 * n
        h, w = 2 * h, 2 * w
    return ll.numpy()


def explicit_matrix(ref, H, W, d):
    """N x N matrix of the oracle's transform: column i = transform of impulse i."""
    N = H * W
    eye = np.eye(N).reshape(N, H, W)
    return ref.haar_fwd(eye, d).T  # [N(out), N(in)]


SHAPES = [(2, 2, 1), (4, 4, 1), (4, 4, 2), (8, 8, 3), (8, 16, 2), (24, 40, 3), (16, 8, 1)]


# --------------------------------------------------------------------------- #
# P1-P3: the transform
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("H,W,d", SHAPES)
def test_orthonormal_and_inverse_is_transpose(ref, H, W, d):
    Hm = explicit_matrix(ref, H, W, d)
    N = H * W
    assert np.abs(Hm @ Hm.T - np.eye(N)).max() < 1e-14
    assert np.abs(Hm.T @ Hm - np.eye(N)).max() < 1e-14
    # the inverse routine is the transposed operator
    inv = ref.haar_inv(np.eye(N), H, W, d).reshape(N, N).T  # column i = inverse of unit i
    assert np.abs(inv - Hm.T).max() < 1e-15


@pytest.mark.parametrize("H,W,d", SHAPES)
def test_matches_library_convolution(ref, H, W, d):
    rng = np.random.default_rng(H * 1000 + W * 10 + d)
    x = rng.standard_normal((3, H, W))
    y = ref.haar_fwd(x, d)
    for c in range(3):
        np.testing.assert_allclose(y[c], lib_hwt(x[c], d), rtol=0, atol=1e-14)
        np.testing.assert_allclose(ref.haar_inv(y[c], H, W, d), lib_ihwt(y[c], H, W, d),
                                   rtol=0, atol=1e-14)


def test_two_level_concatenation_order(ref):
    """Eq. (wavelet_transform): [y1^2, y2^2, y3^2, y4^2, y2^1, y3^1, y4^1]."""
    rng = np.random.default_rng(5)
    x = rng.standard_normal((8, 12))
    y = ref.haar_fwd(x, 2)
    l1 = ref.haar_fwd(x, 1)                      # [y1^1 y2^1 y3^1 y4^1], 24 each
    n1, n2 = 24, 6
    l2 = ref.haar_fwd(l1[:n1].reshape(4, 6), 1)  # transform of y1^1
    np.testing.assert_array_equal(y[: 4 * n2], l2)
    np.testing.assert_array_equal(y[4 * n2:], l1[n1:])


def test_hand_values_of_the_four_kernels(ref):
    """Impulses through Eq. (HaarKernel): [[1,0],[0,0]] -> (1/2,1/2,1/2,1/2) etc."""
    want = {
        (0, 0): [0.5, 0.5, 0.5, 0.5],
        (0, 1): [0.5, -0.5, 0.5, -0.5],
        (1, 0): [0.5, 0.5, -0.5, -0.5],
        (1, 1): [0.5, -0.5, -0.5, 0.5],
    }
    for (r, c), v in want.items():
        x = np.zeros((2, 2))
        x[r, c] = 1.0
        np.testing.assert_array_equal(ref.haar_fwd(x, 1), np.array(v))


def test_separable_1d_composition(ref):
    """The 2-D kernels are products of [1,1]/sqrt2 and [1,-1]/sqrt2: band y2
    differences along a row, band y3 along a column."""
    lo = np.array([1.0, 1.0]) / np.sqrt(2.0)
    hi = np.array([1.0, -1.0]) / np.sqrt(2.0)
    H1 = np.stack([np.kron(np.eye(4), lo).reshape(4, 8), np.kron(np.eye(4), hi).reshape(4, 8)])
    rng = np.random.default_rng(11)
    x = rng.standard_normal((8, 8))
    y = ref.haar_fwd(x, 1).reshape(4, 4, 4)
    # rows filtered by V (vertical), columns by Hh (horizontal)
    for band, (V, Hh) in enumerate([(0, 0), (0, 1), (1, 0), (1, 1)]):
        np.testing.assert_allclose(y[band], H1[V] @ x @ H1[Hh].T, atol=1e-14)


@pytest.mark.parametrize("d", [1, 2, 3])
def test_constant_image_and_average_pool(ref, d):
    H, W = 16, 24
    c = 0.375
    y = ref.haar_fwd(np.full((H, W), c), d)
    n = (H >> d) * (W >> d)
    np.testing.assert_array_equal(y[:n], np.full(n, c * 2 ** d))
    np.testing.assert_array_equal(y[n:], 0.0)
    # y1 of one level = 2 x (2x2 average pooling)
    rng = np.random.default_rng(3)
    x = rng.standard_normal((H, W))
    pool = torch.nn.functional.avg_pool2d(torch.from_numpy(x)[None, None], 2)[0, 0].numpy()
    np.testing.assert_allclose(ref.haar_fwd(x, 1)[: H * W // 4].reshape(H // 2, W // 2),
                               2.0 * pool, atol=1e-15)


@pytest.mark.parametrize("H,W,d", SHAPES)
def test_parseval_and_dyadic_reconstruction(ref, H, W, d):
    rng = np.random.default_rng(17)
    x = rng.standard_normal((2, H, W))
    y = ref.haar_fwd(x, d)
    assert abs(np.linalg.norm(y) - np.linalg.norm(x)) < 1e-13 * np.linalg.norm(x)
    xd = np.rint(np.abs(x) * 64) / 64  # dyadic grid: everything is exact
    np.testing.assert_array_equal(ref.haar_inv(ref.haar_fwd(xd, d), H, W, d), xd)


def test_shape_errors(ref):
    with pytest.raises(ValueError):
        ref.haar_fwd(np.zeros((6, 8)), 2)
    with pytest.raises(ValueError):
        ref.haar_fwd(np.zeros((8, 8)), 0)


# --------------------------------------------------------------------------- #
# P6: joint top-k
# --------------------------------------------------------------------------- #
def test_channel_norm_is_l1(ref):
    rng = np.random.default_rng(2)
    c = rng.standard_normal((3, 5, 40))
    np.testing.assert_allclose(ref.channel_norm(c), np.abs(c).sum(axis=1), atol=1e-14)
    np.testing.assert_allclose(ref.channel_norm(c), np.linalg.norm(c, ord=1, axis=1), atol=1e-14)


def test_channel_norm_l2_is_the_squared_euclidean_norm(ref):
    rng = np.random.default_rng(3)
    c = rng.standard_normal((3, 5, 40))
    np.testing.assert_allclose(ref.channel_norm(c, "l2"), np.linalg.norm(c, ord=2, axis=1) ** 2,
                               rtol=1e-13)
    # a 3-4-5 triangle: L1 = 7, squared L2 = 25
    c = np.zeros((1, 2, 4))
    c[0, :, 1] = [3.0, -4.0]
    np.testing.assert_array_equal(ref.channel_norm(c, "l2")[0], [0.0, 25.0, 0.0, 0.0])
    np.testing.assert_array_equal(ref.channel_norm(c, "l1")[0], [0.0, 7.0, 0.0, 0.0])


def test_l1_and_l2_rank_differently_where_they_should(ref):
    """One pixel per 2x2 block is set so that every wavelet coefficient of the block has the
    magnitude pixel/2 (one level, orthonormal 2x2 kernels).  Block A carries (3, 3) over the two
    channels, block B (5, 0): L1 prefers A (3 > 2.5), L2 prefers B (4.5 < 6.25)."""
    x = np.zeros((1, 2, 2, 4))
    x[0, :, 0, 0] = [3.0, 3.0]     # block A = columns 0..1
    x[0, :, 0, 2] = [5.0, 0.0]     # block B = columns 2..3
    w = np.eye(2)
    coef = ref.haar_fwd(x, 1).reshape(1, 2, 8)
    # N = 8 positions: 4 bands x 2 blocks; the block's column inside each band is 0 (A) or 1 (B)
    _, idx1, _ = ref.forward(x, w, None, 1, 1, 2)
    _, idx2, _ = ref.forward(x, w, None, 1, 1, 2, norm="l2")
    np.testing.assert_array_equal(idx1[0], [0, 2, 4, 6])
    np.testing.assert_array_equal(idx2[0], [1, 3, 5, 7])
    np.testing.assert_allclose(np.abs(coef[0, :, 0]), [1.5, 1.5])
    np.testing.assert_allclose(np.abs(coef[0, :, 1]), [2.5, 0.0])
    # with every position kept the norm no longer matters
    ya, _, _ = ref.forward(x, w, None, 1, 1, 1)
    yb, _, _ = ref.forward(x, w, None, 1, 1, 1, norm="l2")
    np.testing.assert_array_equal(ya, yb)
    np.testing.assert_allclose(ya, x, atol=1e-15)


def test_l2_layer_equals_stage_composition(ref):
    rng = np.random.default_rng(31)
    x = rng.standard_normal((2, 6, 8, 16))
    w = rng.standard_normal((5, 6))
    y, idx, _ = ref.forward(x, w, None, 2, 1, 4, norm="l2")
    coef = ref.haar_fwd(x, 2).reshape(2, 6, 128)
    s = (coef ** 2).sum(axis=1)
    for b in range(2):
        order = np.lexsort((np.arange(128), -s[b]))[:32]
        assert sorted(order) == list(idx[b])
    z = np.zeros((2, 5, 128))
    for b in range(2):
        z[b][:, idx[b]] = w @ coef[b][:, idx[b]]
    np.testing.assert_allclose(y, ref.haar_inv(z, 8, 16, 2), atol=1e-12)


def test_topk_brute_force_tiny(ref):
    rng = np.random.default_rng(23)
    for trial in range(30):
        N = int(rng.integers(4, 13))
        k = int(rng.integers(1, N + 1))
        # few distinct values -> many ties
        s = rng.integers(0, 4, size=(2, N)).astype(np.float64) / 4
        idx = ref.topk(s, k)
        for b in range(2):
            assert list(idx[b]) == sorted(idx[b]) and len(set(idx[b])) == k
            best = max(s[b, list(comb)].sum() for comb in itertools.combinations(range(N), k))
            assert s[b, idx[b]].sum() == best
            # among maximal subsets, the tie rule takes the lexicographically smallest
            lex = min(comb for comb in itertools.combinations(range(N), k)
                      if s[b, list(comb)].sum() == best)
            assert tuple(idx[b]) == lex
            # independent ordering: numpy lexsort on (index, -norm)
            order = np.lexsort((np.arange(N), -s[b]))[:k]
            assert sorted(order) == list(idx[b])


def test_topk_crafted_ties(ref):
    N, k = 16, 5
    np.testing.assert_array_equal(ref.topk(np.ones((1, N)), k)[0], np.arange(k))
    s = np.zeros((1, N))
    s[0, [3, 9, 14]] = 2.0          # above the threshold
    s[0, [1, 4, 6, 12]] = 1.0       # tie class that straddles k
    np.testing.assert_array_equal(ref.topk(s, k)[0], [1, 3, 4, 9, 14])
    np.testing.assert_array_equal(ref.topk(s, N)[0], np.arange(N))
    with pytest.raises(ValueError):
        ref.topk(s, 0)
    with pytest.raises(ValueError):
        ref.topk(s, N + 1)


def test_k_formula(ref):
    assert ref.k_of(4096, 1, 2) == 2048
    assert ref.k_of(131072, 1, 4) == 32768
    assert ref.k_of(524288, 1, 8) == 65536
    assert ref.k_of(122880, 1, 16) == 7680
    assert ref.k_of(10, 1, 3) == 4  # ceil(10/3)
    assert ref.k_of(9, 1, 3) == 3


def test_gather_scatter_are_T_and_T_transpose(ref):
    rng = np.random.default_rng(8)
    B, Cc, N, k = 2, 3, 20, 7
    coef = rng.standard_normal((B, Cc, N))
    idx = np.stack([np.sort(rng.choice(N, k, replace=False)) for _ in range(B)])
    g = ref.gather(coef, idx)
    for b in range(B):
        T = np.zeros((k, N))
        T[np.arange(k), idx[b]] = 1.0
        np.testing.assert_array_equal(g[b], coef[b] @ T.T)
        np.testing.assert_array_equal(ref.scatter(g, idx, N)[b], g[b] @ T)


# --------------------------------------------------------------------------- #
# P7: quantiser
# --------------------------------------------------------------------------- #
def test_quantiser_closed_form_properties(ref):
    rng = np.random.default_rng(31)
    alpha = 3.25
    v = rng.uniform(-alpha, alpha, 5000)
    n = ref.quant_codes(v, alpha, 8)
    assert np.all(n == np.rint(n)) and n.min() >= -127 and n.max() <= 127
    deq = alpha * n / 127.0
    # error of a uniform grid of step alpha/127 (plus fp32 slack on the decision)
    assert np.abs(v - deq).max() <= alpha / 254 * (1 + 1e-5)
    # fixed points
    np.testing.assert_array_equal(ref.quant_codes(np.array([alpha, -alpha, 0.0]), alpha, 8),
                                  [127, -127, 0])
    # idempotent on the grid
    np.testing.assert_array_equal(ref.quant_codes(deq, alpha, 8), n)
    # clipping when alpha is below the data
    big = np.array([10.0, -10.0, 3.3, -4.0])
    np.testing.assert_array_equal(ref.quant_codes(big, alpha, 8), [127, -127, 127, -127])
    # odd symmetry and monotonicity
    np.testing.assert_array_equal(ref.quant_codes(-v, alpha, 8), -n)
    order = np.argsort(v)
    assert np.all(np.diff(n[order]) >= 0)
    # alpha == 0 (all kept coefficients zero)
    np.testing.assert_array_equal(ref.quant_codes(np.zeros(4), 0.0, 8), 0.0)


def test_quantiser_matches_equation_literally(ref):
    """x_b = alpha * q_{b-1}(clip(x/alpha,-1,1)), q_b(t) = round((2^b-1) t)/(2^b-1),
    evaluated with torch's float32 ops (round = half to even)."""
    rng = np.random.default_rng(41)
    alpha = np.float32(1.7)
    v = (np.rint(rng.uniform(-2.5, 2.5, 4000) * 64) / 64).astype(np.float32)
    t = torch.clamp(torch.from_numpy(v) / torch.tensor(alpha), -1.0, 1.0)
    levels = torch.tensor(float(2 ** 7 - 1))
    codes = torch.round(levels * t).numpy().astype(np.float64)
    np.testing.assert_array_equal(ref.quant_codes(v, float(alpha), 8), codes)
    # other bit widths
    for bits in (4, 6):
        lv = float(2 ** (bits - 1) - 1)
        want = torch.round(torch.tensor(lv) * t).numpy().astype(np.float64)
        np.testing.assert_array_equal(ref.quant_codes(v, float(alpha), bits), want)


def test_fp32_code_decision_stays_within_one_code_of_the_real_valued_one(ref):
    """The oracle decides the integer code in fp32 (u = v/alpha, clip, rint(127 u), each step
    rounded to fp32) so that both implementations take the same decision.  Against Eq.
    (quantweights) evaluated in fp64 on the kept coefficients of the synthetic workloads' kind
    (and on arbitrary reals) the two may differ only where 127 v/alpha lies within rounding
    distance of a half-integer: never by more than one code, and on a vanishing share of the
    values."""
    rng = np.random.default_rng(43)
    x, _ = synth.make_inputs(synth.LayerCfg("pin_quant", 1, 8, 8, 64, 128, 2, 1, 4, synth.W_BF16, 8,
                                            sigma=3.0, seed=synth.SEED_BASE + 0x51))
    coef = ref.haar_fwd(x.astype(np.float64), 2).ravel()
    cases = [(coef, float(np.float32(np.abs(coef).max()))),
             (coef, float(np.float32(0.37 * np.abs(coef).max()))),          # clipping live
             (rng.standard_normal(200_000) * 3.0, float(np.float32(np.pi))),
             (rng.uniform(-1, 1, 200_000), float(np.float32(1.0 - 2.0 ** -24)))]
    for v, alpha in cases:
        v32 = v.astype(np.float32).astype(np.float64)   # what the fp32 side sees
        got = ref.quant_codes(v32, alpha, 8)
        want = np.rint(127.0 * np.clip(v32 / alpha, -1.0, 1.0))  # fp64, half to even
        diff = np.abs(got - want)
        assert diff.max() <= 1.0
        differing = int((diff > 0).sum())
        # a decision can flip only if 127 v/alpha is within ~2^-16 of k + 1/2: a share of about
        # 2 * 127 * 2^-17 ~ 2e-3 would already be generous for values spread over the range
        assert differing <= max(4, int(2e-3 * v.size)), (differing, v.size)


def test_round_half_to_even(ref):
    # 127 * (c/alpha) exactly at .5: alpha = 127, c = j + 0.5
    c = np.array([0.5, 1.5, 2.5, -0.5, -1.5, -2.5])
    np.testing.assert_array_equal(ref.quant_codes(c, 127.0, 8), [0, 2, 2, -0.0, -2, -2])


# --------------------------------------------------------------------------- #
# P4, P5, P8: the layer
# --------------------------------------------------------------------------- #
def small_problem(seed, B=2, Ci=5, Co=4, H=8, W=16):
    rng = np.random.default_rng(seed)
    x = np.rint(np.maximum(rng.standard_normal((B, Ci, H, W)), 0) * 64) / 64
    w = np.rint(rng.standard_normal((Co, Ci)) * 1024) / 1024
    return x, w


@pytest.mark.parametrize("d", [1, 2, 3])
def test_keep_all_equals_direct_pointwise_conv(ref, d):
    """Eq. (WCC) with T = I: H^T K H x = K x."""
    x, w = small_problem(1)
    y, idx, _ = ref.forward(x, w, None, d, 1, 1)
    direct = np.einsum("oc,bchw->bohw", w, x)
    np.testing.assert_allclose(y, direct, rtol=0, atol=1e-13)
    np.testing.assert_array_equal(idx, np.tile(np.arange(x.shape[2] * x.shape[3]), (2, 1)))
    # and against a library convolution
    t = torch.nn.functional.conv2d(torch.from_numpy(x), torch.from_numpy(w)[:, :, None, None])
    np.testing.assert_allclose(y, t.numpy(), rtol=0, atol=1e-13)


@pytest.mark.parametrize("d,num,den", [(1, 1, 2), (2, 1, 4), (3, 1, 8), (2, 3, 7)])
def test_commutation_identity(ref, d, num, den):
    """H^T T^T K T H x == H^T T^T T H (K x) when T extracts the same entries."""
    x, w = small_problem(2)
    B, Ci, H, W = x.shape
    y, idx, _ = ref.forward(x, w, None, d, num, den)
    kx = np.einsum("oc,bchw->bohw", w, x)
    coef = ref.haar_fwd(kx, d)
    mask = np.zeros((B, 1, H * W))
    for b in range(B):
        mask[b, 0, idx[b]] = 1.0
    y2 = ref.haar_inv(coef * mask, H, W, d)
    np.testing.assert_allclose(y, y2, rtol=0, atol=1e-12)


@pytest.mark.parametrize("d,num,den", [(1, 1, 2), (2, 1, 4), (2, 5, 9)])
def test_forward_equals_operator_product(ref, d, num, den):
    """Eq. (WCC) as explicit matrices: y_b = (H^T T_b^T) (K x_b-in-wavelet-domain)."""
    x, w = small_problem(3, B=2, Ci=3, Co=2, H=4, W=8)
    B, Ci, H, W = x.shape
    N = H * W
    # transform matrix from the library convolution, not from the oracle
    Hm = np.stack([lib_hwt(np.eye(N)[i].reshape(H, W), d) for i in range(N)]).T
    k = -(-num * N // den)
    y, idx, _ = ref.forward(x, w, None, d, num, den)
    for b in range(B):
        X = x[b].reshape(Ci, N) @ Hm.T                  # rows: H x_c
        s = np.abs(X).sum(axis=0)
        sel = np.sort(np.lexsort((np.arange(N), -s))[:k])
        T = np.zeros((k, N))
        T[np.arange(k), sel] = 1.0
        Y = (w @ (X @ T.T)) @ T @ Hm                    # rows: H^T T^T (K T H x)
        np.testing.assert_array_equal(idx[b], sel)
        np.testing.assert_allclose(y[b].reshape(-1, N), Y, rtol=0, atol=1e-12)


def test_forward_stage_composition(ref):
    """wcc_ref_forward is the composition of the stage routines."""
    x, w = small_problem(4)
    B, Ci, H, W = x.shape
    d, num, den = 2, 1, 4
    y, idx, alpha = ref.forward(x, w, None, d, num, den, act_bits=8)
    coef = ref.haar_fwd(x, d)
    idx2 = ref.topk(ref.channel_norm(coef), ref.k_of(H * W, num, den))
    np.testing.assert_array_equal(idx, idx2)
    xc = ref.gather(coef, idx2)
    a = float(np.float32(ref.absmax(xc)))
    assert a == alpha
    codes = ref.quant_codes(xc, a, 8)
    yc = ref.pointwise(w, np.full(w.shape[0], a / 127.0), codes)
    y2 = ref.haar_inv(ref.scatter(yc, idx2, H * W), H, W, d)
    np.testing.assert_array_equal(y, y2)


def test_quantised_layer_is_linear_in_dequantised_coefficients(ref):
    """With quantisation the output is the unquantised layer applied to the
    dequantised kept coefficients; the error obeys the uniform-grid bound."""
    x, w = small_problem(5, B=2, Ci=6, Co=5, H=16, W=16)
    B, Ci, H, W = x.shape
    d, num, den = 2, 1, 4
    N, k = H * W, H * W // 4
    yq, idx, alpha = ref.forward(x, w, None, d, num, den, act_bits=8)
    y0, idx0, _ = ref.forward(x, w, None, d, num, den, act_bits=0)
    np.testing.assert_array_equal(idx, idx0)  # selection happens before quantisation
    coef = ref.haar_fwd(x, d)
    xc = ref.gather(coef, idx)
    assert alpha == float(np.float32(np.abs(xc).max()))
    deq = alpha * ref.quant_codes(xc, alpha, 8) / 127.0
    assert np.abs(deq - xc).max() <= alpha / 254 * (1 + 1e-5)
    y_lin = ref.haar_inv(ref.scatter(np.einsum("oc,bck->bok", w, deq), idx, N), H, W, d)
    np.testing.assert_allclose(yq, y_lin, rtol=0, atol=1e-12)
    bound = np.linalg.norm(w, 2) * (alpha / 254) * np.sqrt(B * Ci * k) * (1 + 1e-5)
    assert np.linalg.norm(yq - y0) <= bound
    # a caller-supplied clipping parameter below the data clips
    yq2, _, a2 = ref.forward(x, w, None, d, num, den, act_bits=8, alpha_in=alpha / 2)
    assert a2 == float(np.float32(alpha / 2))
    deq2 = a2 * ref.quant_codes(xc, a2, 8) / 127.0
    assert np.abs(deq2).max() == a2
    y_lin2 = ref.haar_inv(ref.scatter(np.einsum("oc,bck->bok", w, deq2), idx, N), H, W, d)
    np.testing.assert_allclose(yq2, y_lin2, rtol=0, atol=1e-12)


def test_int8_weight_scale_rows(ref):
    """Per-output-channel weight scale multiplies row o of the result."""
    x, w = small_problem(6)
    rng = np.random.default_rng(6)
    sw = rng.uniform(0.01, 0.02, w.shape[0])
    codes = np.rint(w * 40)
    y, _, _ = ref.forward(x, codes, sw, 2, 1, 2, act_bits=8)
    y1, _, _ = ref.forward(x, codes, None, 2, 1, 2, act_bits=8)
    np.testing.assert_allclose(y, y1 * sw[None, :, None, None], rtol=1e-12, atol=1e-14)


def test_pointwise_is_a_matrix_product(ref):
    rng = np.random.default_rng(9)
    w = rng.standard_normal((7, 5))
    xc = rng.standard_normal((3, 5, 11))
    np.testing.assert_allclose(ref.pointwise(w, None, xc), np.matmul(w[None], xc), atol=1e-13)
    sc = rng.standard_normal(7)
    np.testing.assert_allclose(ref.pointwise(w, sc, xc), sc[None, :, None] * np.matmul(w[None], xc),
                               atol=1e-13)


def test_thread_count_does_not_change_results(ref):
    x, w = small_problem(7, B=3, Ci=8, Co=8, H=16, W=32)
    ref.set_threads(1)
    y1, i1, a1 = ref.forward(x, w, None, 3, 1, 8, act_bits=8)
    ref.set_threads(4)
    y4, i4, a4 = ref.forward(x, w, None, 3, 1, 8, act_bits=8)
    ref.set_threads(ref.max_threads())
    np.testing.assert_array_equal(y1, y4)
    np.testing.assert_array_equal(i1, i4)
    assert a1 == a4


# --------------------------------------------------------------------------- #
# P9: cost model against the paper's printed numbers
# --------------------------------------------------------------------------- #
def _read_kv(path):
    out = {}
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        k, v = line.split()
        out[k] = int(v)
    return out


def test_bops_worked_example(ref):
    g = _read_kv(os.path.join(GOLDEN, "bops_example.txt"))
    mac = ref.conv_mac(g["c_in"], g["c_out"], g["n_w"], g["n_h"])
    conv = ref.conv_bops(mac, g["b_w"], g["b_a"])
    assert round(conv / 1e6) == g["conv_bops_millions"]
    haar = (ref.haar_bops(g["c_in"], g["n_w"], g["n_h"], g["levels"], g["b_a"])
            + ref.haar_bops(g["c_out"], g["n_w"], g["n_h"], g["levels"], g["b_a"]))
    assert round(haar / 1e6) == g["haar_fwd_plus_inv_bops_millions"]


def test_mac_table_rows(ref):
    for line in open(os.path.join(GOLDEN, "mobilenetv2_mac_rows.txt")):
        if line.startswith("#") or not line.strip():
            continue
        t = line.split()
        ci, co, K, groups, S, H, W, mac = map(int, t[1:])
        assert groups == 1
        assert ref.conv_mac(ci, co, W, H, K, K, S, S) == mac, t[0]


# ---- the depthwise 3x3 convolution and the inverted residual block (Eq. (inverted)) ----------
def test_depthwise_matches_library_correlation(ref):
    from scipy import ndimage
    rng = np.random.default_rng(21)
    x = rng.standard_normal((2, 3, 7, 10))
    w = rng.standard_normal((3, 3, 3))
    y = ref.depthwise3x3(x, w)
    for b in range(2):
        for c in range(3):
            want = ndimage.correlate(x[b, c], w[c], mode="constant", cval=0.0)
            np.testing.assert_allclose(y[b, c], want, rtol=0, atol=1e-13)
    # and against the framework's grouped convolution (cross-correlation, padding 1)
    t = torch.nn.functional.conv2d(torch.from_numpy(x), torch.from_numpy(w)[:, None], padding=1, groups=3)
    np.testing.assert_allclose(y, t.numpy(), rtol=0, atol=1e-13)


@pytest.mark.parametrize("i,j", list(itertools.product(range(3), range(3))))
def test_depthwise_shifted_impulse_kernels(ref, i, j):
    """A kernel that is 1 at tap (i, j) shifts the plane by (i-1, j-1) with zero fill: pins the
    orientation of the taps (no flip, rows before columns) and the border handling."""
    rng = np.random.default_rng(22)
    x = rng.standard_normal((1, 2, 5, 6))
    w = np.zeros((2, 3, 3))
    w[:, i, j] = 1.0
    y = ref.depthwise3x3(x, w)
    want = np.zeros_like(x)
    H, W = 5, 6
    for r in range(H):
        for c in range(W):
            rr, cc = r + i - 1, c + j - 1
            if 0 <= rr < H and 0 <= cc < W:
                want[:, :, r, c] = x[:, :, rr, cc]
    np.testing.assert_array_equal(y, want)


def test_depthwise_uses_its_own_channel_kernel(ref):
    x = np.ones((2, 3, 4, 4))
    w = np.zeros((3, 3, 3))
    w[0, 1, 1], w[1, 1, 1], w[2, 1, 1] = 2.0, 3.0, 5.0
    y = ref.depthwise3x3(x, w)
    for c, f in enumerate((2.0, 3.0, 5.0)):
        np.testing.assert_array_equal(y[:, c], f * np.ones((2, 4, 4)))
    # constant plane, all-ones kernel: 9 inside, 6 on edges, 4 in corners
    y = ref.depthwise3x3(np.ones((1, 1, 4, 5)), np.ones((1, 3, 3)))
    assert y[0, 0, 1, 1] == 9 and y[0, 0, 0, 2] == 6 and y[0, 0, 2, 0] == 6 and y[0, 0, 0, 0] == 4
    assert y[0, 0, 3, 4] == 4


def block_problem(seed, B=2, Cc=4, t=3, H=8, W=16):
    rng = np.random.default_rng(seed)
    x = np.rint(np.maximum(rng.standard_normal((B, Cc, H, W)), 0) * 64) / 64
    w1 = np.rint(rng.standard_normal((t * Cc, Cc)) * 1024) / 1024
    wd = np.rint(rng.standard_normal((t * Cc, 3, 3)) * 256) / 256
    w3 = np.rint(rng.standard_normal((Cc, t * Cc)) * 1024) / 1024
    return x, w1, wd, w3


@pytest.mark.parametrize("d", [1, 2])
def test_block_at_keep_all_equals_its_dense_definition(ref, d):
    """Eq. (inverted) with T = I in both WCC layers: x + K3 (K_dw (K1 x))."""
    x, w1, wd, w3 = block_problem(31)
    y, t1, t2, idx1, idx3, _, _ = ref.block_forward(x, w1, None, wd, w3, None, d, 1, 1)
    tx = torch.from_numpy(x)
    a = torch.nn.functional.conv2d(tx, torch.from_numpy(w1)[:, :, None, None])
    b = torch.nn.functional.conv2d(a, torch.from_numpy(wd)[:, None], padding=1, groups=w1.shape[0])
    c = torch.nn.functional.conv2d(b, torch.from_numpy(w3)[:, :, None, None])
    np.testing.assert_allclose(t1, a.numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(t2, b.numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(y, (tx + c).numpy(), rtol=0, atol=1e-11)


def test_block_structure(ref):
    """The residual is the input itself, the two layers pick their own index sets, and the
    block is the composition of the stages it returns."""
    x, w1, wd, w3 = block_problem(32)
    y0 = ref.block_forward(x, w1, None, wd, np.zeros_like(w3), None, 2, 1, 4, 8)[0]
    np.testing.assert_array_equal(y0, x)  # K3 = 0: only the skip connection is left
    y, t1, t2, idx1, idx3, a1, a3 = ref.block_forward(x, w1, None, wd, w3, None, 2, 1, 4, 8)
    want_t1, want_idx1, want_a1 = ref.forward(x, w1, None, 2, 1, 4, 8)
    np.testing.assert_array_equal(t1, want_t1)
    np.testing.assert_array_equal(idx1, want_idx1)
    t3, want_idx3, want_a3 = ref.forward(ref.depthwise3x3(t1, wd), w3, None, 2, 1, 4, 8)
    np.testing.assert_array_equal(idx3, want_idx3)
    np.testing.assert_array_equal(y, x + t3)
    assert a1 == want_a1 and a3 == want_a3 and a1 > 0 and a3 > 0
    assert idx1.shape == idx3.shape == (2, 32)


# ---- the layer with a given index list ----------------------------------------------------------
@pytest.mark.parametrize("bits", [0, 8])
def test_given_list_equals_selected_list_and_dense_conv(ref, bits):
    x, w = small_problem(41)
    y, idx, alpha = ref.forward(x, w, None, 2, 1, 4, bits)
    y2, alpha2 = ref.forward_with_list(x, w, None, 2, idx, bits)
    np.testing.assert_array_equal(y2, y)  # the list the shrinkage picks: the layer itself
    assert alpha2 == alpha
    # the full list, no quantiser: the dense 1x1 convolution
    N = x.shape[2] * x.shape[3]
    full = np.tile(np.arange(N), (x.shape[0], 1))
    y3, _ = ref.forward_with_list(x, w, None, 2, full, 0)
    np.testing.assert_allclose(y3, np.einsum("oc,bchw->bohw", w, x), rtol=0, atol=1e-13)


def test_prefix_list_is_a_low_pass(ref):
    """Keeping the first n_d positions keeps exactly the coarsest approximation: with K = I the
    output is the block average of x over 2^d x 2^d pixels, spread back over each block."""
    rng = np.random.default_rng(42)
    x = rng.standard_normal((1, 3, 8, 16))
    d, nd = 2, (8 // 4) * (16 // 4)
    idx = np.arange(nd)[None, :]
    y, _ = ref.forward_with_list(x, np.eye(3), None, d, idx, 0)
    want = x.reshape(1, 3, 2, 4, 4, 4).mean(axis=(3, 5), keepdims=True)
    want = np.broadcast_to(want, (1, 3, 2, 4, 4, 4)).reshape(1, 3, 8, 16)
    np.testing.assert_allclose(y, want, rtol=0, atol=1e-13)
