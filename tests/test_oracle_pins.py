"""Pins for the CPU oracle: each test checks it against something other than
itself - a hand-computed fixture, a closed form, a brute-force expansion, a
library routine on a special case, or an algebraic invariant (CPU only)."""
import itertools

import numpy as np
import pytest
import torch

from ebs_workloads import draw_levels
from golden_io import read_sections

BITS = [(kw, ka) for kw in range(1, 6) for ka in range(1, 6)]     # the paper's search space {1..5} (Sec. 5)


def _rand(seed, N, C, H, W, K, R, S, kw, ka):
    rng = np.random.default_rng(seed)
    q = draw_levels(rng, (K, R, S, C), kw)
    a = draw_levels(rng, (N, H, W, C), ka)
    return a, q


# ---------------------------------------------------------------- fixture
def test_hand_worked_example_matrix_form(oracle_mod):
    """Sec. 4.3 worked example (2x3 weights, 3x2 activations, 2 digits each) with
    hand-computed B_w, B_x, P and O."""
    g = read_sections("bd_worked_example_2x3_3x2.txt")
    Wm, Xm = g["W"], g["X"]
    # as a 1x1 convolution: c_o = 2, c_i = 3, two output positions
    q = Wm.reshape(2, 1, 1, 3).astype(np.uint8)
    a = Xm.T.reshape(1, 1, 2, 3).astype(np.uint8)
    O, P = oracle_mod.bd_matrix_form(a, q, 2, 2)
    assert np.array_equal(P, g["P"])
    assert np.array_equal(O.reshape(2, 2).T, g["O"])
    O2, _ = oracle_mod.bd_matrix_form(a, q, 2, 2, explicit_lambda=True)
    assert np.array_equal(O2, O)
    # the C routines on the same numbers
    assert np.array_equal(oracle_mod.conv2d_levels(a, q).reshape(2, 2).T, g["O"])
    acc, planes = oracle_mod.bitplane_conv(a, q, 2, 2, return_planes=True)
    assert np.array_equal(acc.reshape(2, 2).T, g["O"])
    # planes[n,oh,ow,k,m,kk] == P[k*M+m, j*K+kk]
    for j in range(2):
        for i in range(2):
            for m in range(2):
                for kk in range(2):
                    assert planes[0, 0, j, i, m, kk] == g["P"][2 * i + m, 2 * j + kk]
    assert np.array_equal(g["W"] @ g["X"], g["O"])


def test_hand_fixture_decomposition_identity():
    """Eq. 12: W = Lambda_w B_w and X = B_x Lambda_x^T on the fixture's digits."""
    g = read_sections("bd_worked_example_2x3_3x2.txt")
    Lw = np.kron(np.eye(2, dtype=np.int64), np.array([[1, 2]]))
    assert np.array_equal(Lw @ g["B_w"], g["W"])
    Lx = np.kron(np.eye(2, dtype=np.int64), np.array([[1, 2]]))
    assert np.array_equal(g["B_x"] @ Lx.T, g["X"])
    assert np.array_equal(g["B_w"] @ g["B_x"], g["P"])


# ---------------------------------------------------------------- Eq. 2 identity (brute force)
@pytest.mark.parametrize("kw,ka", BITS)
def test_direct_equals_bitplane_bruteforce(oracle_mod, kw, ka):
    geos = [  # N, C, H, W, K, R, S, stride, pad
        (1, 5, 4, 5, 3, 3, 3, 1, 1),
        (2, 33, 5, 4, 2, 3, 3, 2, 1),
        (1, 16, 6, 6, 4, 1, 1, 1, 0),
        (1, 7, 7, 6, 2, 3, 2, 2, 0),
        (1, 3, 5, 5, 2, 5, 5, 1, 2),
    ]
    for gi, (N, C, H, W, K, R, S, st, pad) in enumerate(geos):
        a, q = _rand(1000 + 17 * gi + 4 * kw + ka, N, C, H, W, K, R, S, kw, ka)
        d = oracle_mod.conv2d_levels(a, q, st, pad)
        b = oracle_mod.bitplane_conv(a, q, kw, ka, st, pad)
        assert d.shape == b.shape
        assert np.array_equal(d, b), (kw, ka, gi)


@pytest.mark.parametrize("kw,ka", [(1, 1), (2, 3), (4, 4), (3, 1), (5, 2), (5, 5)])
def test_matrix_form_equals_direct(oracle_mod, kw, ka):
    N, C, H, W, K, R, S, st, pad = 2, 6, 5, 5, 3, 3, 3, 2, 1
    a, q = _rand(77 + kw * 5 + ka, N, C, H, W, K, R, S, kw, ka)
    O, P = oracle_mod.bd_matrix_form(a, q, kw, ka, st, pad)
    d = oracle_mod.conv2d_levels(a, q, st, pad)
    assert np.array_equal(O, d)
    OH, OW = oracle_mod.out_dims(H, W, R, S, st, pad)
    assert P.shape == (K * kw, N * OH * OW * ka)          # c_o M x n K  (Sec. 4.3)
    acc, planes = oracle_mod.bitplane_conv(a, q, kw, ka, st, pad, return_planes=True)
    # P[(i,m),(j,k)] == planes[j][i][m][k]
    Pp = planes.reshape(N * OH * OW, K, kw, ka).transpose(1, 2, 0, 3).reshape(K * kw, -1)
    assert np.array_equal(Pp, P)
    O2, _ = oracle_mod.bd_matrix_form(a, q, kw, ka, st, pad, explicit_lambda=True)
    assert np.array_equal(O2, d)


# ---------------------------------------------------------------- library special case
@pytest.mark.parametrize("geo", [
    (2, 19, 9, 7, 5, 3, 3, 1, 1), (1, 64, 8, 8, 8, 3, 3, 2, 1), (2, 8, 6, 9, 4, 1, 1, 1, 0),
    (1, 4, 9, 9, 3, 5, 3, 2, 2), (1, 10, 7, 7, 2, 3, 3, 3, 0), (3, 16, 8, 8, 16, 3, 3, 1, 1),
])
def test_direct_equals_float64_library_conv(oracle_mod, geo):
    """Integer levels are exactly representable, every partial sum < 2^53, so the
    float64 library convolution is exact and must agree digit for digit."""
    N, C, H, W, K, R, S, st, pad = geo
    a, q = _rand(hash(geo) % 100000, N, C, H, W, K, R, S, 4, 4)
    ref = torch.nn.functional.conv2d(
        torch.from_numpy(a.astype(np.float64)).permute(0, 3, 1, 2),
        torch.from_numpy(q.astype(np.float64)).permute(0, 3, 1, 2), stride=st, padding=pad)
    ref = ref.permute(0, 2, 3, 1).numpy()
    d = oracle_mod.conv2d_levels(a, q, st, pad)
    assert d.shape == ref.shape
    assert np.array_equal(d.astype(np.float64), ref)


def test_1x1_is_integer_matmul(oracle_mod):
    N, C, H, W, K = 3, 70, 4, 5, 11
    a, q = _rand(5, N, C, H, W, K, 1, 1, 3, 4)
    d = oracle_mod.conv2d_levels(a, q, 1, 0)
    ref = a.reshape(-1, C).astype(np.int64) @ q.reshape(K, C).astype(np.int64).T
    assert np.array_equal(d.reshape(-1, K), ref)


# ---------------------------------------------------------------- closed forms
@pytest.mark.parametrize("kw,ka", [(1, 1), (2, 2), (4, 3), (4, 4), (5, 5), (1, 5)])
def test_all_max_levels_closed_form(oracle_mod, kw, ka):
    N, C, H, W, K = 1, 12, 6, 7, 3
    top = (2 ** kw - 1) * (2 ** ka - 1)
    a = np.full((N, H, W, C), 2 ** ka - 1, np.uint8)
    q = np.full((K, 3, 3, C), 2 ** kw - 1, np.uint8)
    d = oracle_mod.conv2d_levels(a, q, 1, 1)
    assert d.shape == (N, H, W, K)
    assert np.all(d[:, 1:-1, 1:-1, :] == 9 * C * top)      # interior: all 9 taps
    for (h, w) in [(0, 0), (0, W - 1), (H - 1, 0), (H - 1, W - 1)]:
        assert np.all(d[:, h, w, :] == 4 * C * top)        # corner: 4 taps
    assert np.all(d[:, 0, 1:-1, :] == 6 * C * top)         # edge: 6 taps
    assert np.all(d[:, 1:-1, 0, :] == 6 * C * top)
    # stride 2, pad 1 on 6x7 -> 3x4; output (0,0) sees taps r,s in {1,2} -> 4 taps
    d2 = oracle_mod.conv2d_levels(a, q, 2, 1)
    assert d2.shape == (N, 3, 4, K)
    assert np.all(d2[:, 0, 0, :] == 4 * C * top)
    assert np.all(d2[:, 1, 1, :] == 9 * C * top)
    assert np.all(d2[:, 0, 1, :] == 6 * C * top)
    # the widest ResNet-18 case stays far below 2^31
    assert 512 * 9 * 15 * 15 == 1036800


def test_single_nonzero_weight_picks_shifted_input(oracle_mod):
    """q[k0,r0,s0,c0] = v, all else 0  =>  acc[n,k0,oh,ow] = v * a_pad[n, oh*st+r0-pad, ow*st+s0-pad, c0]."""
    N, C, H, W, K, R, S = 2, 5, 7, 6, 4, 3, 3
    rng = np.random.default_rng(11)
    a = draw_levels(rng, (N, H, W, C), 4)
    for (k0, r0, s0, c0, v, st, pad) in [(1, 0, 2, 3, 7, 1, 1), (3, 2, 0, 0, 15, 2, 1), (0, 1, 1, 4, 1, 1, 0),
                                          (2, 0, 0, 2, 5, 2, 2)]:
        q = np.zeros((K, R, S, C), np.uint8)
        q[k0, r0, s0, c0] = v
        d = oracle_mod.conv2d_levels(a, q, st, pad)
        OH, OW = oracle_mod.out_dims(H, W, R, S, st, pad)
        ap = np.zeros((N, H + 2 * pad, W + 2 * pad, C), np.int64)
        ap[:, pad:pad + H, pad:pad + W] = a
        for oh in range(OH):
            for ow in range(OW):
                exp = v * ap[:, oh * st + r0, ow * st + s0, c0]
                assert np.array_equal(d[:, oh, ow, k0], exp)
        mask = np.ones(K, bool)
        mask[k0] = False
        assert np.all(d[..., mask] == 0)


def test_output_geometry_matches_library(oracle_mod):
    for H, W, R, S, st, pad in itertools.product([5, 8, 9], [6, 7], [1, 3], [1, 3], [1, 2, 3], [0, 1]):
        if pad >= R or pad >= S:
            continue
        t = torch.nn.functional.conv2d(torch.zeros(1, 1, H, W), torch.zeros(1, 1, R, S), stride=st, padding=pad)
        assert tuple(t.shape[2:]) == oracle_mod.out_dims(H, W, R, S, st, pad)


# ---------------------------------------------------------------- invariants
def test_linearity_in_weights_and_activations(oracle_mod):
    N, C, H, W, K = 1, 9, 6, 6, 3
    rng = np.random.default_rng(3)
    a1 = draw_levels(rng, (N, H, W, C), 2)
    a2 = draw_levels(rng, (N, H, W, C), 2)
    q1 = draw_levels(rng, (K, 3, 3, C), 2)
    q2 = draw_levels(rng, (K, 3, 3, C), 2)
    f = lambda a, q: oracle_mod.conv2d_levels(a, q, 1, 1).astype(np.int64)
    assert np.array_equal(f(a1 + a2, q1), f(a1, q1) + f(a2, q1))
    assert np.array_equal(f(a1, q1 + q2), f(a1, q1) + f(a1, q2))
    assert np.array_equal(f(3 * a1, q1), 3 * f(a1, q1))


def test_full_convolution_checksum(oracle_mod):
    """stride 1, pad = R-1: every (weight tap, pixel) pair meets exactly once, so
    sum(acc) = sum_c (sum of weights in c) * (sum of activations in c)."""
    N, C, H, W, K, R, S = 2, 6, 5, 4, 3, 3, 3
    a, q = _rand(21, N, C, H, W, K, R, S, 3, 4)
    d = oracle_mod.conv2d_levels(a, q, 1, R - 1).astype(np.int64)
    qs = q.astype(np.int64).sum(axis=(0, 1, 2))
    as_ = a.astype(np.int64).sum(axis=(0, 1, 2))
    assert d.sum() == int((qs * as_).sum())


def test_transposed_filter_is_detected(oracle_mod):
    """An asymmetric filter gives a different answer when r and s are swapped, so a
    transposed-operand mistake cannot hide: check against an explicit shift-sum."""
    N, C, H, W, K = 1, 2, 5, 6, 1
    rng = np.random.default_rng(8)
    a = draw_levels(rng, (N, H, W, C), 3)
    q = np.zeros((K, 2, 3, C), np.uint8)
    q[0, 0, 2, 0] = 3
    q[0, 1, 0, 1] = 2
    d = oracle_mod.conv2d_levels(a, q, 1, 0)       # OH=4, OW=4
    exp = 3 * a[0, 0:4, 2:6, 0].astype(np.int64) + 2 * a[0, 1:5, 0:4, 1].astype(np.int64)
    assert np.array_equal(d[0, :, :, 0], exp)


def test_point_matches_full(oracle_mod):
    N, C, H, W, K, R, S, st, pad = 2, 20, 9, 8, 6, 3, 3, 2, 1
    a, q = _rand(31, N, C, H, W, K, R, S, 4, 2)
    d = oracle_mod.conv2d_levels(a, q, st, pad)
    rng = np.random.default_rng(0)
    for _ in range(50):
        n, oh, ow, k = (int(rng.integers(0, s)) for s in d.shape)
        assert oracle_mod.conv2d_point(a, q, st, pad, n, k, oh, ow) == d[n, oh, ow, k]


# ---------------------------------------------------------------- stage-2 special cases
def test_one_bit_is_plain_binary_conv(oracle_mod):
    """(M,K) = (1,1): the result is the bitcount of the AND alone."""
    N, C, H, W, K = 1, 40, 5, 5, 2
    a, q = _rand(41, N, C, H, W, K, 3, 3, 1, 1)
    acc, planes = oracle_mod.bitplane_conv(a, q, 1, 1, 1, 1, return_planes=True)
    assert np.array_equal(acc, planes[..., 0, 0])
    assert np.array_equal(acc, oracle_mod.conv2d_levels(a, q, 1, 1))


def test_all_one_activations_sum_weights(oracle_mod):
    """K = 1 activations all 1 and no padding: acc = sum of the weight levels."""
    C, K = 13, 3
    rng = np.random.default_rng(2)
    q = draw_levels(rng, (K, 3, 3, C), 4)
    a = np.ones((1, 5, 5, C), np.uint8)
    d = oracle_mod.conv2d_levels(a, q, 1, 0)
    for k in range(K):
        assert np.all(d[..., k] == q[k].astype(np.int64).sum())


# ---------------------------------------------------------------- epilogue
def test_dequant_identity_and_values(oracle_mod):
    acc = np.array([[0, 1, -5, 1036800], [7, 8, 9, 10]], dtype=np.int32)
    out = oracle_mod.dequant(acc, np.float32(1.0))
    assert out.dtype == np.float32 and np.array_equal(out, acc.astype(np.float32))
    out = oracle_mod.dequant(acc, np.float32(0.5), np.float32(0.25))
    assert np.array_equal(out, (acc * 0.5 + 0.25).astype(np.float32))   # exact in binary
    sc = np.array([0.1, 0.2, 0.3, 0.4], np.float32)
    of = np.array([1.0, -1.0, 0.5, 0.0], np.float32)
    out = oracle_mod.dequant(acc, sc, of, per_channel=True)
    exp = (sc.astype(np.float64) * acc + of.astype(np.float64)).astype(np.float32)
    assert np.array_equal(out, exp)
    # constant arrays == per-layer broadcast
    c = oracle_mod.dequant(acc, np.full(4, 0.1, np.float32), np.full(4, 0.3, np.float32), per_channel=True)
    l = oracle_mod.dequant(acc, np.float32(0.1), np.float32(0.3))
    assert np.array_equal(c, l)


def test_op_count_formula():
    """Sec. 4.3 complexities: s*n*c_o*M*K ANDs (and as many counted bits)."""
    from ebs_workloads import config_cases
    c = config_cases(3)[0]   # 64->64 @56, N=64, (1,1)
    L = c.layer
    s, n, co = L.C * 9, L.N * 56 * 56, L.K
    assert c.binary_ops == 2 * s * n * co * 1 * 1
    c44 = [x for x in config_cases(3) if x.layer_index == 0 and (x.k_w, x.k_a) == (4, 4)][0]
    assert c44.binary_ops == 16 * c.binary_ops


# ---------------------------------------------------------------- fused re-quantisation (Eq. 1b-1c)
def test_requant_hand_examples(oracle_mod):
    import os
    from golden_io import GOLDEN
    rows = [l.split() for l in open(os.path.join(GOLDEN, "requant_examples.txt"))
            if l.strip() and not l.startswith("#") and not l.startswith("[")]
    assert len(rows) >= 15
    for bits, alpha, scale, offset, acc, exp in rows:
        got = oracle_mod.requant_levels(np.array([[int(acc)]], np.int32), np.float32(scale), np.float32(offset),
                                        False, float(alpha), int(bits))
        assert int(got[0, 0]) == int(exp), (bits, alpha, scale, offset, acc, exp, int(got[0, 0]))


@pytest.mark.parametrize("bits,alpha", [(2, 3.0), (4, 7.5), (3, 3.5), (1, 1.0), (4, 15.0), (5, 15.5), (5, 6.0)])
def test_requant_matches_float64_formula_on_exact_inputs(oracle_mod, bits, alpha):
    """With (2^b-1)/alpha an integer and power-of-two scales, every intermediate is exact in
    single precision, so the float64 textbook formula must give the same levels."""
    acc = np.arange(-50, 400, dtype=np.int32).reshape(-1, 1)
    for scale, offset in [(0.25, 0.125), (0.5, -3.0), (0.0625, 0.0)]:
        got = oracle_mod.requant_levels(acc, np.float32(scale), np.float32(offset), False, alpha, bits)
        x = scale * acc.astype(np.float64) + offset
        top = 2 ** bits - 1
        ref = np.floor(top * np.clip(x, 0, alpha) / alpha + 0.5).astype(np.int64)
        assert np.array_equal(got.astype(np.int64), ref)
        assert got.max() <= top and got.min() >= 0
        assert np.all(np.diff(got[:, 0].astype(np.int64)) >= 0)          # monotone for positive scale


def test_requant_per_channel_and_general_inputs_close_to_float64(oracle_mod):
    """Arbitrary scales: the single-precision decision may differ from float64 only where
    qs*x + 0.5 is within rounding distance of an integer."""
    rng = np.random.default_rng(5)
    K = 7
    acc = rng.integers(-200, 5000, (300, K), dtype=np.int32)
    sc = rng.uniform(0.001, 0.01, K).astype(np.float32)
    of = rng.normal(0, 0.5, K).astype(np.float32)
    alpha, bits = 6.0, 3
    got = oracle_mod.requant_levels(acc, sc, of, True, alpha, bits).astype(np.int64)
    x = sc.astype(np.float64) * acc + of.astype(np.float64)
    y = 7 * np.clip(x, 0, alpha) / alpha + 0.5
    ref = np.floor(y).astype(np.int64)
    diff = got != ref
    # what single precision can do: x carries one rounding of an FMA whose terms are |scale*acc| and |offset|,
    # qs one rounding, the last FMA one more - a few units of 2^-24 of those magnitudes.  A level may differ
    # from the float64 decision only if y lies that close to an integer.
    qs = 7.0 / alpha
    window = 2.0 ** -22 * (qs * (np.abs(sc.astype(np.float64) * acc) + np.abs(of.astype(np.float64))) + np.abs(y) + 1.0)
    assert window.max() < 3e-5
    assert np.all(np.abs(y[diff] - np.round(y[diff])) < window[diff])  # only at rounding boundaries
    assert diff.mean() < 1e-3
    # per-layer call equals per-channel call with constant arrays
    a = oracle_mod.requant_levels(acc, np.float32(0.004), np.float32(0.1), False, alpha, bits)
    b = oracle_mod.requant_levels(acc, np.full(K, 0.004, np.float32), np.full(K, 0.1, np.float32), True, alpha, bits)
    assert np.array_equal(a, b)


# ---------------------------------------------------------------- signed weights (Eq. 1a)
@pytest.mark.parametrize("kw,ka", [(1, 1), (1, 4), (2, 2), (3, 2), (4, 4), (5, 3), (2, 5)])
def test_signed_conv_against_library_and_identity(oracle_mod, kw, ka):
    N, C, H, W, K, R, S, st, pad = 2, 21, 7, 6, 5, 3, 3, 2, 1
    a, q = _rand(300 + kw * 4 + ka, N, C, H, W, K, R, S, kw, ka)
    top = 2 ** kw - 1
    got = oracle_mod.conv2d_signed_levels(a, q, kw, st, pad)
    # float64 library convolution with the integer weights 2q - top (exact)
    wq = 2.0 * q.astype(np.float64) - top
    ref = torch.nn.functional.conv2d(torch.from_numpy(a.astype(np.float64)).permute(0, 3, 1, 2),
                                     torch.from_numpy(wq).permute(0, 3, 1, 2), stride=st, padding=pad)
    assert np.array_equal(got.astype(np.float64), ref.permute(0, 2, 3, 1).numpy())
    # identity: 2 * (unsigned product) - top * (window sum of the activations)
    ones = np.ones_like(q)
    wsum = oracle_mod.conv2d_levels(a, ones, st, pad)
    uns = oracle_mod.conv2d_levels(a, q, st, pad)
    assert np.array_equal(got.astype(np.int64), 2 * uns.astype(np.int64) - top * wsum.astype(np.int64))


def test_signed_conv_closed_forms(oracle_mod):
    C, K = 9, 2
    a = np.full((1, 5, 5, C), 3, np.uint8)
    # all weights at the top level -> integer weight +top; at level 0 -> -top; 1-bit -> -1/+1
    for kw in (1, 2, 4):
        top = 2 ** kw - 1
        hi = oracle_mod.conv2d_signed_levels(a, np.full((K, 3, 3, C), top, np.uint8), kw, 1, 0)
        lo = oracle_mod.conv2d_signed_levels(a, np.zeros((K, 3, 3, C), np.uint8), kw, 1, 0)
        assert np.all(hi == top * 3 * 9 * C) and np.all(lo == -top * 3 * 9 * C)
    q = np.zeros((1, 1, 1, 2), np.uint8)
    q[0, 0, 0, 1] = 1                      # weights (-1, +1)
    a2 = np.array([5, 2], np.uint8).reshape(1, 1, 1, 2)
    assert oracle_mod.conv2d_signed_levels(a2, q, 1, 1, 0)[0, 0, 0, 0] == -5 + 2


# ---------------------------------------------------------------- two separate stages (Sec. 4.3)
def test_depthwise_stage_on_hand_fixture(oracle_mod):
    """The hand-computed P of the worked example goes to its hand-computed O."""
    g = read_sections("bd_worked_example_2x3_3x2.txt")
    assert np.array_equal(oracle_mod.depthwise_pow2(g["P"], 2, 2), g["O"])


def test_depthwise_stage_closed_forms(oracle_mod):
    # all-ones P: every window sums the whole kernel, (2^M - 1)(2^K - 1)
    for M, Kb in [(1, 1), (2, 3), (4, 4), (3, 1)]:
        O = oracle_mod.depthwise_pow2(np.ones((5 * M, 7 * Kb), dtype=np.int64), M, Kb)
        assert O.shape == (5, 7) and (O == ((1 << M) - 1) * ((1 << Kb) - 1)).all()
    # a single non-zero entry lands in exactly one output with weight 2^(m+k): catches a
    # transposed kernel, a wrong stride or swapped window axes (M != K on purpose)
    M, Kb, c_o, n = 3, 2, 4, 5
    for (i, m, j, k) in [(0, 0, 0, 0), (3, 2, 4, 1), (1, 2, 2, 0), (2, 0, 3, 1)]:
        P = np.zeros((c_o * M, n * Kb), dtype=np.int64)
        P[i * M + m, j * Kb + k] = 7
        O = oracle_mod.depthwise_pow2(P, M, Kb)
        want = np.zeros((c_o, n), dtype=np.int64)
        want[i, j] = 7 << (m + k)
        assert np.array_equal(O, want)
    with pytest.raises(ValueError):
        oracle_mod.depthwise_pow2(np.zeros((5, 4)), 2, 2)


def test_depthwise_stage_is_lambda_products(oracle_mod):
    """Eq. 13: O = Lambda_w P Lambda_x^T with the block-diagonal coefficient matrices."""
    rng = np.random.default_rng(4130)
    M, Kb, c_o, n = 3, 4, 3, 6
    P = rng.integers(0, 50, (c_o * M, n * Kb))
    Lw = np.kron(np.eye(c_o, dtype=np.int64), (2 ** np.arange(M))[None, :])
    Lx = np.kron(np.eye(n, dtype=np.int64), (2 ** np.arange(Kb))[None, :])
    assert np.array_equal(oracle_mod.depthwise_pow2(P, M, Kb), Lw @ P @ Lx.T)


@pytest.mark.parametrize("kw,ka", [(1, 1), (2, 3), (4, 4), (3, 1), (1, 4), (5, 5), (3, 5)])
def test_partial_products_match_bitwise_and_matrix_forms(oracle_mod, kw, ka):
    N, C, H, W, K, R, S, st, pad = 2, 7, 6, 5, 5, 3, 2, 2, 1
    a, q = _rand(500 + kw * 5 + ka, N, C, H, W, K, R, S, kw, ka)
    planes = oracle_mod.partial_products(a, q, kw, ka, st, pad)
    OH, OW = oracle_mod.out_dims(H, W, R, S, st, pad)
    assert planes.shape == (kw, ka, N, OH, OW, K)
    # bit-by-bit AND/bitcount route (Eq. 2), stored [n][oh][ow][k][m][kk]
    _, bitwise = oracle_mod.bitplane_conv(a, q, kw, ka, st, pad, return_planes=True)
    assert np.array_equal(planes, bitwise.transpose(4, 5, 0, 1, 2, 3))
    # matrix route: P = B_w B_x
    O, P = oracle_mod.bd_matrix_form(a, q, kw, ka, st, pad)
    Pm = oracle_mod.planes_to_matrix(planes)
    assert np.array_equal(Pm, P)
    # and the two stages chained give the direct convolution
    O2 = oracle_mod.depthwise_pow2(Pm, kw, ka)
    assert np.array_equal(O2.T.reshape(N, OH, OW, K), oracle_mod.conv2d_levels(a, q, st, pad))



# ---------------------------------------------------------------- quantisers (Eq. 1a-1c) and aggregation (Eq. 6, 7, 8)
def test_weight_quantiser_hand_fixture(oracle_mod):
    g = read_sections("quantizer_examples.txt")
    W = np.arctanh(g["tanh_tenths"][0] / 10.0)
    for b in (1, 2, 3):
        L = g[f"levels_b{b}"][0]
        assert np.array_equal(oracle_mod.weight_levels(W, b), L)
        assert np.allclose(oracle_mod.quantize_weights(W, b), 2.0 * L / (2 ** b - 1) - 1.0, atol=1e-15)
    # the paper's aggregate example: B = {2, 3}, r = [0, 0] is 0.5 W^2 + 0.5 W^3
    agg = oracle_mod.aggregate_weights(W, [2, 3], [0.0, 0.0])
    assert np.allclose(agg, g["aggregate_b2_b3_equal_strengths_42nds"][0] / 42.0, atol=1e-15)
    assert np.allclose(agg, 0.5 * oracle_mod.quantize_weights(W, 2) + 0.5 * oracle_mod.quantize_weights(W, 3), atol=1e-15)


def test_quantize_b_rounds_half_up(oracle_mod):
    # (2^b - 1) x exactly at .5: up, never to even
    assert oracle_mod.quantize_b(1.0 / 6.0, 2) == pytest.approx(1.0 / 3.0)     # 0.5 -> 1 (to-even would give 0)
    assert oracle_mod.quantize_b(0.5, 2) == pytest.approx(2.0 / 3.0)           # 1.5 -> 2
    assert oracle_mod.quantize_b(2.5 / 7.0, 3) == pytest.approx(3.0 / 7.0)     # 2.5 -> 3 (to-even would give 2)
    assert oracle_mod.quantize_b(0.0, 4) == 0.0 and oracle_mod.quantize_b(1.0, 4) == 1.0
    x = np.linspace(0, 1, 1001)
    for b in range(1, 6):
        q = oracle_mod.quantize_b(x, b)
        assert np.all(np.abs(q - x) <= 0.5 / (2 ** b - 1) + 1e-12)             # nearest level
        assert len(np.unique(q)) == 2 ** b                                     # a uniform staircase of 2^b levels


@pytest.mark.parametrize("b", [1, 2, 3, 4, 5])
def test_weight_quantiser_properties(oracle_mod, b):
    rng = np.random.default_rng(60 + b)
    W = rng.normal(0, 0.7, (4, 3, 3, 5))
    L = oracle_mod.weight_levels(W, b)
    What = oracle_mod.quantize_weights(W, b)
    n = 2 ** b - 1
    assert L.min() >= 0 and L.max() <= n
    assert np.allclose(What, 2.0 * L / n - 1.0, atol=1e-15)
    # the largest |w| maps to an end of the range, and W_hat lies in [-1, 1]
    i = np.unravel_index(np.argmax(np.abs(W)), W.shape)
    assert What[i] == (1.0 if W[i] > 0 else -1.0)
    assert What.min() >= -1.0 and What.max() <= 1.0
    # monotone in w, and within half a step of the normalised tanh (Eq. 1a before rounding)
    order = np.argsort(W.reshape(-1))
    assert np.all(np.diff(L.reshape(-1)[order].astype(int)) >= 0)
    t = np.tanh(W)
    assert np.all(np.abs(What - t / np.abs(t).max()) <= 1.0 / n + 1e-12)
    # invariant to a common sign flip up to the ties: levels mirror
    Lneg = oracle_mod.weight_levels(-W, b)
    assert np.mean(Lneg.astype(int) + L.astype(int) == n) > 0.999
    if b == 1:
        assert np.array_equal(What, np.where(W >= 0, 1.0, -1.0))               # one bit: the sign
    # all-zero weights: defined (normalised value 1/2), no NaN
    Z = oracle_mod.weight_levels(np.zeros(7), b)
    assert np.all(Z == 2 ** (b - 1))


def test_activation_levels_hand_examples_and_float64_definition(oracle_mod):
    import os
    from golden_io import GOLDEN
    rows = [[float(v) for v in l.split()] for l in open(os.path.join(GOLDEN, "requant_examples.txt"))
            if l.strip() and not l.startswith("#") and not l.startswith("[")]
    for bits, alpha, scale, offset, acc, want in rows:
        x = np.float32(scale) * np.float32(acc) + np.float32(offset)           # exact by construction of the fixture
        assert int(oracle_mod.activation_levels([x], float(alpha), int(bits))[0]) == int(want)
    # against Eq. 1b evaluated in float64 on inputs where single precision is exact (multiples of 1/64, alpha a power of two times n)
    for b, alpha in [(1, 1.0), (2, 3.0), (3, 3.5), (4, 7.5), (5, 15.5)]:
        x = (np.arange(-64, 1200) / 64.0).astype(np.float32)
        L = oracle_mod.activation_levels(x, alpha, b)
        ref = oracle_mod.quantize_activations_f64(x, alpha, b)
        assert np.allclose(alpha * L / (2 ** b - 1), ref, atol=1e-12)
        assert np.allclose(oracle_mod.quantize_activations(x, alpha, b), ref, atol=1e-12)
        assert L[0] == 0 and L[-1] == 2 ** b - 1                               # ReLU side and clip side
        assert np.all(np.diff(L.astype(int)) >= 0)
        # idempotent: a quantised value quantises to itself
        lv = np.arange(2 ** b)
        again = oracle_mod.activation_levels((alpha * lv / (2 ** b - 1)).astype(np.float32), alpha, b)
        assert np.array_equal(again, lv)


def test_activation_levels_general_inputs_close_to_float64(oracle_mod):
    rng = np.random.default_rng(5)
    x = np.abs(rng.normal(0, 2.5, 20000)).astype(np.float32) - 0.3
    for b, alpha in [(2, 6.0), (4, 2.37), (5, 6.0)]:
        L = oracle_mod.activation_levels(x, alpha, b).astype(int)
        n = 2 ** b - 1
        ref = np.floor(n * np.clip(x.astype(np.float64), 0, alpha) / alpha + 0.5).astype(int)
        diff = L != ref
        assert diff.mean() < 1e-3                                              # only inputs within an ulp of a tie may differ
        v = n * np.clip(x.astype(np.float64), 0, alpha) / alpha + 0.5
        assert np.all(np.abs(v[diff] - np.round(v[diff])) < 1e-5) and np.all(np.abs(L - ref) <= 1)


def test_softmax_and_gumbel_coefficients(oracle_mod):
    p = oracle_mod.softmax([0.0, 0.0])
    assert np.allclose(p, [0.5, 0.5])
    p = oracle_mod.softmax([-1.0, 1.0])                                        # the paper's second example: close to the larger bitwidth
    assert np.allclose(p, [1 / (1 + np.e ** 2), np.e ** 2 / (1 + np.e ** 2)]) and p[1] > 0.88
    r = np.array([0.3, -1.2, 2.0, 0.0, 0.7])
    p = oracle_mod.softmax(r)
    assert abs(p.sum() - 1) < 1e-15 and np.argmax(p) == 2
    assert np.allclose(oracle_mod.softmax(r + 100.0), p)                       # shift invariance (and no overflow)
    # zero noise at tau = 1 is the plain softmax; small tau tends to the one-hot of argmax(log p + g)
    assert np.allclose(oracle_mod.gumbel_softmax(r, np.zeros(5), 1.0), p)
    gmb = np.array([0.1, 3.0, -0.5, 0.2, 0.0])
    c = oracle_mod.gumbel_softmax(r, gmb, 0.01)
    assert np.argmax(c) == np.argmax(np.log(p) + gmb) and c.max() > 0.999
    c = oracle_mod.gumbel_softmax(r, gmb, 2.0)
    y = (np.log(p) + gmb) / 2.0
    assert np.allclose(c, np.exp(y) / np.exp(y).sum()) and abs(c.sum() - 1) < 1e-15


def test_aggregates_reduce_to_single_quantisers(oracle_mod):
    rng = np.random.default_rng(8)
    W = rng.normal(0, 1, 300)
    X = (np.abs(rng.normal(0, 2, 300)) - 0.2).astype(np.float32)
    # one candidate, or one dominant strength (Eq. 5: the arg max), is the plain quantiser
    assert np.allclose(oracle_mod.aggregate_weights(W, [3], [0.7]), oracle_mod.quantize_weights(W, 3))
    assert np.allclose(oracle_mod.aggregate_weights(W, [1, 2, 3, 4, 5], [0, 0, 80.0, 0, 0]), oracle_mod.quantize_weights(W, 3), atol=1e-12)
    assert np.allclose(oracle_mod.aggregate_activations(X, 6.0, [2, 4], [0.0, 90.0]), oracle_mod.quantize_activations(X, 6.0, 4), atol=1e-12)
    # a convex combination: between the smallest and the largest candidate value
    bits = [1, 2, 3, 4, 5]
    r = rng.normal(0, 1, 5)
    agg = oracle_mod.aggregate_weights(W, bits, r)
    each = np.stack([oracle_mod.quantize_weights(W, b) for b in bits])
    assert np.all(agg <= each.max(0) + 1e-12) and np.all(agg >= each.min(0) - 1e-12)
    assert np.allclose(agg, (oracle_mod.softmax(r)[:, None] * each).sum(0))
    aggx = oracle_mod.aggregate_activations(X, 6.0, bits, r, gumbel=np.zeros(5), tau=1.0)
    eachx = np.stack([oracle_mod.quantize_activations(X, 6.0, b) for b in bits])
    assert np.allclose(aggx, (oracle_mod.softmax(r)[:, None] * eachx).sum(0))
    # linear in the coefficients: Eq. 7 = (sum_i a_i W^i) * (sum_j b_j X^j) needs only these two factors
    assert np.allclose(oracle_mod.aggregate_weights(W, [2, 3], [0.0, 0.0]),
                       0.5 * oracle_mod.quantize_weights(W, 2) + 0.5 * oracle_mod.quantize_weights(W, 3))
