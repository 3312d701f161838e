"""GPU parity of the signed-weight form (integer weights 2q - (2^k_w - 1) of Eq. 1a): bit-exact
int32 accumulators against the oracle's direct signed convolution, for every bit pair, on shapes
that exercise the K4 / R4 / P4 arrangements and the per-output fallback, plus the fused
re-quantising call with signed weights."""
import numpy as np
import pytest

import ebs_workloads as wl
import paper_2003_07577_amd as ebs
from gpu_harness import POISON, assert_f32_close, pack, unpack_activations, upload

pytestmark = pytest.mark.gpu

GEOS = [  # N, C, H, W, K, R, S, stride, pad
    (2, 64, 20, 20, 64, 3, 3, 1, 1),       # K4
    (3, 100, 9, 11, 17, 3, 3, 2, 1),       # ragged C and K -> P4
    (2, 256, 7, 7, 70, 3, 3, 1, 1),        # long reduction, few positions -> R4
    (2, 33, 8, 8, 9, 5, 5, 1, 2),          # pad 2 -> per-output kernel
    (4, 128, 6, 6, 40, 1, 1, 1, 0),        # 1x1
    (3, 16, 12, 10, 16, 3, 3, 1, 1),       # 16 input channels -> two taps per word, window sums from the pair words
    (2, 12, 9, 11, 20, 3, 3, 2, 1),        # the same, ragged C and K, stride 2
]
# shapes the heuristic sends to the channel-per-lane kernels (window sums counted on the scalar unit)
LANE_GEOS = [
    (8, 64, 40, 28, 128, 3, 3, 1, 1),      # 8960 positions, runs of 14 / 7
    (16, 64, 48, 56, 64, 3, 3, 2, 1),      # stride 2, rows of 28 outputs
    (44, 64, 28, 28, 64, 3, 3, 2, 1),      # stride 2, rows of 14 outputs: short runs at three and four activation bits
    (16, 256, 14, 14, 260, 3, 3, 1, 1),    # 3136 positions, eight words: reduction split among the waves, K ragged
    (12, 256, 28, 28, 64, 3, 3, 2, 1),     # the same at stride 2
]


@pytest.mark.parametrize("kw,ka", wl.PAPER_BITS)
def test_signed_accumulators_match_oracle(oracle_mod, kw, ka):
    import torch
    for gi, (N, C, H, W, K, R, S, st, pad) in enumerate(GEOS):
        inp = wl.random_case(8100 + 20 * gi + 4 * kw + ka, N, C, H, W, K, R, S, st, pad, kw, ka,
                             per_channel=(gi % 2 == 1), with_offset=True)
        print(f"[case] signed geo{gi} kw={kw} ka={ka}", flush=True)
        d = upload(inp, kw, ka, st, pad)
        pack(d)
        g = d["g"]
        ebs.ebs_mixed_conv2d_signed(d["pa"], d["pw"], g["N"], g["C"], g["H"], g["W"], g["K"], g["R"], g["S"], st, pad,
                                    kw, ka, d["scale"], d["offset"], d["per_channel"], d["acc"], d["out"])
        torch.cuda.synchronize()
        ref = oracle_mod.conv2d_signed_levels(inp["a"], inp["q"], kw, st, pad)
        acc = d["acc"].cpu().numpy()
        assert not (acc == POISON).any()
        assert np.array_equal(acc, ref), (gi, kw, ka, int((acc != ref).sum()))
        fref = oracle_mod.dequant(ref, inp["scale"], inp["offset"], inp["per_channel"])
        assert_f32_close(d["out"].cpu().numpy(), fref, ref, inp["scale"], inp["per_channel"])


def test_one_bit_weights_are_plus_minus_one(oracle_mod):
    """k_w = 1: weights -1/+1; with all activations 1 the result is (#ones - #zeros) of the filter."""
    import torch
    C, K = 64, 32
    rng = np.random.default_rng(4)
    q = rng.integers(0, 2, (K, 3, 3, C), dtype=np.uint8)
    inp = {"a": np.ones((1, 5, 5, C), np.uint8), "q": q, "scale": np.ones(1, np.float32), "offset": None,
           "per_channel": False}
    d = upload(inp, 1, 1, 1, 0)
    pack(d)
    g = d["g"]
    ebs.ebs_mixed_conv2d_signed(d["pa"], d["pw"], 1, C, 5, 5, K, 3, 3, 1, 0, 1, 1, d["scale"], None, 0, d["acc"], d["out"])
    torch.cuda.synchronize()
    acc = d["acc"].cpu().numpy()
    for k in range(K):
        ones = int(q[k].sum())
        assert np.all(acc[..., k] == ones - (9 * C - ones))


def test_signed_requant_full_layer(oracle_mod):
    import torch
    c = [x for x in wl.config_cases(3) if x.layer_index == 1 and (x.k_w, x.k_a) == (2, 3)][0]
    inp = wl.make_inputs(c)
    L = c.layer
    inp["scale"] = np.array([0.004], np.float32)
    inp["offset"] = np.array([1.5], np.float32)
    d = upload(inp, c.k_w, c.k_a, L.stride, L.pad)
    pack(d)
    k_next, alpha = 4, 6.0
    nxt = torch.full((ebs.ebs_packed_activations_bytes(L.N, L.OH, L.OW, L.K, k_next) // 4,), POISON, dtype=torch.int32,
                     device=d["a"].device)
    ebs.ebs_mixed_conv2d_requant(d["pa"], d["pw"], L.N, L.C, L.H, L.W, L.K, L.R, L.S, L.stride, L.pad, c.k_w, c.k_a,
                                 d["scale"], d["offset"], False, alpha, k_next, nxt, signed_weights=True)
    torch.cuda.synchronize()
    acc = oracle_mod.conv2d_signed_levels(inp["a"], inp["q"], c.k_w, L.stride, L.pad)
    ref = oracle_mod.requant_levels(acc, inp["scale"], inp["offset"], False, alpha, k_next)
    lv, padbits, border = unpack_activations(nxt.cpu().numpy(), L.N, L.OH, L.OW, L.K, k_next)
    assert np.array_equal(lv, ref)
    assert ref.min() == 0 and ref.max() >= 8         # the case spans a wide range of levels
    assert not padbits.any() and not border.any()


@pytest.mark.parametrize("kw,ka", [(1, 1), (2, 2), (4, 2), (1, 4), (3, 3), (2, 4), (4, 4), (3, 1)])
def test_signed_lane_shapes_plain_and_requant(oracle_mod, kw, ka):
    """Signed weights on the shapes that take the channel-per-lane kernels: int32 accumulators bit-exact, and the
    fused re-quantising call's levels, zero ring and padding bits."""
    import torch
    for gi, (N, C, H, W, K, R, S, st, pad) in enumerate(LANE_GEOS):
        inp = wl.random_case(8600 + 20 * gi + 4 * kw + ka, N, C, H, W, K, R, S, st, pad, kw, ka,
                             per_channel=(gi % 2 == 0), with_offset=True)
        print(f"[case] signed lane geo{gi} kw={kw} ka={ka}", flush=True)
        d = upload(inp, kw, ka, st, pad)
        pack(d)
        g = d["g"]
        geo = (g["N"], g["C"], g["H"], g["W"], g["K"], g["R"], g["S"], st, pad, kw, ka)
        ebs.ebs_mixed_conv2d_signed(d["pa"], d["pw"], *geo, d["scale"], d["offset"], d["per_channel"], d["acc"], d["out"])
        torch.cuda.synchronize()
        ref = oracle_mod.conv2d_signed_levels(inp["a"], inp["q"], kw, st, pad)
        acc = d["acc"].cpu().numpy()
        assert np.array_equal(acc, ref), (gi, kw, ka, int((acc != ref).sum()))
        fref = oracle_mod.dequant(ref, inp["scale"], inp["offset"], inp["per_channel"])
        assert_f32_close(d["out"].cpu().numpy(), fref, ref, inp["scale"], inp["per_channel"])
        # fused re-quantisation: spread the outputs over and beyond the clip range
        top = C * R * S * (2 ** kw - 1) * (2 ** ka - 1)
        sc = (inp["scale"] * np.float32(40.0 / top)).astype(np.float32)
        of = (inp["offset"] * np.float32(4.0) + np.float32(1.0)).astype(np.float32)
        k_next, alpha = 1 + (gi + kw) % 5, 6.0
        nxt = torch.full((ebs.ebs_packed_activations_bytes(N, g["OH"], g["OW"], K, k_next) // 4,), POISON,
                         dtype=torch.int32, device=d["acc"].device)
        ebs.ebs_mixed_conv2d_requant(d["pa"], d["pw"], *geo, torch.from_numpy(sc).to(nxt.device),
                                     torch.from_numpy(of).to(nxt.device), inp["per_channel"], alpha, k_next, nxt,
                                     signed_weights=True)
        torch.cuda.synchronize()
        want = oracle_mod.requant_levels(ref, sc, of, inp["per_channel"], alpha, k_next)
        lv, padbits, border = unpack_activations(nxt.cpu().numpy(), N, g["OH"], g["OW"], K, k_next)
        assert np.array_equal(lv, want), (gi, kw, ka)
        assert not padbits.any() and not border.any(), (gi, kw, ka)
