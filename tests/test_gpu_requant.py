"""GPU parity of the fused re-quantising convolution: the next layer's activation
levels (Eq. 1b-1c) must equal the oracle's bit for bit (the rounding decision is taken in
the same single-precision order on both sides), the packed tensor it writes must be a valid
input of the next layer, and a two-layer chain must match the oracle chain."""
import numpy as np
import pytest

import ebs_workloads as wl
import paper_2003_07577_amd as ebs
from gpu_harness import POISON, pack, unpack_activations, upload

pytestmark = pytest.mark.gpu


def _requant_gpu(inp, kw, ka, stride, pad, alpha, k_next):
    import torch
    d = upload(inp, kw, ka, stride, pad)
    pack(d)
    g = d["g"]
    nb = ebs.ebs_packed_activations_bytes(g["N"], g["OH"], g["OW"], g["K"], k_next)
    nxt = torch.full((nb // 4,), POISON, dtype=torch.int32, device=d["a"].device)
    ebs.ebs_mixed_conv2d_requant(d["pa"], d["pw"], g["N"], g["C"], g["H"], g["W"], g["K"], g["R"], g["S"], stride, pad,
                                 kw, ka, d["scale"], d["offset"], d["per_channel"], alpha, k_next, nxt)
    torch.cuda.synchronize()
    return nxt, g


def _check(oracle_mod, inp, kw, ka, stride, pad, alpha, k_next, tag):
    print(f"[case] requant {tag} kw={kw} ka={ka} a={inp['a'].shape} q={inp['q'].shape} s={stride} p={pad} "
          f"alpha={alpha} k_next={k_next}", flush=True)
    nxt, g = _requant_gpu(inp, kw, ka, stride, pad, alpha, k_next)
    acc = oracle_mod.conv2d_levels(inp["a"], inp["q"], stride, pad)
    ref = oracle_mod.requant_levels(acc, inp["scale"], inp["offset"], inp["per_channel"], alpha, k_next)
    lv, padbits, border = unpack_activations(nxt.cpu().numpy(), g["N"], g["OH"], g["OW"], g["K"], k_next)
    nbad = int((lv != ref).sum())
    assert nbad == 0, f"{tag}: {nbad} of {ref.size} levels differ"
    assert not padbits.any(), "channel padding bits of the next layer's words must be zero"
    assert not border.any(), "zero ring of the next layer's packed activations"
    return nxt, ref, g


GEOS = [  # N, C, H, W, K, R, S, stride, pad
    (2, 64, 20, 20, 64, 3, 3, 1, 1),
    (3, 100, 9, 11, 40, 3, 3, 2, 1),      # K not a multiple of 32
    (1, 32, 13, 7, 17, 1, 1, 1, 0),       # 1x1, K < 32
    (2, 128, 8, 8, 130, 3, 3, 1, 1),      # K = 4 words + 2 channels
    (2, 33, 8, 8, 70, 5, 5, 1, 2),        # pad 2: fallback kernel
    (1, 256, 7, 7, 96, 3, 3, 1, 1),       # few positions, long reduction: reduction-split kernel
    (2, 256, 6, 6, 50, 3, 3, 1, 1),       # the same with K ragged against the bytes and words of the packed output
    (1, 128, 9, 9, 7, 3, 3, 2, 1),        # reduction-split, K < 8
    (3, 16, 12, 10, 16, 3, 3, 1, 1),      # 16 input channels: the two-taps-per-word kernel, 16 channel lanes
    (2, 16, 14, 14, 32, 3, 3, 2, 1),      # the same at stride 2 with 32 channel lanes
    (2, 9, 7, 9, 21, 3, 3, 1, 0),         # fewer channels, K ragged, no padding
    (8, 64, 40, 28, 260, 3, 3, 1, 1),     # 8960 positions: the channel-per-lane kernel (unsigned weights), K ragged vs 64 and 32
    (16, 64, 48, 56, 128, 3, 3, 2, 1),    # the same at stride 2
    (8, 256, 34, 32, 64, 1, 1, 1, 0),     # 1x1 with eight reduction words: lane kernel too
    (16, 256, 14, 14, 260, 3, 3, 1, 1),   # 3136 positions, eight words: lane kernel, reduction split among the waves
    (12, 256, 28, 28, 64, 3, 3, 2, 1),    # the same at stride 2 (runs of seven with one- or two-bit activations)
    (48, 512, 7, 7, 64, 1, 1, 1, 0),      # 1x1, sixteen words, 2352 positions: split as well
    (44, 64, 28, 28, 64, 3, 3, 2, 1),     # stride 2, rows of 14 outputs: runs of 4 + 4 + 3 + 3 at three and four activation bits
]


@pytest.mark.parametrize("kw,ka", [(1, 1), (1, 3), (2, 2), (3, 4), (4, 1), (4, 4), (5, 5), (2, 5), (5, 1)])
def test_requant_levels_match_oracle(oracle_mod, kw, ka):
    for gi, (N, C, H, W, K, R, S, st, pad) in enumerate(GEOS):
        inp = wl.random_case(7000 + 10 * gi + kw * 4 + ka, N, C, H, W, K, R, S, st, pad, kw, ka,
                             per_channel=(gi % 2 == 0), with_offset=True)
        # scale the affine map so that the outputs spread over the clip range (and below zero)
        top = C * R * S * (2 ** kw - 1) * (2 ** ka - 1)
        inp["scale"] = (inp["scale"] * np.float32(60.0 / top)).astype(np.float32)
        inp["offset"] = (inp["offset"] * np.float32(10.0) - np.float32(0.5)).astype(np.float32)
        for alpha, k_next in [(6.0, 1 + (gi + kw) % 5), (2.37, 1 + (gi + ka + 1) % 5)]:
            _check(oracle_mod, inp, kw, ka, st, pad, alpha, k_next, f"geo{gi}")


def _f64_levels_and_window(acc, scale, offset, per_channel, alpha, bits):
    """Eq. 1b-1c in float64 on x = scale*acc + offset (scale, offset as the float32 values given), and the
    distance from a rounding boundary within which a single-precision evaluation may decide otherwise."""
    sc = np.asarray(scale, np.float64).reshape(-1)
    of = np.zeros_like(sc) if offset is None else np.asarray(offset, np.float64).reshape(-1)
    if not per_channel:
        sc, of = sc[:1], of[:1]
    n = (1 << bits) - 1
    x = sc * acc.astype(np.float64) + of
    y = n * np.clip(x, 0.0, alpha) / alpha + 0.5
    qs = n / alpha
    window = 2.0 ** -22 * (qs * (np.abs(sc * acc) + np.abs(of)) + np.abs(y) + 1.0)
    return np.floor(y).astype(np.int64), y, window


def test_requant_levels_against_float64_definition(oracle_mod):
    """The fused call's levels against Eq. 1b-1c evaluated in float64, directly (not through the
    single-precision oracle): equal everywhere except where (2^b - 1) x / alpha + 1/2 lies within
    single-precision rounding distance of an integer; such positions are counted and must be rare."""
    total = differing = 0
    for gi, (N, C, H, W, K, R, S, st, pad) in enumerate(GEOS[:6]):
        for (kw, ka) in [(1, 1), (2, 3), (4, 4)]:
            inp = wl.random_case(7700 + 10 * gi + kw * 4 + ka, N, C, H, W, K, R, S, st, pad, kw, ka,
                                 per_channel=(gi % 2 == 0), with_offset=True)
            top = C * R * S * (2 ** kw - 1) * (2 ** ka - 1)
            inp["scale"] = (inp["scale"] * np.float32(60.0 / top)).astype(np.float32)
            inp["offset"] = (inp["offset"] * np.float32(10.0) - np.float32(0.5)).astype(np.float32)
            alpha, k_next = 6.0, 1 + (gi + kw) % 5
            print(f"[case] requant-vs-f64 geo{gi} kw={kw} ka={ka} k_next={k_next}", flush=True)
            nxt, g = _requant_gpu(inp, kw, ka, st, pad, alpha, k_next)
            acc = oracle_mod.conv2d_levels(inp["a"], inp["q"], st, pad)
            lv, _, _ = unpack_activations(nxt.cpu().numpy(), g["N"], g["OH"], g["OW"], g["K"], k_next)
            ref, y, window = _f64_levels_and_window(acc, inp["scale"], inp["offset"], inp["per_channel"], alpha, k_next)
            diff = lv.astype(np.int64) != ref
            assert np.all(np.abs(y[diff] - np.round(y[diff])) < window[diff]), "a level differs away from a rounding boundary"
            assert np.all(np.abs(lv.astype(np.int64) - ref)[diff] == 1)
            total += ref.size
            differing += int(diff.sum())
    print(f"[info] {differing} of {total} levels differ from the float64 decision, all inside the rounding window", flush=True)
    assert differing <= 1e-4 * total


def test_requant_saturation_and_relu(oracle_mod):
    """All outputs above alpha -> top level everywhere; all below zero -> level 0 everywhere."""
    inp = wl.random_case(1, 1, 64, 6, 6, 32, 3, 3, 1, 1, 2, 2)
    inp["scale"] = np.array([1.0], np.float32)
    inp["offset"] = np.array([1000.0], np.float32)
    nxt, ref, g = _check(oracle_mod, inp, 2, 2, 1, 1, 6.0, 3, "saturate")
    assert ref.min() == 7
    inp["offset"] = np.array([-1.0e7], np.float32)
    nxt, ref, g = _check(oracle_mod, inp, 2, 2, 1, 1, 6.0, 3, "relu")
    assert ref.max() == 0


def test_two_layer_chain_without_repacking(oracle_mod):
    """conv1 -> fused re-quantise/pack -> conv2 reading that packed tensor, against the oracle chain."""
    import torch
    N, C, H, W, K1, K2 = 2, 64, 12, 12, 96, 48
    rng = np.random.default_rng(99)
    inp1 = wl.random_case(501, N, C, H, W, K1, 3, 3, 1, 1, 2, 3, per_channel=True, with_offset=True)
    inp1["scale"] = (inp1["scale"] * np.float32(0.02)).astype(np.float32)
    alpha, k_mid = 6.0, 3
    nxt, mid_levels, g1 = _check(oracle_mod, inp1, 2, 3, 1, 1, alpha, k_mid, "chain.l1")
    q2 = wl.draw_levels(rng, (K2, 3, 3, K1), 4)
    ref2 = oracle_mod.conv2d_levels(mid_levels, q2, 2, 1)
    dev = nxt.device
    q2d = torch.from_numpy(q2).to(dev)
    pw2 = torch.empty(ebs.ebs_packed_weights_bytes(K2, K1, 3, 3, 4) // 4, dtype=torch.int32, device=dev)
    ebs.ebs_pack_weights(q2d, K2, K1, 3, 3, 4, pw2)
    OH2, OW2 = ebs.out_dims(H, W, 3, 3, 2, 1)
    acc2 = torch.full((N, OH2, OW2, K2), POISON, dtype=torch.int32, device=dev)
    sc = torch.ones(1, device=dev)
    ebs.ebs_mixed_conv2d(nxt, pw2, N, K1, H, W, K2, 3, 3, 2, 1, 4, k_mid, sc, None, 0, acc2, None)
    torch.cuda.synchronize()
    assert np.array_equal(acc2.cpu().numpy(), ref2)


def test_requant_full_size_resnet18_layers(oracle_mod):
    """Full-size config-3 layers (N=64) through the fused call, a diagonal of bit pairs."""
    for c in wl.config_cases(3):
        if (c.k_w, c.k_a) not in [(1, 1), (2, 2), (4, 4)] or c.layer_index not in (0, 3, 5):
            continue
        inp = wl.make_inputs(c)
        L = c.layer
        top = L.C * 9 * (2 ** c.k_w - 1) * (2 ** c.k_a - 1)
        inp["scale"] = np.array([24.0 / top], np.float32)
        inp["offset"] = np.array([-1.0], np.float32)
        _check(oracle_mod, inp, c.k_w, c.k_a, L.stride, L.pad, 6.0, 2, c.tag)
