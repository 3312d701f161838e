"""GPU parity on seeded random valid shapes: the fused, signed, re-quantising and two-stage calls against
the oracle on geometries nobody hand-picked (ragged channels, 1-wide images, filters as large as the padded
image, strides up to 3, every bit pair of {1..5}^2 drawn at random)."""
import numpy as np
import pytest

import ebs_workloads as wl
import paper_2003_07577_amd as ebs
from gpu_harness import POISON, assert_f32_close, pack, unpack_activations, upload

pytestmark = pytest.mark.gpu


def _draw_geometry(rng):
    while True:
        R, S = (int(v) for v in rng.choice([1, 1, 2, 3, 3, 3, 5], 2))
        if rng.random() < 0.6:
            S = R
        pad = int(rng.integers(0, min(R, S)))
        stride = int(rng.choice([1, 1, 1, 2, 2, 3]))
        H, W = int(rng.integers(1, 25)), int(rng.integers(1, 25))
        if H + 2 * pad < R or W + 2 * pad < S:
            continue
        N = int(rng.integers(1, 4))
        C = int(rng.choice([1, 3, 16, 31, 32, 33, 64, 96, 100, 128, 160, 256]))
        K = int(rng.choice([1, 2, 7, 8, 15, 16, 17, 31, 32, 33, 40, 64, 65, 100, 128]))
        if N * H * W * C > 400000 or K * R * S * C > 400000:
            continue
        return N, C, H, W, K, R, S, stride, pad


@pytest.mark.parametrize("block", range(12))
def test_random_shapes_all_entry_points(oracle_mod, block):
    import torch
    rng = np.random.default_rng(4242 + block)
    for i in range(12):
        N, C, H, W, K, R, S, st, pad = _draw_geometry(rng)
        kw, ka = int(rng.integers(1, 6)), int(rng.integers(1, 6))
        per_channel = bool(rng.integers(0, 2))
        inp = wl.random_case(int(rng.integers(1 << 30)), N, C, H, W, K, R, S, st, pad, kw, ka,
                             per_channel=per_channel, with_offset=bool(rng.integers(0, 2)))
        tag = f"block{block}.{i} N{N} C{C} H{H} W{W} K{K} R{R} S{S} s{st} p{pad} w{kw} a{ka}"
        print(f"[case] {tag}", flush=True)
        d = upload(inp, kw, ka, st, pad)
        pack(d)
        g = d["g"]
        geo = (g["N"], g["C"], g["H"], g["W"], g["K"], g["R"], g["S"], st, pad, kw, ka)
        ref = oracle_mod.conv2d_levels(inp["a"], inp["q"], st, pad)
        fref = oracle_mod.dequant(ref, inp["scale"], inp["offset"], inp["per_channel"])

        # fused call
        ebs.ebs_mixed_conv2d(d["pa"], d["pw"], *geo, d["scale"], d["offset"], d["per_channel"], d["acc"], d["out"])
        torch.cuda.synchronize()
        assert np.array_equal(d["acc"].cpu().numpy(), ref), tag
        assert_f32_close(d["out"].cpu().numpy(), fref, ref, inp["scale"], inp["per_channel"])

        # signed weights
        d["acc"].fill_(POISON)
        ebs.ebs_mixed_conv2d_signed(d["pa"], d["pw"], *geo, d["scale"], d["offset"], d["per_channel"], d["acc"], None)
        torch.cuda.synchronize()
        assert np.array_equal(d["acc"].cpu().numpy(), oracle_mod.conv2d_signed_levels(inp["a"], inp["q"], kw, st, pad)), tag

        # two stages
        nb = ebs.ebs_partial_products_bytes(N, H, W, K, R, S, st, pad, kw, ka)
        planes = torch.full((nb // 4,), POISON, dtype=torch.int32, device=d["acc"].device)
        d["acc"].fill_(POISON)
        ebs.ebs_binary_conv_planes(d["pa"], d["pw"], *geo, planes)
        ebs.ebs_pow2_depthwise(planes, g["N"] * g["OH"] * g["OW"], K, kw, ka, d["scale"], d["offset"], d["per_channel"],
                               d["acc"], d["out"])
        torch.cuda.synchronize()
        assert np.array_equal(planes.cpu().numpy().reshape(kw, ka, N, g["OH"], g["OW"], K),
                              oracle_mod.partial_products(inp["a"], inp["q"], kw, ka, st, pad)), tag
        assert np.array_equal(d["acc"].cpu().numpy(), ref), tag

        # fused re-quantisation (outputs spread over and beyond the clip range)
        top = max(1, C * R * S * (2 ** kw - 1) * (2 ** ka - 1))
        sc = (inp["scale"] * np.float32(40.0 / top)).astype(np.float32)
        of = (np.zeros_like(sc) if inp["offset"] is None else inp["offset"] * np.float32(5.0)) - np.float32(0.25)
        k_next, alpha = int(rng.integers(1, 6)), float(rng.choice([6.0, 2.37, 1.0]))
        nxt = torch.full((ebs.ebs_packed_activations_bytes(N, g["OH"], g["OW"], K, k_next) // 4,), POISON,
                         dtype=torch.int32, device=d["acc"].device)
        ebs.ebs_mixed_conv2d_requant(d["pa"], d["pw"], *geo, torch.from_numpy(sc).to(nxt.device),
                                     torch.from_numpy(of.astype(np.float32)).to(nxt.device), per_channel, alpha, k_next, nxt)
        torch.cuda.synchronize()
        want = oracle_mod.requant_levels(ref, sc, of.astype(np.float32), per_channel, alpha, k_next)
        lv, padbits, border = unpack_activations(nxt.cpu().numpy(), N, g["OH"], g["OW"], K, k_next)
        assert np.array_equal(lv, want), tag
        assert not padbits.any() and not border.any(), tag


def _draw_lane_or_pair_geometry(rng):
    """Shapes the channel-per-lane kernel (3x3 / 1x1, an even number of 32-channel words) or the
    two-taps-per-word kernel (3x3, at most 16 input and 32 output channels) accept."""
    kind = int(rng.integers(0, 3))
    if kind == 0:        # channel-per-lane, 3x3
        R, C, pad, st = 3, 64 * int(rng.integers(1, 4)), int(rng.integers(0, 2)), int(rng.integers(1, 3))
        K, H, W, N = int(rng.choice([64, 70, 128, 130, 260])), int(rng.integers(5, 24)), int(rng.integers(9, 30)), int(rng.integers(1, 4))
        bits = (int(rng.integers(1, 5)), int(rng.integers(1, 5)))
    elif kind == 1:      # channel-per-lane, 1x1
        R, C, pad, st = 1, 64 * int(rng.integers(1, 7)), 0, int(rng.integers(1, 3))
        K, H, W, N = int(rng.choice([64, 100, 128, 192])), int(rng.integers(4, 20)), int(rng.integers(8, 30)), int(rng.integers(1, 4))
        bits = (int(rng.integers(1, 5)), int(rng.integers(1, 5)))
    else:                # two taps per word
        R, C, pad, st = 3, int(rng.integers(1, 17)), int(rng.integers(0, 2)), int(rng.integers(1, 3))
        K, H, W, N = int(rng.integers(1, 33)), int(rng.integers(3, 30)), int(rng.integers(3, 30)), int(rng.integers(1, 7))
        bits = (int(rng.integers(1, 6)), int(rng.integers(1, 6)))
    return kind, (N, C, H, W, K, R, R, st, pad), bits


@pytest.mark.parametrize("block", range(6))
def test_random_shapes_forced_lane_and_pair_kernels(oracle_mod, block):
    """The heuristic sends only large layers to the channel-per-lane kernel; here it and the two-taps-per-word
    kernel are forced (by variant) on random small shapes and compared with the oracle."""
    import torch
    names = {ebs.ebs_conv_variant_name(v): v for v in range(ebs.ebs_conv_variant_count() + 1)}
    rng = np.random.default_rng(9090 + block)
    ran = {"lane.big": 0, "lane.small": 0, "pair": 0}
    for i in range(10):
        kind, (N, C, H, W, K, R, S, st, pad), (kw, ka) = _draw_lane_or_pair_geometry(rng)
        if H + 2 * pad < R or W + 2 * pad < S:
            continue
        per_channel = bool(rng.integers(0, 2))
        inp = wl.random_case(int(rng.integers(1 << 30)), N, C, H, W, K, R, S, st, pad, kw, ka,
                             per_channel=per_channel, with_offset=bool(rng.integers(0, 2)))
        tag = f"block{block}.{i} N{N} C{C} H{H} W{W} K{K} R{R} s{st} p{pad} w{kw} a{ka}"
        d = upload(inp, kw, ka, st, pad)
        pack(d)
        g = d["g"]
        ref = oracle_mod.conv2d_levels(inp["a"], inp["q"], st, pad)
        fref = oracle_mod.dequant(ref, inp["scale"], inp["offset"], inp["per_channel"])
        for name in (("pair",) if kind == 2 else ("lane.big", "lane.small")):
            print(f"[case] {tag} {name}", flush=True)
            d["acc"].fill_(POISON)
            d["out"].fill_(float("nan"))
            rc = ebs.ebs_mixed_conv2d_variant(names[name], d["pa"], d["pw"], g["N"], g["C"], g["H"], g["W"], g["K"], g["R"],
                                              g["S"], st, pad, kw, ka, d["scale"], d["offset"], d["per_channel"], d["acc"],
                                              d["out"], check=False)
            if rc == -5:
                continue                 # e.g. a row shorter than the kernel's run of positions
            assert rc == 0, (tag, name, rc)
            torch.cuda.synchronize()
            ran[name] += 1
            assert np.array_equal(d["acc"].cpu().numpy(), ref), (tag, name)
            assert_f32_close(d["out"].cpu().numpy(), fref, ref, inp["scale"], inp["per_channel"])
    assert ran["pair"] + ran["lane.big"] + ran["lane.small"] >= 6, ran


@pytest.mark.parametrize("block", range(2))
def test_random_fully_connected_shapes_forced_image_runs(oracle_mod, block):
    """Layers with one output position per image (fully-connected layers as 1x1 convolutions; also 2x2 images at
    stride 2) through the channel-per-lane kernel's runs over images, forced by variant: random batch sizes
    (ragged against the runs of 8 and 4 images), channel counts ragged against the 64 lanes, 8 to 256 reduction
    words (the four waves of a work-group take a quarter each)."""
    import torch
    names = {ebs.ebs_conv_variant_name(v): v for v in range(ebs.ebs_conv_variant_count() + 1)}
    rng = np.random.default_rng(7171 + block)
    ran = {"lane.big": 0, "lane.small": 0}
    for i in range(8):
        C = (2048, 8192)[i] if i < 2 else 256 * int(rng.integers(1, 5))      # 8192: the most words a wave's quarter takes
        N = int(rng.integers(4, 40)) if i < 2 else int(rng.integers(4, 600))
        K = int(rng.integers(1, 300))
        hw, st = (2, 2) if i % 4 == 3 else (1, 1)
        kw, ka = int(rng.integers(1, 5)), int(rng.integers(1, 5))
        inp = wl.random_case(int(rng.integers(1 << 30)), N, C, hw, hw, K, 1, 1, st, 0, kw, ka,
                             per_channel=bool(rng.integers(0, 2)), with_offset=bool(rng.integers(0, 2)))
        tag = f"block{block}.{i} N{N} C{C} HW{hw} K{K} s{st} w{kw} a{ka}"
        d = upload(inp, kw, ka, st, 0)
        pack(d)
        g = d["g"]
        ref = oracle_mod.conv2d_levels(inp["a"], inp["q"], st, 0)
        assert ref.shape[1:3] == (1, 1)
        fref = oracle_mod.dequant(ref, inp["scale"], inp["offset"], inp["per_channel"])
        for name in ("lane.big", "lane.small"):
            print(f"[case] {tag} {name}", flush=True)
            d["acc"].fill_(POISON)
            d["out"].fill_(float("nan"))
            rc = ebs.ebs_mixed_conv2d_variant(names[name], d["pa"], d["pw"], g["N"], g["C"], g["H"], g["W"], g["K"], 1, 1,
                                              st, 0, kw, ka, d["scale"], d["offset"], d["per_channel"], d["acc"],
                                              d["out"], check=False)
            if rc == -5:
                assert N < (8 if name == "lane.big" else 4), (tag, name)      # a batch shorter than one run
                continue
            assert rc == 0, (tag, name, rc)
            torch.cuda.synchronize()
            ran[name] += 1
            assert np.array_equal(d["acc"].cpu().numpy(), ref), (tag, name)
            assert_f32_close(d["out"].cpu().numpy(), fref, ref, inp["scale"], inp["per_channel"])
    assert ran["lane.big"] >= 6 and ran["lane.small"] >= 6, ran


@pytest.mark.parametrize("block", range(2))
def test_random_deep_layers_forced_split_reduction(oracle_mod, block):
    """3x3 layers with 256 or 512 input channels through the channel-per-lane kernel whose four waves split the
    reduction (forced by variant; a wave's quarter starts inside a filter row or wraps into the next one)."""
    import torch
    v = {ebs.ebs_conv_variant_name(i): i for i in range(ebs.ebs_conv_variant_count() + 1)}["lane.split"]
    rng = np.random.default_rng(5151 + block)
    ran = 0
    for i in range(8):
        C, st, pad = int(rng.choice([256, 512])), int(rng.integers(1, 3)), int(rng.integers(0, 2))
        N, H, W = int(rng.integers(1, 4)), int(rng.integers(5, 15)), int(rng.integers(9, 20)) * st
        K = int(rng.choice([40, 64, 70, 128, 200]))
        kw, ka = int(rng.integers(1, 5)), int(rng.integers(1, 5))
        inp = wl.random_case(int(rng.integers(1 << 30)), N, C, H, W, K, 3, 3, st, pad, kw, ka,
                             per_channel=bool(rng.integers(0, 2)), with_offset=bool(rng.integers(0, 2)))
        tag = f"block{block}.{i} N{N} C{C} H{H} W{W} K{K} s{st} p{pad} w{kw} a{ka}"
        print(f"[case] {tag}", flush=True)
        d = upload(inp, kw, ka, st, pad)
        pack(d)
        g = d["g"]
        d["acc"].fill_(POISON)
        d["out"].fill_(float("nan"))
        rc = ebs.ebs_mixed_conv2d_variant(v, d["pa"], d["pw"], g["N"], g["C"], g["H"], g["W"], g["K"], 3, 3, st, pad, kw, ka,
                                          d["scale"], d["offset"], d["per_channel"], d["acc"], d["out"], check=False)
        assert rc == 0, (tag, rc)
        torch.cuda.synchronize()
        ran += 1
        ref = oracle_mod.conv2d_levels(inp["a"], inp["q"], st, pad)
        fref = oracle_mod.dequant(ref, inp["scale"], inp["offset"], inp["per_channel"])
        assert np.array_equal(d["acc"].cpu().numpy(), ref), tag
        assert_f32_close(d["out"].cpu().numpy(), fref, ref, inp["scale"], inp["per_channel"])
    assert ran == 8


@pytest.mark.parametrize("ka", [3, 4])
def test_stride2_rows_of_every_length_forced_lane_kernels(oracle_mod, ka):
    """Stride 2 with three- or four-bit activations: the channel-per-lane kernels cover an output row with runs of
    four and three positions (a short run leaves its first position out), or move the last run left where the row
    is too short for that.  Every row length from 4 to 17, unsplit and split reduction, both paddings."""
    import torch
    names = {ebs.ebs_conv_variant_name(v): v for v in range(ebs.ebs_conv_variant_count() + 1)}
    for OW in range(4, 18):
        pad = OW % 2
        W = 2 * (OW - 1) + 3 - 2 * pad
        kw = 1 + OW % 4
        inp = wl.random_case(8800 + 20 * ka + OW, 2, 256, 7, W, 70, 3, 3, 2, pad, kw, ka, per_channel=bool(OW & 1),
                             with_offset=True)
        d = upload(inp, kw, ka, 2, pad)
        pack(d)
        g = d["g"]
        assert g["OW"] == OW
        ref = oracle_mod.conv2d_levels(inp["a"], inp["q"], 2, pad)
        fref = oracle_mod.dequant(ref, inp["scale"], inp["offset"], inp["per_channel"])
        for name in ("lane.small", "lane.split"):
            print(f"[case] OW={OW} pad={pad} kw={kw} ka={ka} {name}", flush=True)
            d["acc"].fill_(POISON)
            d["out"].fill_(float("nan"))
            rc = ebs.ebs_mixed_conv2d_variant(names[name], d["pa"], d["pw"], g["N"], g["C"], g["H"], g["W"], g["K"], 3, 3,
                                              2, pad, kw, ka, d["scale"], d["offset"], d["per_channel"], d["acc"],
                                              d["out"], check=False)
            assert rc == 0, (OW, name, rc)
            torch.cuda.synchronize()
            assert np.array_equal(d["acc"].cpu().numpy(), ref), (OW, name)
            assert_f32_close(d["out"].cpu().numpy(), fref, ref, inp["scale"], inp["per_channel"])
