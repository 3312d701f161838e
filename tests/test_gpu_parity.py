"""GPU parity: the HIP path, called through the C-ABI, against the CPU oracle on
the same seeded inputs.  Integer accumulators must be bit-exact; fp32 outputs
within 1e-5 relative."""
import numpy as np
import pytest

import ebs_workloads as wl
import paper_2003_07577_amd as ebs
from gpu_harness import (MUST_ACCEPT, MUST_ACCEPT_LANE, POISON, VARIANT_GEOS, assert_f32_close, conv, pack, run_case,
                         unpack_activations, unpack_weight_pairs, unpack_weights, upload)

pytestmark = pytest.mark.gpu

BITS = wl.PAPER_BITS


def _check(oracle_mod, inp, k_w, k_a, stride, pad, variant=0, tag=""):
    print(f"[case] {tag} variant={variant} kw={k_w} ka={k_a} a={inp['a'].shape} q={inp['q'].shape} "
          f"stride={stride} pad={pad}", flush=True)
    acc, out, d = run_case(inp, k_w, k_a, stride, pad, variant)
    ref = oracle_mod.conv2d_levels(inp["a"], inp["q"], stride, pad)
    assert acc.shape == ref.shape
    assert not (acc == POISON).any(), "unwritten accumulators"
    assert np.array_equal(acc, ref), f"{tag}: {(acc != ref).sum()} of {ref.size} accumulators differ"
    fref = oracle_mod.dequant(ref, inp["scale"], inp["offset"], inp["per_channel"])
    assert not np.isnan(out).any(), "unwritten fp32 outputs"
    assert_f32_close(out, fref, ref, inp["scale"], inp["per_channel"])
    return d


def _variants():
    return list(range(0, ebs.ebs_conv_variant_count() + 1))


# ------------------------------------------------------------------ config 1
def test_config1_tiny(oracle_mod):
    c = wl.config_cases(1)[0]
    inp = wl.make_inputs(c)
    L = c.layer
    d = _check(oracle_mod, inp, c.k_w, c.k_a, L.stride, L.pad, tag=c.tag)
    assert tuple(d["acc"].shape) == (1, 8, 8, 16)      # logical 1x16x8x8, stored NHWC


# ------------------------------------------------------------------ packing
@pytest.mark.parametrize("C", [11, 16, 32, 48, 64, 100, 1000])
@pytest.mark.parametrize("bits", [1, 2, 3, 4, 5])
def test_pack_roundtrip(C, bits):
    import torch
    rng = np.random.default_rng(C * 10 + bits)
    N, H, W, K, R, S = 2, 5, 3, 19, 3, 3
    inp = {"a": rng.integers(0, 256, (N, H, W, C), dtype=np.uint8),      # high bits set on purpose
           "q": rng.integers(0, 256, (K, R, S, C), dtype=np.uint8),
           "scale": np.ones(1, np.float32), "offset": None, "per_channel": False}
    d = upload(inp, bits, bits, 1, 1)
    pack(d)
    torch.cuda.synchronize()
    mask = (1 << bits) - 1
    lv, padbits, border = unpack_activations(d["pa"].cpu().numpy(), N, H, W, C, bits)
    assert np.array_equal(lv, inp["a"] & mask)
    assert not padbits.any(), "channel padding bits must be zero"
    assert not border.any(), "the ring of positions around every image must be zero"
    wv, kpad, cpad = unpack_weights(d["pw"].cpu().numpy(), K, C, R, S, bits)
    assert np.array_equal(wv, inp["q"] & mask)
    assert not kpad.any() and not cpad.any()
    if C <= 16:
        # 3x3 with at most 16 input channels: the two-taps-per-word section holds the same levels
        pv, stray = unpack_weight_pairs(d["pw"].cpu().numpy(), K, C, bits)
        assert np.array_equal(pv, inp["q"] & mask)
        assert not stray.any(), "unused halves and padding channels of the pair section must be zero"
    # plane population counts against numpy
    words = d["pa"].cpu().numpy().view(np.uint32)[:N * (H + 2) * (W + 2) * ((C + 31) // 32) * bits].reshape(-1, bits)
    for j in range(bits):
        pop = int(np.unpackbits(words[:, j].copy().view(np.uint8)).sum())
        assert pop == int(((inp["a"] >> j) & 1).sum())


def test_pack_all_ones_padding_is_zero():
    import torch
    for C in (16, 48, 1000):
        inp = {"a": np.full((1, 3, 3, C), 15, np.uint8), "q": np.full((5, 1, 1, C), 15, np.uint8),
               "scale": np.ones(1, np.float32), "offset": None, "per_channel": False}
        d = upload(inp, 4, 4, 1, 0)
        pack(d)
        torch.cuda.synchronize()
        _, padbits, border = unpack_activations(d["pa"].cpu().numpy(), 1, 3, 3, C, 4)
        assert not padbits.any() and not border.any()
        words = d["pa"].cpu().numpy().view(np.uint32)[:25 * ((C + 31) // 32) * 4].copy()
        assert int(np.unpackbits(words.view(np.uint8)).sum()) == 9 * C * 4


def test_check_levels_flag():
    import torch
    dev = torch.device("cuda:0")
    lv = torch.full((100000,), 3, dtype=torch.uint8, device=dev)
    flag = torch.full((1,), 7, dtype=torch.int32, device=dev)
    ebs.ebs_check_levels(lv, lv.numel(), 2, flag)
    torch.cuda.synchronize()
    assert int(flag.item()) == 0
    lv[77777] = 4
    ebs.ebs_check_levels(lv, lv.numel(), 2, flag)
    torch.cuda.synchronize()
    assert int(flag.item()) != 0


# ------------------------------------------------------------------ all bit pairs, several tiles, ragged tails
GEOS = VARIANT_GEOS


@pytest.mark.parametrize("kw,ka", BITS)
def test_all_bit_pairs_every_variant(oracle_mod, kw, ka):
    import torch
    for gi, (N, C, H, W, K, R, S, st, pad) in enumerate(GEOS):
        inp = wl.random_case(9000 + 100 * gi + 4 * kw + ka, N, C, H, W, K, R, S, st, pad, kw, ka,
                             per_channel=(gi % 2 == 1), with_offset=(gi % 3 == 0))
        ref = oracle_mod.conv2d_levels(inp["a"], inp["q"], st, pad)
        fref = oracle_mod.dequant(ref, inp["scale"], inp["offset"], inp["per_channel"])
        ran = set()
        for v in _variants():
            d = upload(inp, kw, ka, st, pad)
            pack(d)
            g = d["g"]
            launch = lambda: ebs.ebs_mixed_conv2d_variant(v, d["pa"], d["pw"], g["N"], g["C"], g["H"], g["W"], g["K"],
                                                          g["R"], g["S"], st, pad, kw, ka, d["scale"], d["offset"],
                                                          d["per_channel"], d["acc"], d["out"], None, check=False)
            rc = launch()
            torch.cuda.synchronize()
            print(f"[case] geo{gi} kw={kw} ka={ka} variant={v}:{ebs.ebs_conv_variant_name(v)} rc={rc}", flush=True)
            if rc == -5 and v >= 2:
                continue          # this tiling does not take this shape (the must-accept sets are checked below)
            assert rc == 0
            ran.add(ebs.ebs_conv_variant_name(v))
            acc = d["acc"].cpu().numpy()
            assert np.array_equal(acc, ref), (gi, kw, ka, v, int((acc != ref).sum()))
            assert_f32_close(d["out"].cpu().numpy(), fref, ref, inp["scale"], inp["per_channel"])
            # race check: a second launch into re-poisoned outputs must give the same bytes
            first = d["acc"].clone()
            d["acc"].fill_(POISON)
            assert launch() == 0
            torch.cuda.synchronize()
            assert torch.equal(first, d["acc"]), (gi, kw, ka, v, "two launches differ")
        need = set(MUST_ACCEPT[gi]) | (MUST_ACCEPT_LANE[gi] if kw <= 4 and ka <= 4 else set())
        assert need <= ran, f"geo{gi} ({kw},{ka}): tilings that must take this shape did not run: {sorted(need - ran)}"


# ------------------------------------------------------------------ edge cases
def test_edge_shapes(oracle_mod):
    cases = [
        (1, 1, 1, 1, 1, 1, 1, 1, 0, 1, 1),        # smallest possible
        (1, 4, 1, 1, 3, 1, 1, 1, 0, 4, 4),
        (1, 32, 3, 3, 16, 3, 3, 1, 0, 2, 3),      # single output position
        (1, 8, 2, 2, 2, 3, 3, 1, 1, 3, 2),        # filter larger than image (pad makes it fit)
        (5, 31, 1, 9, 7, 1, 3, 2, 0, 1, 4),       # H = 1
        (2, 65, 6, 1, 9, 3, 1, 1, 0, 4, 1),       # W = 1
        (1, 512, 4, 4, 20, 3, 3, 1, 1, 4, 4),     # maximum level product, C=512
    ]
    for i, (N, C, H, W, K, R, S, st, pad, kw, ka) in enumerate(cases):
        inp = wl.random_case(500 + i, N, C, H, W, K, R, S, st, pad, kw, ka)
        _check(oracle_mod, inp, kw, ka, st, pad, tag=f"edge{i}")


def test_all_max_levels_closed_form(oracle_mod):
    """Largest accumulator of the ResNet-18 workload: C=512, 3x3, both 4-bit, all levels 15."""
    C, K = 512, 32
    inp = {"a": np.full((1, 5, 5, C), 15, np.uint8), "q": np.full((K, 3, 3, C), 15, np.uint8),
           "scale": np.array([1.0], np.float32), "offset": None, "per_channel": False}
    acc, out, _ = run_case(inp, 4, 4, 1, 1)
    assert np.all(acc[:, 1:-1, 1:-1, :] == 1036800)
    assert np.all(acc[:, 0, 0, :] == 4 * C * 225)
    assert np.array_equal(out, acc.astype(np.float32))          # scale 1, offset 0: exact


def test_null_f32_output_is_allowed(oracle_mod):
    import torch
    inp = wl.random_case(3, 1, 64, 9, 9, 16, 3, 3, 1, 1, 2, 2)
    d = upload(inp, 2, 2, 1, 1)
    pack(d)
    conv(d, want_f32=False)
    torch.cuda.synchronize()
    assert np.array_equal(d["acc"].cpu().numpy(), oracle_mod.conv2d_levels(inp["a"], inp["q"], 1, 1))
    assert torch.isnan(d["out"]).all()        # untouched


def test_deterministic_and_race_free(oracle_mod):
    """Integer accumulation has one right answer; two runs must be byte-identical."""
    import torch
    inp = wl.random_case(77, 4, 128, 14, 14, 64, 3, 3, 1, 1, 3, 3)
    d = upload(inp, 3, 3, 1, 1)
    pack(d)
    conv(d)
    torch.cuda.synchronize()
    first = d["acc"].clone()
    d["acc"].fill_(POISON)
    conv(d)
    torch.cuda.synchronize()
    assert torch.equal(first, d["acc"])


def test_high_bits_of_levels_are_ignored(oracle_mod):
    inp = wl.random_case(12, 1, 40, 6, 6, 8, 3, 3, 1, 1, 2, 3)
    noisy = dict(inp)
    noisy["a"] = inp["a"] | 0xF8
    noisy["q"] = inp["q"] | 0xFC
    acc, _, _ = run_case(noisy, 2, 3, 1, 1)
    assert np.array_equal(acc, oracle_mod.conv2d_levels(inp["a"], inp["q"], 1, 1))


def test_nondefault_stream(oracle_mod):
    import torch
    inp = wl.random_case(13, 2, 64, 12, 12, 32, 3, 3, 1, 1, 2, 2)
    d = upload(inp, 2, 2, 1, 1)
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    pack(d, s)
    conv(d, 0, s)
    s.synchronize()
    assert np.array_equal(d["acc"].cpu().numpy(), oracle_mod.conv2d_levels(inp["a"], inp["q"], 1, 1))


# ------------------------------------------------------------------ int8 matrix-core comparison path
def test_mfma_i8_comparison_matches_oracle(oracle_mod):
    import torch
    dev = torch.device("cuda:0")
    geos = [  # N, C, H, W, K, R, S, stride, pad
        (2, 64, 20, 20, 40, 3, 3, 1, 1), (3, 96, 9, 11, 130, 3, 3, 2, 1), (1, 32, 13, 7, 5, 1, 1, 1, 0),
        (2, 128, 8, 8, 64, 3, 3, 1, 1), (1, 256, 7, 7, 70, 3, 3, 1, 1), (2, 64, 10, 9, 33, 3, 2, 3, 0),
        (5, 64, 9, 11, 130, 3, 3, 2, 1), (2, 64, 6, 6, 70, 1, 1, 1, 0), (1, 192, 30, 30, 64, 3, 3, 1, 1),
    ]
    for gi, (N, C, H, W, K, R, S, st, pad) in enumerate(geos):
        inp = wl.random_case(4000 + gi, N, C, H, W, K, R, S, st, pad, 4, 4, per_channel=(gi % 2 == 0), with_offset=True)
        print(f"[case] mfma geo{gi}", flush=True)
        OH, OW = ebs.out_dims(H, W, R, S, st, pad)
        a = torch.from_numpy(inp["a"]).to(dev)
        q = torch.from_numpy(inp["q"]).to(dev)
        sc = torch.from_numpy(inp["scale"]).to(dev)
        of = torch.from_numpy(inp["offset"]).to(dev)
        acc = torch.full((N, OH, OW, K), POISON, dtype=torch.int32, device=dev)
        out = torch.full((N, OH, OW, K), float("nan"), dtype=torch.float32, device=dev)
        ebs.ebs_mixed_conv2d_mfma_i8(a, q, N, C, H, W, K, R, S, st, pad, sc, of, inp["per_channel"], acc, out)
        torch.cuda.synchronize()
        ref = oracle_mod.conv2d_levels(inp["a"], inp["q"], st, pad)
        assert np.array_equal(acc.cpu().numpy(), ref), gi
        fref = oracle_mod.dequant(ref, inp["scale"], inp["offset"], inp["per_channel"])
        assert_f32_close(out.cpu().numpy(), fref, ref, inp["scale"], inp["per_channel"])
    # unsupported channel count is an error code, not a crash
    rc = ebs.ebs_mixed_conv2d_mfma_i8(a, q, 1, 16, 4, 4, 8, 3, 3, 1, 1, sc, None, 0, acc, out, None, check=False)
    assert rc == -5
    # full-size deep layers (few output positions, long reductions), with and without fp32
    for c in wl.config_cases(3):
        if (c.k_w, c.k_a) != (4, 4) or c.layer_index not in (3, 6):
            continue
        L = c.layer
        inp = wl.make_inputs(c)
        print(f"[case] mfma {c.tag}", flush=True)
        a = torch.from_numpy(inp["a"]).to(dev)
        q = torch.from_numpy(inp["q"]).to(dev)
        sc = torch.from_numpy(inp["scale"]).to(dev)
        ref = oracle_mod.conv2d_levels(inp["a"], inp["q"], L.stride, L.pad)
        for want_f32 in (True, False):
            acc = torch.full((L.N, L.OH, L.OW, L.K), POISON, dtype=torch.int32, device=dev)
            out = torch.full((L.N, L.OH, L.OW, L.K), float("nan"), dtype=torch.float32, device=dev)
            ebs.ebs_mixed_conv2d_mfma_i8(a, q, L.N, L.C, L.H, L.W, L.K, L.R, L.S, L.stride, L.pad, sc, None, False, acc,
                                         out if want_f32 else None)
            torch.cuda.synchronize()
            assert np.array_equal(acc.cpu().numpy(), ref)
            if want_f32:
                fref = oracle_mod.dequant(ref, inp["scale"], None, False)
                assert_f32_close(out.cpu().numpy(), fref, ref, inp["scale"], False)


# ------------------------------------------------------------------ measurement probes
def test_probes_run_and_report_plausible_rates():
    import torch
    dev = torch.device("cuda:0")
    seed = torch.randint(0, 2 ** 31 - 1, (512,), dtype=torch.int32, device=dev)
    blocks, trips = 512, 200
    sink = torch.zeros(blocks * 256, dtype=torch.int32, device=dev)
    ebs.ebs_probe_and_bcnt(seed, sink, blocks, trips)
    torch.cuda.synchronize()
    assert ebs.ebs_probe_and_bcnt_pairs(blocks, trips) == blocks * 256 * trips * 128
    assert int(sink.max().item()) > 0                      # the counted bits are observable
    n = 1 << 24
    src = torch.arange(n // 4, dtype=torch.int32, device=dev)
    dst = torch.zeros(n // 4, dtype=torch.int32, device=dev)
    ebs.ebs_probe_copy(src, dst, n, 256)
    torch.cuda.synchronize()
    assert torch.equal(src, dst)
    ebs.ebs_probe_copy(None, dst, n, 256)                  # fill variant: writes the pattern 1,2,3,4
    torch.cuda.synchronize()
    assert dst[:8].tolist() == [1, 2, 3, 4, 1, 2, 3, 4]
    assert ebs.ebs_probe_copy(src, dst, 7, 256, check=False) == -3
    assert ebs.ebs_probe_and_bcnt(None, sink, 1, 1, check=False) == -1
