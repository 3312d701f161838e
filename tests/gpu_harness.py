"""Shared helpers for the GPU parity tests: run the hot path through the C-ABI
on cuda:0 and bring results back as numpy.  Nothing here computes the method."""
import numpy as np

import paper_2003_07577_amd as ebs

POISON = -842150451  # 0xCDCDCDCD as int32: an output the kernel forgot to write stands out


def _dev():
    import torch
    assert torch.cuda.is_available(), "GPU test without a GPU"
    return torch.device("cuda:0")


# Shapes of the every-variant parity sweep and, per shape, tilings that must accept it (for every bit pair up
# to five bits); the host test checks the acceptance without a GPU, the GPU test that they ran.
VARIANT_GEOS = [  # N, C, H, W, K, R, S, stride, pad
    (2, 64, 20, 20, 40, 3, 3, 1, 1),      # several pixel tiles, K ragged vs 16
    (3, 100, 9, 11, 17, 3, 3, 2, 1),      # C ragged vs 32, stride 2, odd sizes
    (1, 16, 13, 7, 5, 1, 1, 1, 0),        # 1x1, half-filled word
    (2, 33, 8, 8, 3, 5, 5, 1, 2),         # 5x5 filter, pad 2
    (1, 256, 7, 7, 70, 3, 3, 1, 1),       # deep reduction
    (2, 40, 10, 9, 33, 3, 2, 3, 0),       # asymmetric filter, stride 3, no pad
    (2, 64, 9, 15, 70, 1, 1, 1, 0),       # 1x1, two words, K ragged vs 64
    (2, 128, 16, 18, 64, 1, 1, 2, 0),     # 1x1 stride 2, four words
    (3, 16, 12, 10, 16, 3, 3, 1, 1),      # 16 input channels: two taps per word; several tiles, an image boundary inside one
    (2, 12, 9, 11, 20, 3, 3, 2, 1),       # fewer than 16 input channels, stride 2, K ragged against the 32 channel lanes
    (1, 7, 6, 5, 3, 3, 3, 1, 0),          # no padding, a single partial tile
    (301, 256, 1, 1, 200, 1, 1, 1, 0),    # fully-connected: one position per image, batch and K ragged
    (2, 256, 15, 16, 130, 3, 3, 2, 1),    # deep reduction at stride 2 (rows of 8 outputs), K ragged vs 64
]
MUST_ACCEPT = [
    {"p4.tile32.ch2", "k4.tile16.ch2", "k4.tile16.ch1", "k4.tile32.ch2"},
    {"p4.tile32.ch4", "k4.tile16.ch4", "k4.tile16.ch2", "r4.tile16.ch4"},
    {"p4.tile32.ch1", "k4.tile16.ch1", "k4.tile32.ch1"},
    set(),                                 # pad 2 exceeds the stored zero ring: the per-output kernel only
    {"r4.tile16.ch4", "k4.tile16.ch4", "p4.tile32.ch4"},
    {"p4.tile32.ch2", "k4.tile16.ch2"},
    {"p4.tile32.ch2", "k4.tile16.ch2"},
    {"p4.tile32.ch2", "k4.tile16.ch4"},
    {"pair", "p4.tile32.ch1"},
    {"pair", "p4.tile32.ch1"},
    {"pair", "p4.tile32.ch1"},
    {"p4.tile32.ch4", "k4.tile16.ch4"},
    {"p4.tile32.ch4", "k4.tile16.ch4", "r4.tile16.ch4"},
]
# the channel-per-lane kernel (3x3 and 1x1 filters, bitwidths up to four, an even number of reduction steps):
# shapes whose rows hold a short run
MUST_ACCEPT_LANE = [{"lane.small"}, {"lane.small"}, set(), set(), {"lane.small", "lane.split"}, set(), {"lane.small"},
                    {"lane.small"}, set(), set(), set(), {"lane.big", "lane.small", "lane.split"}, {"lane.small", "lane.split"}]


def unpack_weight_pairs(words, K, C, k_w):
    """Second section of the packed weights of a 3x3 layer with C <= 16: uint32 [k][5][plane] for k < ceil16(K),
    two taps per word (low half | high half << 16): words 0..2 = taps (r,0), (r,1); word 3 = taps (0,2), (1,2);
    word 4 = tap (2,2).  -> levels KRSC rebuilt from it, and every bit that must be zero."""
    kpad = (K + 15) // 16 * 16
    first = kpad * 9 * 1 * k_w
    w = np.asarray(words).view(np.uint32)[first:first + kpad * 5 * k_w].reshape(kpad, 5, k_w)
    halves = [((0, 0), (0, 1)), ((1, 0), (1, 1)), ((2, 0), (2, 1)), ((0, 2), (1, 2)), ((2, 2), None)]
    lv = np.zeros((kpad, 3, 3, 16), np.uint8)
    stray = []
    for t5, (lo, hi) in enumerate(halves):
        for half, tap in enumerate((lo, hi)):
            bits = ((w[:, t5, :, None] >> (np.arange(16, dtype=np.uint32) + 16 * half)) & 1).astype(np.uint8)  # k,plane,c
            if tap is None:
                stray.append(bits.reshape(-1))
                continue
            for i in range(k_w):
                lv[:, tap[0], tap[1], :] |= bits[:, i, :] << i
    stray.append(lv[K:].reshape(-1))
    stray.append(lv[:K, :, :, C:].reshape(-1))
    return lv[:K, :, :, :C], np.concatenate(stray)


def geometry(inp, stride, pad):
    N, H, W, C = inp["a"].shape
    K, R, S, _ = inp["q"].shape
    OH, OW = ebs.out_dims(H, W, R, S, stride, pad)
    return dict(N=N, C=C, H=H, W=W, K=K, R=R, S=S, stride=stride, pad=pad, OH=OH, OW=OW)


def upload(inp, k_w, k_a, stride, pad):
    """Device tensors for one case (levels, packed buffers, scale/offset, outputs)."""
    import torch
    dev = _dev()
    g = geometry(inp, stride, pad)
    d = dict(g=g, k_w=k_w, k_a=k_a)
    d["a"] = torch.from_numpy(inp["a"]).to(dev)
    d["q"] = torch.from_numpy(inp["q"]).to(dev)
    nba = ebs.ebs_packed_activations_bytes(g["N"], g["H"], g["W"], g["C"], k_a)
    nbw = ebs.ebs_packed_weights_bytes(g["K"], g["C"], g["R"], g["S"], k_w)
    assert nba > 0 and nbw > 0
    d["pa"] = torch.full((nba // 4,), POISON, dtype=torch.int32, device=dev)
    d["pw"] = torch.full((nbw // 4,), POISON, dtype=torch.int32, device=dev)
    d["scale"] = torch.from_numpy(np.ascontiguousarray(inp["scale"], dtype=np.float32)).to(dev)
    d["offset"] = None if inp["offset"] is None else torch.from_numpy(
        np.ascontiguousarray(inp["offset"], dtype=np.float32)).to(dev)
    d["per_channel"] = bool(inp["per_channel"])
    shape = (g["N"], g["OH"], g["OW"], g["K"])
    d["acc"] = torch.full(shape, POISON, dtype=torch.int32, device=dev)
    d["out"] = torch.full(shape, float("nan"), dtype=torch.float32, device=dev)
    return d


def pack(d, stream=None):
    g = d["g"]
    ebs.ebs_pack_weights(d["q"], g["K"], g["C"], g["R"], g["S"], d["k_w"], d["pw"], stream)
    ebs.ebs_pack_activations(d["a"], g["N"], g["H"], g["W"], g["C"], d["k_a"], d["pa"], stream)


def conv(d, variant=0, stream=None, want_f32=True):
    g = d["g"]
    ebs.ebs_mixed_conv2d_variant(variant, d["pa"], d["pw"], g["N"], g["C"], g["H"], g["W"], g["K"], g["R"], g["S"],
                                 g["stride"], g["pad"], d["k_w"], d["k_a"], d["scale"], d["offset"],
                                 d["per_channel"], d["acc"], d["out"] if want_f32 else None, stream)


def run_case(inp, k_w, k_a, stride, pad, variant=0):
    """Full hot path on the GPU; returns (acc int32 NHWC, out float32 NHWC, device dict).
    The convolution is launched twice into re-poisoned outputs and the two results must be
    byte-identical: integer accumulation has one right answer, so any run-to-run difference is a race."""
    import torch
    d = upload(inp, k_w, k_a, stride, pad)
    pack(d)
    conv(d, variant)
    torch.cuda.synchronize()
    first_acc, first_out = d["acc"].clone(), d["out"].clone()
    d["acc"].fill_(POISON)
    d["out"].fill_(float("nan"))
    conv(d, variant)
    torch.cuda.synchronize()
    assert torch.equal(first_acc, d["acc"]), "two launches of the same case differ (int32)"
    assert torch.equal(first_out.view(torch.int32), d["out"].view(torch.int32)), "two launches of the same case differ (fp32)"
    return d["acc"].cpu().numpy(), d["out"].cpu().numpy(), d


def assert_f32_close(out, ref, acc_ref, scale, per_channel):
    """|gpu - ref| <= 1e-5 * max(|ref|, |scale*acc|): 1e-5 relative, with the second
    term guarding results that cancel against the offset."""
    sc = np.asarray(scale, dtype=np.float64)
    mag = np.abs(acc_ref.astype(np.float64) * (sc if per_channel else sc.reshape(-1)[0]))
    tol = 1e-5 * np.maximum(np.abs(ref.astype(np.float64)), mag)
    err = np.abs(out.astype(np.float64) - ref.astype(np.float64))
    bad = err > tol
    assert not bad.any(), f"{int(bad.sum())} fp32 outputs beyond 1e-5 relative; worst {err.max()}"


def unpack_activations(words, N, H, W, C, k_a):
    """Test-side inverse of the activation packing: uint32 [word][n][H+2][W+2][plane]
    (one zero position all round every image, a few slack words at the very end)
    -> (levels NHWC, channel-padding bits, border words)."""
    cw = (C + 31) // 32
    Hp, Wp = H + 2, W + 2
    w = np.asarray(words).view(np.uint32)[:N * Hp * Wp * cw * k_a].reshape(cw, N, Hp, Wp, k_a).transpose(1, 2, 3, 0, 4)
    inner = w[:, 1:-1, 1:-1]
    border = np.concatenate([w[:, 0].reshape(-1), w[:, -1].reshape(-1), w[:, :, 0].reshape(-1), w[:, :, -1].reshape(-1)])
    bits = ((inner[..., None] >> np.arange(32, dtype=np.uint32)) & 1).astype(np.uint8)   # n,h,w,word,plane,bit
    lv = np.zeros((N, H, W, cw, 32), np.uint8)
    for j in range(k_a):
        lv |= bits[..., j, :] << j
    full = lv.reshape(N, H, W, cw * 32)
    return full[..., :C], full[..., C:], border


def unpack_weights(words, K, C, R, S, k_w):
    """uint32 [k/16][tap][word][k%16][plane] -> levels KRSC (and the padded remainder).  (3x3 layers with at
    most 16 input channels carry a second section behind this one: unpack_weight_pairs.)"""
    cw = (C + 31) // 32
    kg = (K + 15) // 16
    w = np.asarray(words).view(np.uint32)[:kg * R * S * cw * 16 * k_w].reshape(kg, R * S, cw, 16, k_w)
    bits = ((w[..., None] >> np.arange(32, dtype=np.uint32)) & 1).astype(np.uint8)  # kg,tap,word,kl,plane,bit
    lv = np.zeros((kg, R * S, cw, 16, 32), np.uint8)
    for i in range(k_w):
        lv |= bits[:, :, :, :, i, :] << i
    lv = lv.transpose(0, 3, 1, 2, 4).reshape(kg * 16, R * S, cw * 32)
    return lv[:K, :, :C].reshape(K, R, S, C), lv[K:], lv[:K, :, C:]
