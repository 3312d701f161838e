"""GPU parity of the literal two-stage form (Sec. 4.3): stage 1 (the partial products P of the
binary convolution, Eq. 13) bit-exact against the oracle's plane-by-plane binary convolutions,
stage 2 (power-of-two depthwise recombination, Eq. 14, plus scale/offset) against the oracle's
strided depthwise convolution over the paper's P matrix, and the chain against the fused call."""
import numpy as np
import pytest

import ebs_workloads as wl
import paper_2003_07577_amd as ebs
from gpu_harness import POISON, assert_f32_close, pack, upload

pytestmark = pytest.mark.gpu

GEOS = [  # N, C, H, W, K, R, S, stride, pad
    (2, 64, 20, 20, 40, 3, 3, 1, 1),       # several position tiles, K ragged vs the channel block
    (3, 100, 9, 11, 17, 3, 3, 2, 1),       # ragged C (single-word chunks) and K, stride 2
    (1, 128, 13, 7, 70, 1, 1, 1, 0),       # 1x1, four-word chunks
    (2, 33, 8, 8, 9, 5, 5, 1, 2),          # pad 2 -> per-output kernel
    (2, 40, 10, 9, 33, 3, 2, 3, 0),        # asymmetric filter, stride 3; odd output count (scalar stage 2)
]


def _planes_buffer(g, kw, ka):
    import torch
    nb = ebs.ebs_partial_products_bytes(g["N"], g["H"], g["W"], g["K"], g["R"], g["S"], g["stride"], g["pad"], kw, ka)
    assert nb == g["N"] * g["OH"] * g["OW"] * g["K"] * kw * ka * 4
    return torch.full((nb // 4,), POISON, dtype=torch.int32, device="cuda:0")


def _two_stage(d, kw, ka, st, pad):
    import torch
    g = d["g"]
    planes = _planes_buffer(g, kw, ka)
    ebs.ebs_binary_conv_planes(d["pa"], d["pw"], g["N"], g["C"], g["H"], g["W"], g["K"], g["R"], g["S"], st, pad,
                               kw, ka, planes)
    ebs.ebs_pow2_depthwise(planes, g["N"] * g["OH"] * g["OW"], g["K"], kw, ka, d["scale"], d["offset"],
                           d["per_channel"], d["acc"], d["out"])
    torch.cuda.synchronize()
    return planes.cpu().numpy().reshape(kw, ka, g["N"], g["OH"], g["OW"], g["K"])


@pytest.mark.parametrize("kw,ka", wl.PAPER_BITS)
def test_two_stage_matches_oracle(oracle_mod, kw, ka):
    for gi, (N, C, H, W, K, R, S, st, pad) in enumerate(GEOS):
        inp = wl.random_case(7300 + 20 * gi + 4 * kw + ka, N, C, H, W, K, R, S, st, pad, kw, ka,
                             per_channel=(gi % 2 == 0), with_offset=(gi % 3 != 1))
        print(f"[case] two-stage geo{gi} kw={kw} ka={ka}", flush=True)
        d = upload(inp, kw, ka, st, pad)
        pack(d)
        planes = _two_stage(d, kw, ka, st, pad)
        assert not (planes == POISON).any(), "unwritten partial products"
        ref_planes = oracle_mod.partial_products(inp["a"], inp["q"], kw, ka, st, pad)
        assert np.array_equal(planes, ref_planes), (gi, kw, ka, int((planes != ref_planes).sum()))
        # stage 2 against the strided depthwise convolution over the paper's P matrix
        g = d["g"]
        O = oracle_mod.depthwise_pow2(oracle_mod.planes_to_matrix(ref_planes), kw, ka)
        ref = O.T.reshape(g["N"], g["OH"], g["OW"], g["K"])
        acc = d["acc"].cpu().numpy()
        assert np.array_equal(acc, ref), (gi, kw, ka, int((acc != ref).sum()))
        assert np.array_equal(ref, oracle_mod.conv2d_levels(inp["a"], inp["q"], st, pad))
        fref = oracle_mod.dequant(ref.astype(np.int32), inp["scale"], inp["offset"], inp["per_channel"])
        assert_f32_close(d["out"].cpu().numpy(), fref, ref, inp["scale"], inp["per_channel"])


@pytest.mark.parametrize("kw,ka,positions,K", [(2, 3, 37, 5), (4, 4, 64, 32), (1, 1, 3, 1), (3, 2, 1000, 12), (4, 1, 129, 7), (5, 5, 50, 6), (2, 5, 31, 3)])
def test_depthwise_stage_alone_on_arbitrary_planes(oracle_mod, kw, ka, positions, K):
    """Stage 2 does not depend on where P came from: random int32 planes (values as large as a
    C*R*S = 4608 reduction gives), vector and scalar paths, per-channel scales."""
    import torch
    rng = np.random.default_rng(100 * kw + 10 * ka + K)
    planes = rng.integers(0, 4609, (kw, ka, positions, K)).astype(np.int32)
    scale = rng.uniform(0.01, 0.2, K).astype(np.float32)
    offset = rng.normal(0, 0.1, K).astype(np.float32)
    dev = "cuda:0"
    dp = torch.from_numpy(planes).to(dev)
    acc = torch.full((positions, K), POISON, dtype=torch.int32, device=dev)
    out = torch.full((positions, K), float("nan"), dtype=torch.float32, device=dev)
    ebs.ebs_pow2_depthwise(dp, positions, K, kw, ka, torch.from_numpy(scale).to(dev), torch.from_numpy(offset).to(dev),
                           True, acc, out)
    torch.cuda.synchronize()
    O = oracle_mod.depthwise_pow2(oracle_mod.planes_to_matrix(planes), kw, ka)      # (K, positions)
    ref = np.ascontiguousarray(O.T).astype(np.int32)
    assert np.array_equal(acc.cpu().numpy(), ref)
    fref = oracle_mod.dequant(ref, scale, offset, True)
    assert_f32_close(out.cpu().numpy(), fref, ref, scale, True)
    # without the fp32 output and with a single scale
    acc2 = torch.full((positions, K), POISON, dtype=torch.int32, device=dev)
    ebs.ebs_pow2_depthwise(dp, positions, K, kw, ka, torch.from_numpy(scale[:1].copy()).to(dev), None, False, acc2, None)
    torch.cuda.synchronize()
    assert np.array_equal(acc2.cpu().numpy(), ref)


def test_two_stage_equals_fused_on_a_full_size_layer(oracle_mod):
    """ResNet-18-shaped layer at the benchmark's batch size: both stages at full size, planes compared
    in full with the oracle, the chain with the fused kernel."""
    import torch
    case = [c for c in wl.config_cases(3) if c.layer.C == 128 and c.layer.stride == 1 and (c.k_w, c.k_a) == (2, 3)][0]
    inp = wl.make_inputs(case)
    L = case.layer
    print(f"[case] two-stage full size {case.tag}", flush=True)
    d = upload(inp, 2, 3, L.stride, L.pad)
    pack(d)
    planes = _two_stage(d, 2, 3, L.stride, L.pad)
    ref_planes = oracle_mod.partial_products(inp["a"], inp["q"], 2, 3, L.stride, L.pad)
    assert np.array_equal(planes, ref_planes)
    acc_two = d["acc"].cpu().numpy().copy()
    out_two = d["out"].cpu().numpy().copy()
    g = d["g"]
    d["acc"].fill_(POISON)
    ebs.ebs_mixed_conv2d(d["pa"], d["pw"], g["N"], g["C"], g["H"], g["W"], g["K"], g["R"], g["S"], L.stride, L.pad,
                         2, 3, d["scale"], d["offset"], d["per_channel"], d["acc"], d["out"])
    torch.cuda.synchronize()
    assert np.array_equal(acc_two, d["acc"].cpu().numpy())
    assert np.array_equal(out_two, d["out"].cpu().numpy())       # same fmaf on the same integers
    assert np.array_equal(acc_two, oracle_mod.conv2d_levels(inp["a"], inp["q"], L.stride, L.pad))


def test_two_stage_argument_errors():
    import torch
    dev = "cuda:0"
    buf = torch.zeros(1024, dtype=torch.int32, device=dev)
    sc = torch.ones(1, dtype=torch.float32, device=dev)
    assert ebs.ebs_pow2_depthwise(None, 4, 4, 2, 2, sc, None, False, buf, None, check=False) == -1
    assert ebs.ebs_pow2_depthwise(buf, 4, 4, 6, 2, sc, None, False, buf, None, check=False) == -2
    assert ebs.ebs_pow2_depthwise(buf, 0, 4, 2, 2, sc, None, False, buf, None, check=False) == -3
    assert ebs.ebs_pow2_depthwise(buf.data_ptr() + 4, 4, 4, 2, 2, sc, None, False, buf, None, check=False) == -4
    assert ebs.ebs_binary_conv_planes(buf, buf, 1, 16, 8, 8, 16, 3, 3, 1, 1, 2, 2, None, check=False) == -1
    assert ebs.ebs_binary_conv_planes(buf, buf, 1, 16, 8, 8, 16, 3, 3, 1, 1, 0, 2, buf, check=False) == -2
    assert ebs.ebs_partial_products_bytes(1, 8, 8, 16, 3, 3, 1, 1, 2, 6) == 0
    assert ebs.ebs_partial_products_bytes(1, 2, 2, 16, 5, 5, 1, 1, 2, 2) == 0
