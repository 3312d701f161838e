"""Host-only checks of the C-ABI: the library loads, exports every symbol the
header declares, and rejects bad arguments before anything is enqueued (no GPU
is touched: every call below fails validation on the host)."""
import os
import re

import pytest

import paper_2003_07577_amd as ebs

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x10000  # a non-null, 16-byte aligned value; never dereferenced by the host


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(ebs.library_path()):
        from paper_2003_07577_amd.build import build_library
        build_library()
    return ebs.load_library()


def test_every_declared_symbol_is_exported(lib):
    names = set()
    for fn in os.listdir(os.path.join(ROOT, "include")):
        if fn.endswith(".h"):
            text = open(os.path.join(ROOT, "include", fn)).read()
            text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
            names |= set(re.findall(r"\b(ebs_[a-z0-9_]+)\s*\(", text))
    assert {"ebs_pack_weights", "ebs_pack_activations", "ebs_mixed_conv2d"} <= names
    for n in sorted(names):
        assert hasattr(lib, n), f"{n} declared in include/ but not exported"


def test_version_and_status_strings(lib):
    assert ebs.ebs_version() >= 100
    assert ebs.ebs_status_string(0) == "EBS_OK"
    for s in range(-7, 0):
        assert ebs.ebs_status_string(s).startswith("EBS_ERR_")
    assert "unknown" in ebs.ebs_status_string(-99)
    assert ebs.ebs_last_hip_error() == "hipSuccess"      # no launch has failed in this thread


def test_quantizer_calls_reject_bad_arguments_on_the_host(lib):
    ok = dict(w=FAKE, count=64, k=2, levels=FAKE, ws=FAKE)
    q = lambda **kw: (lambda d: ebs.ebs_quantize_weights(d["w"], d["count"], d["k"], d["levels"], d["ws"], check=False))({**ok, **kw})
    assert q(w=None) == -1 and q(levels=None) == -1 and q(ws=None) == -1
    assert q(k=0) == -2 and q(k=9) == -2
    assert q(count=0) == -3
    assert q(w=FAKE + 4) == -4 and q(ws=FAKE + 8) == -4
    a = lambda alpha, k: ebs.ebs_quantize_activations(FAKE, 64, alpha, k, FAKE, check=False)
    assert a(0.0, 2) == -3 and a(float("inf"), 2) == -3 and a(float("nan"), 2) == -3 and a(6.0, 0) == -2
    agg = lambda bits, tau=1.0, g=None, r=FAKE: ebs.ebs_aggregate_weights(FAKE, 64, bits, r, g, tau, FAKE, FAKE, check=False)
    assert agg([]) == -2 and agg([1] * (ebs.MAX_CANDIDATES + 1)) == -2 and agg([0, 2]) == -2 and agg([2, 9]) == -2
    assert agg([2, 3], r=None) == -1
    assert agg([2, 3], tau=0.0, g=FAKE) == -3 and agg([2, 3], tau=-1.0, g=FAKE) == -3
    act = lambda alpha: ebs.ebs_aggregate_activations(FAKE, 64, alpha, [2, 3], FAKE, None, 1.0, FAKE, FAKE, check=False)
    assert act(0.0) == -3 and act(float("nan")) == -3


def test_packed_sizes(lib):
    # activations: N*(H+2)*(W+2) positions x ceil(C/32) words x k_a planes x 4 bytes + 16 slack bytes
    assert ebs.ebs_packed_activations_bytes(64, 56, 56, 64, 4) == 64 * 58 * 58 * 2 * 4 * 4 + 16
    assert ebs.ebs_packed_activations_bytes(1, 8, 8, 16, 2) == 100 * 1 * 2 * 4 + 16
    assert ebs.ebs_packed_activations_bytes(1, 1, 1, 33, 1) == 9 * 2 * 4 + 16
    # weights: K rounded up to 16
    assert ebs.ebs_packed_weights_bytes(64, 64, 3, 3, 1) == 64 * 9 * 2 * 4
    assert ebs.ebs_packed_weights_bytes(1000, 2048, 1, 1, 4) == 1008 * 64 * 4 * 4
    # 3x3 with at most 16 input channels: the ordinary section plus five two-tap words per channel and plane
    assert ebs.ebs_packed_weights_bytes(20, 16, 3, 3, 3) == (32 * 9 * 3 + 32 * 5 * 3) * 4
    assert ebs.ebs_packed_weights_bytes(20, 16, 1, 1, 3) == 32 * 1 * 3 * 4
    assert ebs.ebs_packed_weights_bytes(20, 17, 3, 3, 3) == 32 * 9 * 3 * 4
    for bad in [(0, 8, 8, 16, 2), (1, 8, 8, 16, 0), (1, 8, 8, 16, 6), (1, -1, 8, 16, 2)]:
        assert ebs.ebs_packed_activations_bytes(*bad) == 0
    assert ebs.ebs_packed_weights_bytes(16, 16, 3, 3, 9) == 0
    assert ebs.ebs_packed_weights_bytes(16, 0, 3, 3, 2) == 0


def _conv(**kw):
    d = dict(packed_act=FAKE, packed_wgt=FAKE, N=1, C=16, H=8, W=8, K=16, R=3, S=3, stride=1, pad=1,
             k_w=2, k_a=2, scale=FAKE, offset=None, per_channel=0, acc_out=FAKE, out_f32=FAKE)
    d.update(kw)
    return ebs.ebs_mixed_conv2d(d["packed_act"], d["packed_wgt"], d["N"], d["C"], d["H"], d["W"], d["K"],
                                d["R"], d["S"], d["stride"], d["pad"], d["k_w"], d["k_a"], d["scale"],
                                d["offset"], d["per_channel"], d["acc_out"], d["out_f32"], None, check=False)


def test_conv_argument_errors(lib):
    E = {n: v for n, v in [("NULL", -1), ("BITS", -2), ("SHAPE", -3), ("ALIGN", -4)]}
    assert _conv(packed_act=None) == E["NULL"]
    assert _conv(packed_wgt=None) == E["NULL"]
    assert _conv(scale=None) == E["NULL"]
    assert _conv(acc_out=None) == E["NULL"]
    for k in (0, 6, -1):
        assert _conv(k_w=k) == E["BITS"]
        assert _conv(k_a=k) == E["BITS"]
    # accumulators must fit an int32: 2^17 channels x 25 taps x 31 x 31 does not, 15 x 15 does
    assert _conv(C=1 << 17, H=8, W=8, K=1, R=5, S=5, pad=2, k_w=5, k_a=5) == E["SHAPE"]
    # (the passing shape is given a misaligned pointer so that the call still ends on the host)
    assert _conv(C=1 << 17, H=8, W=8, K=1, R=5, S=5, pad=2, k_w=4, k_a=4, packed_act=FAKE + 4) == E["ALIGN"]
    for bad in [dict(N=0), dict(C=0), dict(H=-2), dict(W=0), dict(K=0), dict(R=0), dict(S=0),
                dict(stride=0), dict(pad=-1), dict(pad=3), dict(H=1, W=1, pad=0),
                dict(N=1 << 20, H=1 << 10, W=1 << 10)]:
        assert _conv(**bad) == E["SHAPE"], bad
    assert _conv(packed_act=FAKE + 4) == E["ALIGN"]
    assert _conv(acc_out=FAKE + 8) == E["ALIGN"]
    assert _conv(out_f32=FAKE + 2) == E["ALIGN"]
    assert _conv(scale=FAKE + 1) == E["ALIGN"]
    with pytest.raises(ebs.EbsError) as ei:
        ebs.ebs_mixed_conv2d(None, FAKE, 1, 16, 8, 8, 16, 3, 3, 1, 1, 2, 2, FAKE, None, 0, FAKE, FAKE)
    assert ei.value.status == -1


def test_position_count_stays_far_below_32_bits(lib):
    """Kernels number output positions in 32 bits and round the last tile up: the interface must refuse shapes
    whose bordered input has 2^29 positions or more (its packed form would pass 2^31 bytes per plane and word),
    which keeps N*OH*OW, at most N*H*W for every filter, far from the 32-bit limit."""
    for (N, H, W) in [(1 << 19, 32, 32), (1, 1 << 15, 1 << 15), (1 << 29, 1, 1)]:
        assert ebs.ebs_packed_activations_bytes(N, H, W, 1, 1) == 0, (N, H, W)
        assert _conv(N=N, H=H, W=W, C=1, K=1, R=1, S=1, pad=0, k_w=1, k_a=1) == -3, (N, H, W)
    # the largest accepted square image of one channel: its position count is below 2^29
    assert ebs.ebs_packed_activations_bytes(1, 23000, 23000, 1, 1) > 0
    assert 23002 * 23002 < 1 << 29


def test_tilings_accept_the_parity_shapes(lib):
    """Which tilings take which shape is host logic: every tiling in the must-accept sets of the every-variant
    parity sweep has to get past the host checks for every bit pair (it then tries to launch, which fails here
    for want of a device; EBS_ERR_UNSUPPORTED, -5, is the answer that must not come)."""
    import torch
    if torch.cuda.is_available():
        pytest.skip("host-only probe with fake pointers: not on a machine with a GPU")
    import sys
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    from gpu_harness import MUST_ACCEPT, MUST_ACCEPT_LANE, VARIANT_GEOS
    names = {ebs.ebs_conv_variant_name(v): v for v in range(ebs.ebs_conv_variant_count() + 1)}
    for gi, (N, C, H, W, K, R, S, st, pad) in enumerate(VARIANT_GEOS):
        for kw in range(1, 6):
            for ka in range(1, 6):
                need = set(MUST_ACCEPT[gi]) | (MUST_ACCEPT_LANE[gi] if kw <= 4 and ka <= 4 else set())
                for name in sorted(need):
                    rc = ebs.ebs_mixed_conv2d_variant(names[name], FAKE, FAKE, N, C, H, W, K, R, S, st, pad, kw, ka,
                                                      FAKE, None, 0, FAKE, FAKE, None, check=False)
                    assert rc != -5, (gi, kw, ka, name)
                # and a tiling that cannot take the shape says so instead of launching
                if pad > 1:
                    for v in range(2, ebs.ebs_conv_variant_count() + 1):
                        assert ebs.ebs_mixed_conv2d_variant(v, FAKE, FAKE, N, C, H, W, K, R, S, st, pad, kw, ka, FAKE,
                                                            None, 0, FAKE, FAKE, None, check=False) == -5


def test_pack_argument_errors(lib):
    assert ebs.ebs_pack_weights(None, 16, 16, 3, 3, 2, FAKE, check=False) == -1
    assert ebs.ebs_pack_weights(FAKE, 16, 16, 3, 3, 2, None, check=False) == -1
    assert ebs.ebs_pack_weights(FAKE, 16, 16, 3, 3, 7, FAKE, check=False) == -2
    assert ebs.ebs_pack_weights(FAKE, 0, 16, 3, 3, 2, FAKE, check=False) == -3
    assert ebs.ebs_pack_weights(FAKE, 16, 16, 3, 3, 2, FAKE + 4, check=False) == -4
    assert ebs.ebs_pack_activations(None, 1, 8, 8, 16, 2, FAKE, check=False) == -1
    assert ebs.ebs_pack_activations(FAKE, 1, 8, 8, 16, 0, FAKE, check=False) == -2
    assert ebs.ebs_pack_activations(FAKE, 1, 8, 0, 16, 2, FAKE, check=False) == -3
    assert ebs.ebs_pack_activations(FAKE + 1, 1, 8, 8, 16, 2, FAKE, check=False) == -4
    assert ebs.ebs_check_levels(None, 10, 2, FAKE, check=False) == -1
    assert ebs.ebs_check_levels(FAKE, 0, 2, FAKE, check=False) == -3
    assert ebs.ebs_check_levels(FAKE, 10, 0, FAKE, check=False) == -2


def test_variant_errors(lib):
    n = ebs.ebs_conv_variant_count()
    assert n >= 1
    assert ebs.ebs_conv_variant_name(0) == "heuristic"
    assert ebs.ebs_conv_variant_name(1) == "naive"
    rc = ebs.ebs_mixed_conv2d_variant(n + 5, FAKE, FAKE, 1, 16, 8, 8, 16, 3, 3, 1, 1, 2, 2, FAKE, None, 0,
                                      FAKE, FAKE, None, check=False)
    assert rc == -5


def test_mfma_argument_errors(lib):
    rc = ebs.ebs_mixed_conv2d_mfma_i8(None, FAKE, 1, 16, 8, 8, 16, 3, 3, 1, 1, FAKE, None, 0, FAKE, FAKE, None,
                                      check=False)
    assert rc == -1
    rc = ebs.ebs_mixed_conv2d_mfma_i8(FAKE, FAKE, 1, 16, 8, 8, 16, 3, 3, 1, 5, FAKE, None, 0, FAKE, FAKE, None,
                                      check=False)
    assert rc == -3


def test_requant_argument_errors(lib):
    def call(**kw):
        d = dict(pa=FAKE, pw=FAKE, N=1, C=16, H=8, W=8, K=16, R=3, S=3, stride=1, pad=1, kw=2, ka=2, sc=FAKE,
                 of=None, pc=0, alpha=6.0, kn=2, nxt=FAKE)
        d.update(kw)
        return ebs.ebs_mixed_conv2d_requant(d["pa"], d["pw"], d["N"], d["C"], d["H"], d["W"], d["K"], d["R"], d["S"],
                                            d["stride"], d["pad"], d["kw"], d["ka"], d["sc"], d["of"], d["pc"],
                                            d["alpha"], d["kn"], d["nxt"], None, check=False)
    assert call(nxt=None) == -1
    assert call(pa=None) == -1
    assert call(kn=0) == -2 and call(kn=6) == -2
    assert call(kw=7) == -2
    assert call(alpha=0.0) == -3 and call(alpha=-1.0) == -3 and call(alpha=float("inf")) == -3
    assert call(alpha=float("nan")) == -3
    assert call(H=0) == -3
    assert call(nxt=FAKE + 8) == -4


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU; asking for more must end with a message, not with a wrong number."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and "--gpus 2" in r.stderr
    assert r.stdout.strip() == ""
