"""GPU parity at the size limit of the interface: an output tensor of 2 130 706 432 elements (99.2 % of the
2^31 - 1 the calls accept; 8.5 GB of int32 plus 8.5 GB of fp32), whose byte offsets need 64-bit arithmetic.
The oracle checks it image group by image group so that the host never holds more than a slice."""
import numpy as np
import pytest

import ebs_workloads as wl
import paper_2003_07577_amd as ebs
from gpu_harness import assert_f32_close

pytestmark = pytest.mark.gpu


def test_output_tensor_near_two_to_the_31_elements(oracle_mod):
    import torch
    N, C, H, W, K, kw, ka = 127, 32, 512, 512, 64, 2, 1
    assert N * H * W * K == 2130706432 and (N + 1) * H * W * K > 2 ** 31 - 1
    free, _ = torch.cuda.mem_get_info()
    if free < 24 * 2 ** 30:
        pytest.skip("needs 24 GB of free device memory")
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(20200317)
    a = wl.draw_levels(rng, (N, H, W, C), ka)
    q = wl.draw_levels(rng, (K, 1, 1, C), kw)
    scale = rng.uniform(0.01, 0.2, K).astype(np.float32)
    offset = rng.normal(0, 0.1, K).astype(np.float32)
    print(f"[case] large N={N} C={C} H={H} W={W} K={K} 1x1 w{kw}a{ka}", flush=True)
    da = torch.from_numpy(a).to(dev)
    pa = torch.empty(ebs.ebs_packed_activations_bytes(N, H, W, C, ka) // 4, dtype=torch.int32, device=dev)
    pw = torch.empty(ebs.ebs_packed_weights_bytes(K, C, 1, 1, kw) // 4, dtype=torch.int32, device=dev)
    acc = torch.empty((N, H, W, K), dtype=torch.int32, device=dev)
    out = torch.empty((N, H, W, K), dtype=torch.float32, device=dev)
    ebs.ebs_pack_weights(torch.from_numpy(q).to(dev), K, C, 1, 1, kw, pw)
    ebs.ebs_pack_activations(da, N, H, W, C, ka, pa)
    ebs.ebs_mixed_conv2d(pa, pw, N, C, H, W, K, 1, 1, 1, 0, kw, ka, torch.from_numpy(scale).to(dev),
                         torch.from_numpy(offset).to(dev), True, acc, out)
    torch.cuda.synchronize()
    step = 16
    for n0 in range(0, N, step):
        n1 = min(N, n0 + step)
        ref = oracle_mod.conv2d_levels(a[n0:n1], q, 1, 0)
        got = acc[n0:n1].cpu().numpy()
        assert np.array_equal(got, ref), f"images {n0}..{n1 - 1}: {int((got != ref).sum())} accumulators differ"
        fref = oracle_mod.dequant(ref, scale, offset, True)
        assert_f32_close(out[n0:n1].cpu().numpy(), fref, ref, scale, True)
        print(f"[ok] images {n0}..{n1 - 1}", flush=True)
    # the two-stage form at the same size: 17 GB of partial products, plane offsets beyond 2^32 bytes
    if torch.cuda.mem_get_info()[0] >= 40 * 2 ** 30:
        planes = torch.empty(ebs.ebs_partial_products_bytes(N, H, W, K, 1, 1, 1, 0, kw, ka) // 4, dtype=torch.int32, device=dev)
        acc2 = torch.empty_like(acc)
        ebs.ebs_binary_conv_planes(pa, pw, N, C, H, W, K, 1, 1, 1, 0, kw, ka, planes)
        ebs.ebs_pow2_depthwise(planes, N * H * W, K, kw, ka, torch.from_numpy(scale).to(dev), torch.from_numpy(offset).to(dev),
                               True, acc2, None)
        torch.cuda.synchronize()
        assert torch.equal(acc2, acc)
        pl = planes.view(kw, ka, N, H, W, K)
        ref_planes = oracle_mod.partial_products(a[N - 3:], q, kw, ka, 1, 0)
        assert np.array_equal(pl[:, :, N - 3:].cpu().numpy(), ref_planes)
        del planes, acc2
        print("[ok] two-stage form", flush=True)
    # one more image is beyond the interface's limit and must be refused on the host
    rc = ebs.ebs_mixed_conv2d(pa, pw, N + 1, C, H, W, K, 1, 1, 1, 0, kw, ka, torch.from_numpy(scale).to(dev), None, True,
                              acc, out, check=False)
    assert rc == -3
