"""The entry point that allocates nothing (ebs_quantize_weights_static: the workspace is a device
array inside the library) against ebs_quantize_weights with a caller-provided workspace: the two
run the same kernels, so the integer levels must be identical.  Two calls in a row share the
library's array; the second is smaller than the first."""
import numpy as np
import pytest

import paper_2003_07577_amd as ebs

pytestmark = pytest.mark.gpu


def _levels(fn, w, bits, dev, **kw):
    import torch
    dw = torch.from_numpy(w).to(dev)
    lv = torch.full((w.size,), 255, dtype=torch.uint8, device=dev)
    fn(dw, w.size, bits, lv, **kw)
    torch.cuda.synchronize()
    return lv.cpu().numpy()


def test_static_workspace_matches_caller_workspace(oracle_mod):
    import torch
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(77)
    # the second tensor is smaller and has a smaller maximum: a stale maximum left in the shared
    # array by the first call would change its levels
    sizes = [(147456, 3.0, 4), (4099, 0.05, 3), (1, 1.0, 1), (36864, 0.7, 5)]
    for n, sigma, bits in sizes:
        w = rng.normal(0, sigma, n).astype(np.float32)
        print(f"[case] quantize_weights_static n={n} sigma={sigma} bits={bits}", flush=True)
        ws = torch.full((ebs.QUANT_WORKSPACE_BYTES // 4,), -1, dtype=torch.int32, device=dev)
        want = _levels(lambda a, c, b, l: ebs.ebs_quantize_weights(a, c, b, l, ws), w, bits, dev)
        got = _levels(ebs.ebs_quantize_weights_static, w, bits, dev)
        assert np.array_equal(got, want), f"n={n}: {int((got != want).sum())} levels differ"
        # and both agree with the oracle away from rounding ties of tanh (the bar of the quantiser tests)
        ref = oracle_mod.weight_levels(w, bits)
        assert (got != ref).mean() < 1e-4


def test_static_workspace_rejects_bad_arguments():
    import torch
    dev = torch.device("cuda:0")
    w = torch.zeros(64, dtype=torch.float32, device=dev)
    lv = torch.zeros(64, dtype=torch.uint8, device=dev)
    assert ebs.ebs_quantize_weights_static(w, ebs.STATIC_MAX_COUNT + 1, 2, lv, check=False) == -3
    assert ebs.ebs_quantize_weights_static(w, 0, 2, lv, check=False) == -3
    assert ebs.ebs_quantize_weights_static(w, 64, 9, lv, check=False) == -2
    assert ebs.ebs_quantize_weights_static(None, 64, 2, lv, check=False) == -1
    assert ebs.ebs_quantize_weights_static(w.data_ptr() + 4, 60, 2, lv, check=False) == -4
