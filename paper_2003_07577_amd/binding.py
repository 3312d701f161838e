"""ctypes binding with the same names as the C-ABI (include/ebs.h).

Arguments are torch tensors (device memory) or raw integer device pointers;
nothing is computed here.  If the shared library has not been built the first
call raises: there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os

_PKG = os.path.dirname(os.path.abspath(__file__))
# EBS_LIBRARY_PATH: load another build of the same library (the host-sanitized one of the test suite)
_LIB_PATH = os.environ.get("EBS_LIBRARY_PATH") or os.path.join(_PKG, "libebs.so")
_lib = None

_vp = ctypes.c_void_p
_ci = ctypes.c_int


class EbsError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        detail = f" [{ebs_last_hip_error()}]" if status == -6 else ""
        super().__init__(f"{what}: {ebs_status_string(status)} ({status}){detail}")


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Loads libebs.so; raises if it is missing (build it with build.py / __graft_entry__.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise FileNotFoundError(
                f"{_LIB_PATH} is not built; run `python -m paper_2003_07577_amd.build` "
                "(there is no non-HIP fallback)")
        # One HIP runtime per process: PyTorch ships its own libamdhip64 and asks for it by
        # file name, so it must be loaded before libebs.so (which asks by soname and then
        # shares it).  In the other order two runtimes end up loaded and kernels of the
        # second one fail with hipErrorNoDevice on pointers of the first.
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        lib = ctypes.CDLL(_LIB_PATH)
        lib.ebs_version.restype = _ci
        lib.ebs_status_string.restype = ctypes.c_char_p
        lib.ebs_status_string.argtypes = [_ci]
        lib.ebs_last_hip_error.restype = ctypes.c_char_p
        lib.ebs_last_hip_error.argtypes = []
        lib.ebs_packed_weights_bytes.restype = ctypes.c_size_t
        lib.ebs_packed_weights_bytes.argtypes = [_ci] * 5
        lib.ebs_packed_activations_bytes.restype = ctypes.c_size_t
        lib.ebs_packed_activations_bytes.argtypes = [_ci] * 5
        lib.ebs_pack_weights.restype = _ci
        lib.ebs_pack_weights.argtypes = [_vp] + [_ci] * 5 + [_vp, _vp]
        lib.ebs_pack_activations.restype = _ci
        lib.ebs_pack_activations.argtypes = [_vp] + [_ci] * 5 + [_vp, _vp]
        conv_tail = [_vp, _vp] + [_ci] * 11 + [_vp, _vp, _ci, _vp, _vp, _vp]
        lib.ebs_mixed_conv2d.restype = _ci
        lib.ebs_mixed_conv2d.argtypes = conv_tail
        lib.ebs_mixed_conv2d_variant.restype = _ci
        lib.ebs_mixed_conv2d_variant.argtypes = [_ci] + conv_tail
        lib.ebs_mixed_conv2d_requant.restype = _ci
        lib.ebs_mixed_conv2d_requant.argtypes = [_vp, _vp] + [_ci] * 12 + [_vp, _vp, _ci, ctypes.c_float, _ci, _vp, _vp]
        lib.ebs_mixed_conv2d_signed.restype = _ci
        lib.ebs_mixed_conv2d_signed.argtypes = conv_tail
        lib.ebs_partial_products_bytes.restype = ctypes.c_size_t
        lib.ebs_partial_products_bytes.argtypes = [_ci] * 10
        lib.ebs_binary_conv_planes.restype = _ci
        lib.ebs_binary_conv_planes.argtypes = [_vp, _vp] + [_ci] * 11 + [_vp, _vp]
        lib.ebs_pow2_depthwise.restype = _ci
        lib.ebs_pow2_depthwise.argtypes = [_vp, ctypes.c_longlong, _ci, _ci, _ci, _vp, _vp, _ci, _vp, _vp, _vp]
        _sz, _fl = ctypes.c_size_t, ctypes.c_float
        lib.ebs_quantize_weights.restype = _ci
        lib.ebs_quantize_weights.argtypes = [_vp, _sz, _ci, _vp, _vp, _vp]
        lib.ebs_quantize_weights_static.restype = _ci
        lib.ebs_quantize_weights_static.argtypes = [_vp, _sz, _ci, _vp, _vp]
        lib.ebs_quantize_activations.restype = _ci
        lib.ebs_quantize_activations.argtypes = [_vp, _sz, _fl, _ci, _vp, _vp]
        lib.ebs_aggregate_weights.restype = _ci
        lib.ebs_aggregate_weights.argtypes = [_vp, _sz, ctypes.POINTER(_ci), _ci, _vp, _vp, _fl, _vp, _vp, _vp]
        lib.ebs_aggregate_activations.restype = _ci
        lib.ebs_aggregate_activations.argtypes = [_vp, _sz, _fl, ctypes.POINTER(_ci), _ci, _vp, _vp, _fl, _vp, _vp, _vp]
        lib.ebs_conv_variant_count.restype = _ci
        lib.ebs_conv_variant_name.restype = ctypes.c_char_p
        lib.ebs_conv_variant_name.argtypes = [_ci]
        lib.ebs_mixed_conv2d_mfma_i8.restype = _ci
        lib.ebs_mixed_conv2d_mfma_i8.argtypes = [_vp, _vp] + [_ci] * 9 + [_vp, _vp, _ci, _vp, _vp, _vp]
        lib.ebs_check_levels.restype = _ci
        lib.ebs_check_levels.argtypes = [_vp, ctypes.c_size_t, _ci, _vp, _vp]
        lib.ebs_probe_and_bcnt.restype = _ci
        lib.ebs_probe_and_bcnt.argtypes = [_vp, _vp, _ci, _ci, _vp]
        lib.ebs_probe_and_bcnt_pairs.restype = ctypes.c_longlong
        lib.ebs_probe_and_bcnt_pairs.argtypes = [_ci, _ci]
        lib.ebs_probe_copy.restype = _ci
        lib.ebs_probe_copy.argtypes = [_vp, _vp, ctypes.c_size_t, _ci, _vp]
        _lib = lib
    return _lib


def _ptr(x):
    """Device pointer of a tensor-like (anything with data_ptr()), an int, or None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()


def _stream(stream):
    if stream is None:
        return None
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream     # torch.cuda.Stream


def _check(rc: int, what: str):
    if rc != 0:
        raise EbsError(rc, what)


def out_dims(H, W, R, S, stride, pad):
    return (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1


def ebs_version() -> int:
    return load_library().ebs_version()


def ebs_status_string(status: int) -> str:
    return load_library().ebs_status_string(status).decode()


def ebs_last_hip_error() -> str:
    return load_library().ebs_last_hip_error().decode()


def ebs_packed_weights_bytes(K, C, R, S, k_w) -> int:
    return load_library().ebs_packed_weights_bytes(K, C, R, S, k_w)


def ebs_packed_activations_bytes(N, H, W, C, k_a) -> int:
    return load_library().ebs_packed_activations_bytes(N, H, W, C, k_a)


def ebs_pack_weights(levels_krsc, K, C, R, S, k_w, packed, stream=None, check=True) -> int:
    rc = load_library().ebs_pack_weights(_ptr(levels_krsc), K, C, R, S, k_w, _ptr(packed), _stream(stream))
    if check:
        _check(rc, "ebs_pack_weights")
    return rc


def ebs_pack_activations(levels_nhwc, N, H, W, C, k_a, packed, stream=None, check=True) -> int:
    rc = load_library().ebs_pack_activations(_ptr(levels_nhwc), N, H, W, C, k_a, _ptr(packed), _stream(stream))
    if check:
        _check(rc, "ebs_pack_activations")
    return rc


def ebs_mixed_conv2d(packed_act, packed_wgt, N, C, H, W, K, R, S, stride, pad, k_w, k_a,
                     scale, offset, per_channel, acc_out, out_f32, stream=None, check=True) -> int:
    rc = load_library().ebs_mixed_conv2d(
        _ptr(packed_act), _ptr(packed_wgt), N, C, H, W, K, R, S, stride, pad, k_w, k_a,
        _ptr(scale), _ptr(offset), int(bool(per_channel)), _ptr(acc_out), _ptr(out_f32), _stream(stream))
    if check:
        _check(rc, "ebs_mixed_conv2d")
    return rc


def ebs_mixed_conv2d_signed(packed_act, packed_wgt, N, C, H, W, K, R, S, stride, pad, k_w, k_a,
                            scale, offset, per_channel, acc_out, out_f32, stream=None, check=True) -> int:
    rc = load_library().ebs_mixed_conv2d_signed(
        _ptr(packed_act), _ptr(packed_wgt), N, C, H, W, K, R, S, stride, pad, k_w, k_a,
        _ptr(scale), _ptr(offset), int(bool(per_channel)), _ptr(acc_out), _ptr(out_f32), _stream(stream))
    if check:
        _check(rc, "ebs_mixed_conv2d_signed")
    return rc


def ebs_partial_products_bytes(N, H, W, K, R, S, stride, pad, k_w, k_a) -> int:
    return load_library().ebs_partial_products_bytes(N, H, W, K, R, S, stride, pad, k_w, k_a)


def ebs_binary_conv_planes(packed_act, packed_wgt, N, C, H, W, K, R, S, stride, pad, k_w, k_a,
                           planes, stream=None, check=True) -> int:
    rc = load_library().ebs_binary_conv_planes(
        _ptr(packed_act), _ptr(packed_wgt), N, C, H, W, K, R, S, stride, pad, k_w, k_a,
        _ptr(planes), _stream(stream))
    if check:
        _check(rc, "ebs_binary_conv_planes")
    return rc


def ebs_pow2_depthwise(planes, positions, K, k_w, k_a, scale, offset, per_channel, acc_out, out_f32,
                       stream=None, check=True) -> int:
    rc = load_library().ebs_pow2_depthwise(
        _ptr(planes), positions, K, k_w, k_a, _ptr(scale), _ptr(offset), int(bool(per_channel)),
        _ptr(acc_out), _ptr(out_f32), _stream(stream))
    if check:
        _check(rc, "ebs_pow2_depthwise")
    return rc


QUANT_WORKSPACE_BYTES = 256     # EBS_QUANT_WORKSPACE_BYTES
STATIC_MAX_COUNT = 1 << 31      # EBS_STATIC_MAX_COUNT
MAX_CANDIDATES = 8              # EBS_MAX_CANDIDATES


def _int_array(values):
    values = [int(v) for v in values]
    return (ctypes.c_int * max(len(values), 1))(*values), len(values)


def ebs_quantize_weights(w, count, k_w, levels, workspace, stream=None, check=True) -> int:
    rc = load_library().ebs_quantize_weights(_ptr(w), count, k_w, _ptr(levels), _ptr(workspace), _stream(stream))
    if check:
        _check(rc, "ebs_quantize_weights")
    return rc


def ebs_quantize_weights_static(w, count, k_w, levels, stream=None, check=True) -> int:
    rc = load_library().ebs_quantize_weights_static(_ptr(w), count, k_w, _ptr(levels), _stream(stream))
    if check:
        _check(rc, "ebs_quantize_weights_static")
    return rc


def ebs_quantize_activations(x, count, alpha, k_a, levels, stream=None, check=True) -> int:
    rc = load_library().ebs_quantize_activations(_ptr(x), count, alpha, k_a, _ptr(levels), _stream(stream))
    if check:
        _check(rc, "ebs_quantize_activations")
    return rc


def ebs_aggregate_weights(w, count, bits, strengths, gumbel, tau, w_hat, workspace, stream=None, check=True) -> int:
    arr, n = _int_array(bits)
    rc = load_library().ebs_aggregate_weights(_ptr(w), count, arr, n, _ptr(strengths), _ptr(gumbel), tau,
                                              _ptr(w_hat), _ptr(workspace), _stream(stream))
    if check:
        _check(rc, "ebs_aggregate_weights")
    return rc


def ebs_aggregate_activations(x, count, alpha, bits, strengths, gumbel, tau, x_hat, workspace, stream=None,
                              check=True) -> int:
    arr, n = _int_array(bits)
    rc = load_library().ebs_aggregate_activations(_ptr(x), count, alpha, arr, n, _ptr(strengths), _ptr(gumbel), tau,
                                                  _ptr(x_hat), _ptr(workspace), _stream(stream))
    if check:
        _check(rc, "ebs_aggregate_activations")
    return rc


def ebs_mixed_conv2d_requant(packed_act, packed_wgt, N, C, H, W, K, R, S, stride, pad, k_w, k_a,
                             scale, offset, per_channel, alpha_next, k_next, packed_next, stream=None, check=True,
                             signed_weights=False) -> int:
    rc = load_library().ebs_mixed_conv2d_requant(
        _ptr(packed_act), _ptr(packed_wgt), N, C, H, W, K, R, S, stride, pad, k_w, k_a, int(bool(signed_weights)),
        _ptr(scale), _ptr(offset), int(bool(per_channel)), ctypes.c_float(alpha_next), k_next, _ptr(packed_next),
        _stream(stream))
    if check:
        _check(rc, "ebs_mixed_conv2d_requant")
    return rc


def ebs_conv_variant_count() -> int:
    return load_library().ebs_conv_variant_count()


def ebs_conv_variant_name(variant: int) -> str:
    return load_library().ebs_conv_variant_name(variant).decode()


def ebs_mixed_conv2d_variant(variant, packed_act, packed_wgt, N, C, H, W, K, R, S, stride, pad, k_w, k_a,
                             scale, offset, per_channel, acc_out, out_f32, stream=None, check=True) -> int:
    rc = load_library().ebs_mixed_conv2d_variant(
        variant, _ptr(packed_act), _ptr(packed_wgt), N, C, H, W, K, R, S, stride, pad, k_w, k_a,
        _ptr(scale), _ptr(offset), int(bool(per_channel)), _ptr(acc_out), _ptr(out_f32), _stream(stream))
    if check:
        _check(rc, "ebs_mixed_conv2d_variant")
    return rc


def ebs_mixed_conv2d_mfma_i8(act_levels_nhwc, wgt_levels_krsc, N, C, H, W, K, R, S, stride, pad,
                             scale, offset, per_channel, acc_out, out_f32, stream=None, check=True) -> int:
    rc = load_library().ebs_mixed_conv2d_mfma_i8(
        _ptr(act_levels_nhwc), _ptr(wgt_levels_krsc), N, C, H, W, K, R, S, stride, pad,
        _ptr(scale), _ptr(offset), int(bool(per_channel)), _ptr(acc_out), _ptr(out_f32), _stream(stream))
    if check:
        _check(rc, "ebs_mixed_conv2d_mfma_i8")
    return rc


def ebs_check_levels(levels, count, bits, device_flag, stream=None, check=True) -> int:
    rc = load_library().ebs_check_levels(_ptr(levels), count, bits, _ptr(device_flag), _stream(stream))
    if check:
        _check(rc, "ebs_check_levels")
    return rc


def ebs_probe_and_bcnt(seed, sink, blocks, trips, stream=None, check=True) -> int:
    rc = load_library().ebs_probe_and_bcnt(_ptr(seed), _ptr(sink), blocks, trips, _stream(stream))
    if check:
        _check(rc, "ebs_probe_and_bcnt")
    return rc


def ebs_probe_and_bcnt_pairs(blocks, trips) -> int:
    return load_library().ebs_probe_and_bcnt_pairs(blocks, trips)


def ebs_probe_copy(src, dst, nbytes, blocks, stream=None, check=True) -> int:
    rc = load_library().ebs_probe_copy(_ptr(src), _ptr(dst), nbytes, blocks, _stream(stream))
    if check:
        _check(rc, "ebs_probe_copy")
    return rc
