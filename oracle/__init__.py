"""CPU oracle for the binary-decomposition mixed-precision convolution.

TEST INFRASTRUCTURE ONLY: the product (the HIP library and its binding) never
imports this package, and this package never imports the product.  Only tests,
the smoke check and the benchmark's CPU-baseline leg call it.

Two layers:

* ``bd_oracle.c`` (plain C, gcc): the direct integer convolution of unpacked
  levels (the definition of the result; paper Sec. 3 Eq. 2 summed over the
  img2col'd reduction), the literal bit-by-bit right-hand side of Eq. 2, and
  the double-precision scale/offset epilogue.
* ``bd_matrix_form`` below (numpy): the paper's two-stage statement of binary
  decomposition in matrix notation (Sec. 4.3, Eq. 12-15), used on small cases.

* ``quantizers.py`` (numpy, float64): the weight and activation quantisers (Eq. 1a-1c) and the
  aggregated quantisation functions of the bitwidth search (Eq. 6, 7, 8).

Parity status: every function here is pinned by ``tests/test_oracle_pins.py``
(closed forms, brute force, float64 library convolution, integer matmul,
hand-computed fixture).  Nothing is "parity unpinned".
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "bd_oracle.c")
# EBS_ORACLE_SANITIZE=1 (set by tests/test_sanitizers.py for a child process that preloads the sanitizer
# run-time) builds and loads the same source with AddressSanitizer and UndefinedBehaviorSanitizer.
_SANITIZE = os.environ.get("EBS_ORACLE_SANITIZE") == "1"
_LIB = os.path.join(_HERE, "libbd_oracle_san.so" if _SANITIZE else "libbd_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (host only, OpenMP for the timed baseline)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        opt = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
               "-fno-omit-frame-pointer"] if _SANITIZE else ["-O2"]
        cmd = ["gcc", *opt, "-fopenmp", "-fPIC", "-shared", "-std=c99", "-ffp-contract=off", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        u8p = ctypes.POINTER(ctypes.c_uint8)
        i32p = ctypes.POINTER(ctypes.c_int32)
        f32p = ctypes.POINTER(ctypes.c_float)
        ci = ctypes.c_int
        lib.oracle_conv2d_levels.argtypes = [u8p, u8p] + [ci] * 9 + [i32p]
        lib.oracle_conv2d_levels.restype = ci
        lib.oracle_conv2d_signed_levels.argtypes = [u8p, u8p] + [ci] * 10 + [i32p]
        lib.oracle_conv2d_signed_levels.restype = ci
        lib.oracle_conv2d_point.argtypes = [u8p, u8p] + [ci] * 13 + [ctypes.POINTER(ctypes.c_int64)]
        lib.oracle_conv2d_point.restype = ci
        lib.oracle_bitplane_conv.argtypes = [u8p, u8p] + [ci] * 11 + [i32p, i32p]
        lib.oracle_bitplane_conv.restype = ci
        lib.oracle_dequant.argtypes = [i32p, ctypes.c_size_t, ci, f32p, f32p, ci, f32p]
        lib.oracle_dequant.restype = None
        lib.oracle_requant_levels.argtypes = [i32p, ctypes.c_size_t, ci, f32p, f32p, ci, ctypes.c_float, ci, u8p]
        lib.oracle_requant_levels.restype = None
        lib.oracle_activation_levels.argtypes = [f32p, ctypes.c_size_t, ctypes.c_float, ci, u8p]
        lib.oracle_activation_levels.restype = None
        lib.oracle_num_threads.argtypes = []
        lib.oracle_num_threads.restype = ci
        _lib = lib
    return _lib


def _u8(x):
    x = np.ascontiguousarray(x, dtype=np.uint8)
    return x, x.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8))


def out_dims(H, W, R, S, stride, pad):
    """OH, OW = floor((H + 2 pad - R)/stride) + 1 (likewise for W)."""
    if stride <= 0 or H + 2 * pad - R < 0 or W + 2 * pad - S < 0:
        raise ValueError("empty output")
    return (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1


def _shapes(a, q):
    N, H, W, C = a.shape
    K, R, S, C2 = q.shape
    if C != C2:
        raise ValueError("channel mismatch")
    return N, C, H, W, K, R, S


def conv2d_levels(a_nhwc, q_krsc, stride=1, pad=0):
    """Direct integer convolution of unpacked levels -> int32 [N][OH][OW][K]."""
    lib = _load()
    a, ap = _u8(a_nhwc)
    q, qp = _u8(q_krsc)
    N, C, H, W, K, R, S = _shapes(a, q)
    OH, OW = out_dims(H, W, R, S, stride, pad)
    acc = np.empty((N, OH, OW, K), dtype=np.int32)
    rc = lib.oracle_conv2d_levels(ap, qp, N, C, H, W, K, R, S, stride, pad,
                                  acc.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)))
    if rc != 0:
        raise RuntimeError(f"oracle_conv2d_levels failed: {rc}")
    return acc


def conv2d_signed_levels(a_nhwc, q_krsc, k_w, stride=1, pad=0):
    """Direct convolution with the signed integer weights 2q - (2^k_w - 1) of Eq. 1a -> int32 NHWC."""
    lib = _load()
    a, ap = _u8(a_nhwc)
    q, qp = _u8(q_krsc)
    N, C, H, W, K, R, S = _shapes(a, q)
    OH, OW = out_dims(H, W, R, S, stride, pad)
    acc = np.empty((N, OH, OW, K), dtype=np.int32)
    rc = lib.oracle_conv2d_signed_levels(ap, qp, N, C, H, W, K, R, S, stride, pad, k_w,
                                         acc.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)))
    if rc != 0:
        raise RuntimeError(f"oracle_conv2d_signed_levels failed: {rc}")
    return acc


def conv2d_point(a_nhwc, q_krsc, stride, pad, n, k, oh, ow):
    """One output value of the direct convolution (python int)."""
    lib = _load()
    a, ap = _u8(a_nhwc)
    q, qp = _u8(q_krsc)
    N, C, H, W, K, R, S = _shapes(a, q)
    v = ctypes.c_int64(0)
    rc = lib.oracle_conv2d_point(ap, qp, N, C, H, W, K, R, S, stride, pad, n, k, oh, ow,
                                 ctypes.byref(v))
    if rc != 0:
        raise RuntimeError(f"oracle_conv2d_point failed: {rc}")
    return int(v.value)


def bitplane_conv(a_nhwc, q_krsc, k_w, k_a, stride=1, pad=0, return_planes=False):
    """Eq. 2 right-hand side, bit by bit (tiny inputs).  Optionally also returns
    the bit-plane partial products P[n][oh][ow][k][m][kk] of Eq. 13."""
    lib = _load()
    a, ap = _u8(a_nhwc)
    q, qp = _u8(q_krsc)
    N, C, H, W, K, R, S = _shapes(a, q)
    OH, OW = out_dims(H, W, R, S, stride, pad)
    acc = np.empty((N, OH, OW, K), dtype=np.int32)
    planes = np.empty((N, OH, OW, K, k_w, k_a), dtype=np.int32) if return_planes else None
    pp = planes.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)) if return_planes else None
    rc = lib.oracle_bitplane_conv(ap, qp, N, C, H, W, K, R, S, stride, pad, k_w, k_a,
                                  acc.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), pp)
    if rc != 0:
        raise RuntimeError(f"oracle_bitplane_conv failed: {rc}")
    return (acc, planes) if return_planes else acc


def dequant(acc, scale, offset=None, per_channel=False):
    """out = (float)((double)scale[k]*acc + (double)offset[k]); acc is [...][K]."""
    lib = _load()
    acc = np.ascontiguousarray(acc, dtype=np.int32)
    K = acc.shape[-1]
    n_pix = acc.size // K
    scale = np.ascontiguousarray(np.atleast_1d(scale), dtype=np.float32)
    f32p = ctypes.POINTER(ctypes.c_float)
    if offset is not None:
        offset = np.ascontiguousarray(np.atleast_1d(offset), dtype=np.float32)
        op = offset.ctypes.data_as(f32p)
    else:
        op = None
    need = K if per_channel else 1
    if scale.size < need or (offset is not None and offset.size < need):
        raise ValueError("scale/offset too short")
    out = np.empty(acc.shape, dtype=np.float32)
    lib.oracle_dequant(acc.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), n_pix, K,
                       scale.ctypes.data_as(f32p), op, 1 if per_channel else 0,
                       out.ctypes.data_as(f32p))
    return out


def requant_levels(acc, scale, offset, per_channel, alpha, bits):
    """Next layer's activation levels (Eq. 1b-1c, round half up) of x = scale*acc + offset,
    in the fixed single-precision order documented in bd_oracle.c.  acc is [...][K]."""
    lib = _load()
    acc = np.ascontiguousarray(acc, dtype=np.int32)
    K = acc.shape[-1]
    scale = np.ascontiguousarray(np.atleast_1d(scale), dtype=np.float32)
    f32p = ctypes.POINTER(ctypes.c_float)
    op = None
    if offset is not None:
        offset = np.ascontiguousarray(np.atleast_1d(offset), dtype=np.float32)
        op = offset.ctypes.data_as(f32p)
    need = K if per_channel else 1
    if scale.size < need or (offset is not None and offset.size < need):
        raise ValueError("scale/offset too short")
    out = np.empty(acc.shape, dtype=np.uint8)
    lib.oracle_requant_levels(acc.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), acc.size // K, K,
                              scale.ctypes.data_as(f32p), op, 1 if per_channel else 0,
                              ctypes.c_float(alpha), bits, out.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)))
    return out


def num_threads() -> int:
    return int(_load().oracle_num_threads())


# --------------------------------------------------------------------------
# The paper's matrix statement of binary decomposition (Sec. 4.3), in numpy.
# --------------------------------------------------------------------------

def img2col(a_nhwc, R, S, stride, pad):
    """X_hat in S^{s x n}: column j = output position (n, oh, ow) flattened,
    row = reduction index (r, s, c) flattened, s = c_i * k * k (Sec. 4.3)."""
    a = np.asarray(a_nhwc, dtype=np.int64)
    N, H, W, C = a.shape
    OH, OW = out_dims(H, W, R, S, stride, pad)
    ap = np.zeros((N, H + 2 * pad, W + 2 * pad, C), dtype=np.int64)
    ap[:, pad:pad + H, pad:pad + W, :] = a
    X = np.empty((R * S * C, N * OH * OW), dtype=np.int64)
    col = 0
    for n in range(N):
        for oh in range(OH):
            for ow in range(OW):
                patch = ap[n, oh * stride:oh * stride + R, ow * stride:ow * stride + S, :]
                X[:, col] = patch.reshape(-1)
                col += 1
    return X


def bd_matrix_form(a_nhwc, q_krsc, k_w, k_a, stride=1, pad=0, explicit_lambda=False):
    """Binary decomposition as the paper states it (Eq. 12-15):

    W_hat (c_o x s) = Lambda_w B_w with B_w in {0,1}^{c_o M x s}, row i*M+m =
    digit m of output channel i;  X_hat (s x n) = B_x Lambda_x^T with B_x in
    {0,1}^{s x n K}, column j*K+k = digit k of position j.  Stage 1:
    P = B_w B_x (AND + bitcount only).  Stage 2: O = Lambda_w P Lambda_x^T,
    i.e. o_ij = sum_m sum_k 2^(m+k) p_(iM+m, jK+k) (0-based), a depthwise
    convolution of P with kernel delta_w^T delta_x, size and stride (M, K).

    Returns (O reshaped to [N][OH][OW][c_o], P).
    """
    a = np.asarray(a_nhwc)
    q = np.asarray(q_krsc)
    N, H, W, C = a.shape
    K_out, R, S, _ = q.shape
    OH, OW = out_dims(H, W, R, S, stride, pad)
    M, Kb = k_w, k_a
    W_hat = q.reshape(K_out, R * S * C).astype(np.int64)          # c_o x s
    X_hat = img2col(a, R, S, stride, pad)                         # s x n
    s, n = X_hat.shape
    B_w = np.empty((K_out * M, s), dtype=np.int64)
    for i in range(K_out):
        for m in range(M):
            B_w[i * M + m, :] = (W_hat[i, :] >> m) & 1
    B_x = np.empty((s, n * Kb), dtype=np.int64)
    for j in range(n):
        for k in range(Kb):
            B_x[:, j * Kb + k] = (X_hat[:, j] >> k) & 1
    P = B_w @ B_x                                                 # stage 1, c_o M x n K
    if explicit_lambda:
        delta_w = 2 ** np.arange(M, dtype=np.int64)
        delta_x = 2 ** np.arange(Kb, dtype=np.int64)
        Lw = np.kron(np.eye(K_out, dtype=np.int64), delta_w[None, :])   # c_o x c_o M
        Lx = np.kron(np.eye(n, dtype=np.int64), delta_x[None, :])       # n x n K
        O = Lw @ P @ Lx.T
    else:
        O = np.zeros((K_out, n), dtype=np.int64)
        for m in range(M):
            for k in range(Kb):
                O += (P[m::M, k::Kb] << (m + k))                  # stage 2 shift-adds
    return O.T.reshape(N, OH, OW, K_out), P


# --------------------------------------------------------------------------
# The two stages of Sec. 4.3 as separate operations (what a literal
# implementation materialises between its two convolutions).
# --------------------------------------------------------------------------

def partial_products(a_nhwc, q_krsc, k_w, k_a, stride=1, pad=0):
    """Stage 1 of Sec. 4.3: the ordinary convolution with binary weights and binary
    activations.  Digit m of the weights convolved with digit k of the activations,
    each as a 0/1 tensor through the direct integer convolution.

    Returns planes[m][k][N][OH][OW][c_o] (int32); planes[m][k][j][i] is the entry
    p_(i*M+m, j*K+k) of the paper's P (0-based, j = flattened output position).
    """
    a = np.asarray(a_nhwc).astype(np.uint8)
    q = np.asarray(q_krsc).astype(np.uint8)
    out = None
    for m in range(k_w):
        qm = ((q >> m) & 1).astype(np.uint8)
        for k in range(k_a):
            ak = ((a >> k) & 1).astype(np.uint8)
            pm = conv2d_levels(ak, qm, stride, pad)
            if out is None:
                out = np.empty((k_w, k_a) + pm.shape, dtype=np.int32)
            out[m, k] = pm
    return out


def planes_to_matrix(planes):
    """Layout change only: planes[m][k][...positions...][c_o] -> P of shape (c_o*M, n*K)
    with row i*M+m and column j*K+k (Sec. 4.3)."""
    planes = np.asarray(planes)
    M, Kb = planes.shape[:2]
    c_o = planes.shape[-1]
    flat = planes.reshape(M, Kb, -1, c_o)                 # [m][k][j][i]
    n = flat.shape[2]
    return np.ascontiguousarray(flat.transpose(3, 0, 2, 1)).reshape(c_o * M, n * Kb)


def depthwise_pow2(P, M, Kb):
    """Stage 2 of Sec. 4.3 (Eq. 14): one depthwise kernel delta_w^T delta_x of
    shape (M, K), entries 2^(m+k), slid over P with stride (M, K).
    P is (c_o*M, n*K); returns O (c_o, n) as int64."""
    P = np.asarray(P, dtype=np.int64)
    rows, cols = P.shape
    if rows % M or cols % Kb:
        raise ValueError("P does not tile into (M, K) windows")
    kernel = np.empty((M, Kb), dtype=np.int64)
    for m in range(M):
        for k in range(Kb):
            kernel[m, k] = 1 << (m + k)
    c_o, n = rows // M, cols // Kb
    O = np.empty((c_o, n), dtype=np.int64)
    for i in range(c_o):
        for j in range(n):
            window = P[i * M:(i + 1) * M, j * Kb:(j + 1) * Kb]
            O[i, j] = int((window * kernel).sum())
    return O


from .quantizers import (  # noqa: E402,F401
    quantize_b, weight_levels, quantize_weights, activation_levels, quantize_activations,
    quantize_activations_f64, softmax, gumbel_softmax, aggregate_weights, aggregate_activations,
)

