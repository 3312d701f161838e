/*
 * libebs - mixed-precision convolution by binary decomposition on MI355X (gfx950).
 *
 * The operation (paper Sec. 3, Eq. 2; Sec. 4.3, Eq. 12-15): a convolution of
 * k_w-bit unsigned weight levels with k_a-bit unsigned activation levels is
 * computed from the bit planes of both operands: every (weight plane i,
 * activation plane j) pair is multiplied with bitwise AND + bitcount, and the
 * partial products are recombined with the power-of-two factors 2^(i+j).  The
 * layer's affine terms (clip parameter, level spacing, batch-norm folding;
 * Sec. 4.3 "Complexities", first paragraph) are applied after the integer
 * result as out = scale * acc + offset.
 *
 * Conventions common to every call
 *  - All data pointers are DEVICE pointers (HBM) owned by the caller; the
 *    library allocates nothing, frees nothing and keeps no state between
 *    calls.  Buffers must be 16-byte aligned.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Every call only enqueues kernels on that stream and returns; results are
 *    valid once the stream has been synchronised by the caller.
 *  - Return value: EBS_OK (0) or a negative ebs_status.  Argument errors are
 *    detected on the host before anything is enqueued.  Nothing throws or
 *    aborts across this boundary.
 *  - Levels: uint8, one level per byte.  Activations are NHWC
 *    a[n][h][w][c]; weights are KRSC q[k][r][s][c].  Only the low k bits of a
 *    level are used (level & (2^k - 1)); plane m is bit m, plane 0 the LSB.
 *  - Outputs are NHWC: acc[n][oh][ow][k] with
 *    OH = floor((H + 2*pad - R)/stride) + 1 and OW likewise; taps outside the
 *    image contribute zero (activation level 0 is the real value 0).
 *  - Bitwidths: 1 <= k_w, k_a <= 5 (the paper's search space, Sec. 5).
 *  - Packed buffers are opaque: their size comes from the *_bytes() calls and
 *    their content is only meaningful to ebs_mixed_conv2d of the same library
 *    version.
 */
#ifndef EBS_H
#define EBS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    EBS_OK = 0,
    EBS_ERR_NULL = -1,        /* a required pointer is NULL                         */
    EBS_ERR_BITWIDTH = -2,    /* k_w or k_a outside [1, 5]                          */
    EBS_ERR_SHAPE = -3,       /* non-positive extent, empty output, pad >= filter,
                                 a tensor with 2^31 or more elements, more than
                                 2^31 - 1025 output positions, or a reduction
                                 whose largest sum C*R*S*(2^k_w-1)*(2^k_a-1) does
                                 not fit an int32                                   */
    EBS_ERR_ALIGN = -4,       /* a buffer is not 16-byte aligned                    */
    EBS_ERR_UNSUPPORTED = -5, /* valid request this build has no kernel for         */
    EBS_ERR_HIP = -6,         /* the HIP runtime refused a launch                   */
    EBS_ERR_LEVEL_RANGE = -7  /* ebs_check_levels found a level >= 2^bits           */
} ebs_status;

/* Library version (major*10000 + minor*100 + patch). */
int ebs_version(void);

/* Static, human-readable name of a status code. */
const char *ebs_status_string(int status);

/* Name of the HIP runtime error behind the calling thread's most recent
 * EBS_ERR_HIP ("hipSuccess" if there was none).  Static string. */
const char *ebs_last_hip_error(void);

/*
 * Size in bytes of the packed bit-plane form of a weight tensor (the binary
 * matrix B_w of Eq. 12/15: k_w planes, channel bits packed into 32-bit words)
 * and of an activation tensor (B_x, k_a planes).  Return 0 on invalid
 * arguments.
 */
size_t ebs_packed_weights_bytes(int K, int C, int R, int S, int k_w);
size_t ebs_packed_activations_bytes(int N, int H, int W, int C, int k_a);

/*
 * Weight decomposition W = Lambda_w B_w (Eq. 12, 15): split the KRSC levels
 * into k_w bit planes and pack input-channel bits into 32-bit words.  Done
 * once per layer (offline in the paper's deployment flow).
 *   levels_krsc : in,  device, K*R*S*C bytes
 *   packed      : out, device, ebs_packed_weights_bytes(...) bytes
 * The packed form is opaque: it is what the convolution calls expect for the
 * same (K, C, R, S, k_w) and nothing else may write it (for 3x3 filters on at
 * most 16 input channels it holds a second arrangement of the same planes, two
 * filter taps per 32-bit word, which the size above includes).
 */
int ebs_pack_weights(const uint8_t *levels_krsc, int K, int C, int R, int S, int k_w,
                     void *packed, void *stream);

/*
 * Activation decomposition X = B_x Lambda_x^T (Eq. 12, 15): split the NHWC
 * levels into k_a bit planes, channel bits packed into 32-bit words.  Runs
 * once per layer invocation.
 *   levels_nhwc : in,  device, N*H*W*C bytes
 *   packed      : out, device, ebs_packed_activations_bytes(...) bytes
 */
int ebs_pack_activations(const uint8_t *levels_nhwc, int N, int H, int W, int C, int k_a,
                         void *packed, void *stream);

/*
 * The mixed-precision convolution (Eq. 2 applied to every output; stage 1
 * P = B_w B_x by AND + bitcount, Eq. 13; stage 2 o = sum_i sum_j 2^(i+j) p_ij,
 * Eq. 14, fused into the same kernel) followed by the affine epilogue.
 *   packed_act : in, device, from ebs_pack_activations(N,H,W,C,k_a)
 *   packed_wgt : in, device, from ebs_pack_weights(K,C,R,S,k_w)
 *   scale      : in, device, 1 float (per_channel == 0) or K floats
 *   offset     : in, device, same count as scale, or NULL for zero
 *   acc_out    : out, device, int32 [N][OH][OW][K], exact integer result
 *   out_f32    : out, device, float [N][OH][OW][K] = scale*acc + offset
 *                (one fused multiply-add in fp32); may be NULL to skip it
 * Groups = 1, dilation = 1, square stride, symmetric zero padding, pad < R,S.
 */
int ebs_mixed_conv2d(const void *packed_act, const void *packed_wgt,
                     int N, int C, int H, int W, int K, int R, int S,
                     int stride, int pad, int k_w, int k_a,
                     const float *scale, const float *offset, int per_channel,
                     int32_t *acc_out, float *out_f32, void *stream);

/*
 * The same convolution with the NEXT layer's activation quantiser fused into the epilogue
 * (Eq. 1b-1c: clip to [0, alpha_next] - the clip at 0 is the ReLU -, normalise, round half
 * up to k_next bits) and the result written directly as the next layer's packed activations:
 *     x = scale[k]*acc + offset[k];  level = floor((2^k_next - 1)/alpha_next * clip(x, 0, alpha_next) + 0.5)
 * evaluated in single precision in exactly this order: fmaf(acc, scale, offset), min/max,
 * fmaf(z, qs, 0.5) with qs = (float)(2^k_next - 1)/alpha_next, floor.  No int32/fp32 tensor is
 * written (k_next/8 bytes per output instead of 8) and no separate pack call is needed.
 *   packed_next : out, device, ebs_packed_activations_bytes(N, OH, OW, K, k_next) bytes; ready to
 *                 be the packed_act of a layer with C = K, H = OH, W = OW (its zero ring is written
 *                 by this call)
 * signed_weights != 0 selects the signed-weight product of ebs_mixed_conv2d_signed for acc.
 * Other arguments as for ebs_mixed_conv2d; alpha_next must be positive and finite.
 */
int ebs_mixed_conv2d_requant(const void *packed_act, const void *packed_wgt,
                             int N, int C, int H, int W, int K, int R, int S,
                             int stride, int pad, int k_w, int k_a, int signed_weights,
                             const float *scale, const float *offset, int per_channel,
                             float alpha_next, int k_next, void *packed_next, void *stream);

/*
 * Signed-weight form of ebs_mixed_conv2d.  The weight quantiser (Eq. 1a) maps a level q to the
 * real weight 2q/(2^k_w - 1) - 1, i.e. to the integer weight 2q - (2^k_w - 1) times a factor the
 * caller folds into scale[k].  Binary decomposition (Eq. 2, Sec. 4.3) runs on the unsigned levels;
 * this call adds the data-dependent correction so that
 *     acc_out = sum (2q - (2^k_w - 1)) * a = 2 * sum q*a - (2^k_w - 1) * sum a
 * (sum a = window sum of the activation levels, obtained in the same pass from bitcounts of the
 * activation planes alone), and out_f32 = scale[k]*acc_out + offset[k].  For k_w = 1 the weights
 * are -1 / +1.  Same packed operands, arguments and conventions as ebs_mixed_conv2d;
 * ebs_mixed_conv2d_requant takes the same choice through its signed_weights flag.
 */
int ebs_mixed_conv2d_signed(const void *packed_act, const void *packed_wgt,
                            int N, int C, int H, int W, int K, int R, int S,
                            int stride, int pad, int k_w, int k_a,
                            const float *scale, const float *offset, int per_channel,
                            int32_t *acc_out, float *out_f32, void *stream);

/*
 * The literal two-stage form of Sec. 4.3, as a measured comparison with the fused call: the
 * intermediate P that ebs_mixed_conv2d keeps in registers goes through device memory here.
 *
 * Stage 1, ebs_binary_conv_planes: the ordinary convolution with binary weights and binary
 * activations (Eq. 13, P = B_w B_x; AND + bitcount only, no shifts).
 *   planes : out, device, int32, ebs_partial_products_bytes(...) bytes, 16-byte aligned.
 *            k_w*k_a tensors [N][OH][OW][K] in the order m*k_a + k (m: weight digit, k:
 *            activation digit).  Entry p_(i*M+m, j*K+k) of the paper's (c_o M) x (n K) matrix,
 *            i = output channel and j = flattened output position (n, oh, ow), is element
 *            [j][i] of plane (m, k).
 * Stage 2, ebs_pow2_depthwise: the depthwise convolution of P with the single kernel
 * delta_w^T delta_x of shape (M, K), entries 2^(m+k), stride (M, K) (Eq. 14), then the affine
 * epilogue of ebs_mixed_conv2d:
 *   acc_out[j][i] = sum_m sum_k planes[m*k_a + k][j][i] << (m + k);  out_f32 = scale*acc + offset.
 *   positions = N*OH*OW; scale/offset/per_channel/acc_out/out_f32 as for ebs_mixed_conv2d.
 * ebs_partial_products_bytes returns 0 on invalid arguments.  Other arguments and error codes as
 * for ebs_mixed_conv2d; nothing is allocated by either call.
 */
size_t ebs_partial_products_bytes(int N, int H, int W, int K, int R, int S,
                                  int stride, int pad, int k_w, int k_a);
int ebs_binary_conv_planes(const void *packed_act, const void *packed_wgt,
                           int N, int C, int H, int W, int K, int R, int S,
                           int stride, int pad, int k_w, int k_a,
                           int32_t *planes, void *stream);
int ebs_pow2_depthwise(const int32_t *planes, long long positions, int K, int k_w, int k_a,
                       const float *scale, const float *offset, int per_channel,
                       int32_t *acc_out, float *out_f32, void *stream);

/*
 * Same call with the kernel variant chosen by the caller instead of the
 * library's shape heuristic; exists so that measurements can sweep tilings.
 * variant 0 = heuristic; ebs_conv_variant_count() gives the number of
 * variants (valid values 0..count); a variant that cannot run the given shape
 * returns EBS_ERR_UNSUPPORTED.  Results are identical for every variant.
 */
int ebs_conv_variant_count(void);
const char *ebs_conv_variant_name(int variant);
int ebs_mixed_conv2d_variant(int variant,
                             const void *packed_act, const void *packed_wgt,
                             int N, int C, int H, int W, int K, int R, int S,
                             int stride, int pad, int k_w, int k_a,
                             const float *scale, const float *offset, int per_channel,
                             int32_t *acc_out, float *out_f32, void *stream);

/*
 * Measured comparison only (not the binary-decomposition path): the same
 * integer convolution taken directly on the unpacked levels with int8 matrix
 * instructions.  Same outputs and conventions as ebs_mixed_conv2d; needs
 * C to be a multiple of 32 (EBS_ERR_UNSUPPORTED otherwise); levels must be
 * below 128.
 */
int ebs_mixed_conv2d_mfma_i8(const uint8_t *act_levels_nhwc, const uint8_t *wgt_levels_krsc,
                             int N, int C, int H, int W, int K, int R, int S,
                             int stride, int pad,
                             const float *scale, const float *offset, int per_channel,
                             int32_t *acc_out, float *out_f32, void *stream);

/*
 * Quantisers (Preliminaries, Eq. 1a-1c; round() is round half up) and the aggregated quantisation
 * functions of the bitwidth search (Sec. 4.1).  Element-wise; all pointers are device memory and
 * 16-byte aligned unless said otherwise; count > 0 elements; nothing is allocated.
 *
 * workspace: EBS_QUANT_WORKSPACE_BYTES bytes of device memory owned by the caller, overwritten by
 * the call (holds the max reduction and the candidates' coefficients); calls that share one
 * workspace must be ordered on one stream.
 *
 * ebs_quantize_weights (Eq. 1a): levels[i] = round((2^k_w - 1) (tanh w_i / (2 max_j |tanh w_j|) + 1/2)),
 *   an integer in [0, 2^k_w - 1]; the quantised weight is 2 level/(2^k_w - 1) - 1, i.e. the signed-
 *   weight form of ebs_mixed_conv2d_signed.  Evaluated in double precision (a rounding decides an
 *   integer).  An all-zero tensor gives level 2^(k_w - 1) everywhere; NaN inputs are not supported.
 * ebs_quantize_activations (Eq. 1b-1c): levels[i] = round((2^k_a - 1) clip(x_i, 0, alpha) / alpha), the
 *   quantised activation is alpha level/(2^k_a - 1).  Single precision in the order of
 *   ebs_mixed_conv2d_requant: z = min(max(x, 0), alpha); level = floor(fmaf(z, (float)(2^k_a - 1)/alpha, 0.5)).
 * ebs_aggregate_weights (Eq. 6; Eq. 8 when gumbel != NULL): w_hat[i] = sum_c coef_c * W_hat^{bits[c]}[i]
 *   with coef = softmax(strengths), or softmax((log softmax(strengths) + gumbel) / tau): ONE meta
 *   weight tensor in, one aggregated tensor out, whatever the number of candidates.
 * ebs_aggregate_activations (Eq. 7, activation factor): x_hat[i] = sum_c coef_c * X_hat^{bits[c]}[i].
 *   bits      : in, HOST, n_bits candidate bitwidths, each in [1, 8]; 1 <= n_bits <= EBS_MAX_CANDIDATES
 *   strengths : in, device, n_bits floats (the learnable strengths r or s)
 *   gumbel    : in, device, n_bits Gumbel(0,1) samples drawn by the caller, or NULL (deterministic search)
 *   tau       : temperature of Eq. 8 (> 0; ignored when gumbel is NULL)
 * k_w and k_a may be 1..8 here (a level is one byte); the convolution calls take up to 5.
 * Errors: EBS_ERR_NULL, EBS_ERR_BITWIDTH (a bitwidth outside its range, n_bits outside its range),
 * EBS_ERR_SHAPE (count == 0 or >= 2^40, alpha or tau not positive and finite), EBS_ERR_ALIGN.
 */
#define EBS_MAX_CANDIDATES 8
#define EBS_QUANT_WORKSPACE_BYTES 256
int ebs_quantize_weights(const float *w, size_t count, int k_w, uint8_t *levels,
                         void *workspace, void *stream);
int ebs_quantize_activations(const float *x, size_t count, float alpha, int k_a,
                             uint8_t *levels, void *stream);
int ebs_aggregate_weights(const float *w, size_t count, const int *bits, int n_bits,
                          const float *strengths, const float *gumbel, float tau,
                          float *w_hat, void *workspace, void *stream);
int ebs_aggregate_activations(const float *x, size_t count, float alpha,
                              const int *bits, int n_bits,
                              const float *strengths, const float *gumbel, float tau,
                              float *x_hat, void *workspace, void *stream);

/*
 * ebs_quantize_weights for callers that cannot allocate device memory and therefore have no
 * workspace to pass: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same kernels and the same levels as ebs_quantize_weights; the 256-byte workspace is
 * a device array inside the library (EBS_QUANT_WORKSPACE_BYTES per GPU, held until the process
 * ends).  The call allocates and frees nothing and records no memset: the word that must start at
 * zero is cleared by a kernel of the call.
 *   - count must not exceed EBS_STATIC_MAX_COUNT (EBS_ERR_SHAPE otherwise; the workspace itself
 *     does not grow with count, the bound is what one launch of the element-wise kernel covers).
 *   - The device that owns `stream` must be the current device of the calling thread.
 *   - Every call on one GPU shares that GPU's array: calls that may overlap on one GPU (different
 *     streams, different threads) race on it and must be ordered by the caller.
 *   - More than 64 devices in one process: EBS_ERR_UNSUPPORTED.
 * Other arguments and error codes as for ebs_quantize_weights.
 */
#define EBS_STATIC_MAX_COUNT (1ull << 31)
int ebs_quantize_weights_static(const float *w, size_t count, int k_w, uint8_t *levels, void *stream);

/*
 * Debug aid: *device_flag (int32 on the device, cleared by this call) becomes
 * non-zero if any of `count` levels is >= 2^bits.  The pack calls themselves
 * never fail on range; they keep the low bits.
 */
int ebs_check_levels(const uint8_t *levels, size_t count, int bits,
                     int32_t *device_flag, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* EBS_H */
