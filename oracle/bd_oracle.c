/*
 * CPU oracle for the mixed-precision convolution by binary decomposition.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is the slow, plain,
 * obviously-correct statement of what the GPU library must compute.  It shares
 * no code, header, table or layout helper with the HIP library; only tests,
 * the smoke check and the CPU-baseline leg of the benchmark may call it.
 *
 * What the method computes (paper Sec. 3, Eq. 2; Sec. 4.3, Eq. 12-14): the
 * dot product of M-bit unsigned weight levels and K-bit unsigned activation
 * levels, obtained from AND+bitcount products of their bit planes recombined
 * with 2^(m+k).  Binary decomposition reproduces the integer matrix product of
 * the img2col'd operands exactly ("no extra computation", Sec. 4.3
 * complexities), so the result has a plain definition: the direct integer
 * convolution of the unpacked levels.  `oracle_conv2d_levels` is that
 * definition written out as seven nested loops.  `oracle_bitplane_conv` is the
 * right-hand side of Eq. 2 written out bit by bit (no packing, no popcount
 * instruction) and serves to pin the former on tiny inputs.
 *
 * Layouts (re-declared here on purpose, nothing is shared with the library):
 *   activations a[n][h][w][c]   uint8 levels, 0 <= level < 2^K      (NHWC)
 *   weights     q[k][r][s][c]   uint8 levels, 0 <= level < 2^M      (KRSC)
 *   accumulators acc[n][oh][ow][k] int32                            (NHWC)
 *   OH = floor((H + 2*pad - R)/stride) + 1, OW likewise; taps that fall
 *   outside the image read level 0 (an activation level of 0 is the real
 *   value 0 under Eq. 1b, so zero padding is exact).
 *
 * Floating point: the scale/offset epilogue is evaluated in double and
 * rounded to float once (the per-layer clip parameter and any affine term are
 * folded after the integer result, Sec. 4.3 complexities, first paragraph).
 */
#include <stdint.h>
#include <stddef.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>

static int out_extent(int in, int pad, int filt, int stride)
{
    int span = in + 2 * pad - filt;
    if (span < 0 || stride <= 0) return 0;
    return span / stride + 1;
}

int oracle_out_dims(int H, int W, int R, int S, int stride, int pad, int *OH, int *OW)
{
    *OH = out_extent(H, pad, R, stride);
    *OW = out_extent(W, pad, S, stride);
    return (*OH > 0 && *OW > 0) ? 0 : -1;
}

/* One output value of the direct integer convolution, in 64-bit. */
static int64_t direct_point(const uint8_t *a, const uint8_t *q,
                            int C, int H, int W, int R, int S,
                            int stride, int pad, int n, int k, int oh, int ow)
{
    int64_t sum = 0;
    for (int r = 0; r < R; ++r) {
        int h = oh * stride + r - pad;
        if (h < 0 || h >= H) continue;              /* zero padding */
        for (int s = 0; s < S; ++s) {
            int w = ow * stride + s - pad;
            if (w < 0 || w >= W) continue;          /* zero padding */
            const uint8_t *ap = a + (((size_t)n * H + h) * W + w) * C;
            const uint8_t *qp = q + (((size_t)k * R + r) * S + s) * C;
            for (int c = 0; c < C; ++c)
                sum += (int64_t)qp[c] * (int64_t)ap[c];
        }
    }
    return sum;
}

/*
 * Direct integer convolution of the unpacked levels: the definition of the
 * result (Eq. 2 summed over the img2col'd reduction index s = c_i*k*k).
 * Returns 0, or -1 on bad geometry, or -2 if some value does not fit int32.
 * The loop nest over (n, oh) may be split over OpenMP threads when compiled
 * with -fopenmp; each output is still one plain sum.
 */
int oracle_conv2d_levels(const uint8_t *a, const uint8_t *q,
                         int N, int C, int H, int W, int K, int R, int S,
                         int stride, int pad, int32_t *acc)
{
    int OH, OW;
    if (N <= 0 || C <= 0 || K <= 0 || R <= 0 || S <= 0 || pad < 0) return -1;
    if (oracle_out_dims(H, W, R, S, stride, pad, &OH, &OW)) return -1;
    int overflow = 0;
#pragma omp parallel for collapse(2) schedule(static) reduction(|:overflow)
    for (int n = 0; n < N; ++n)
        for (int oh = 0; oh < OH; ++oh)
            for (int ow = 0; ow < OW; ++ow)
                for (int k = 0; k < K; ++k) {
                    int64_t v = direct_point(a, q, C, H, W, R, S, stride, pad, n, k, oh, ow);
                    if (v > INT32_MAX || v < INT32_MIN) overflow = 1;
                    acc[(((size_t)n * OH + oh) * OW + ow) * K + k] = (int32_t)v;
                }
    return overflow ? -2 : 0;
}

/*
 * Signed-weight form.  The weight quantiser (Eq. 1a) maps an M-bit level q to the real weight
 * 2*q/(2^M - 1) - 1 = (2q - (2^M - 1)) / (2^M - 1), i.e. the integer weight 2q - (2^M - 1) in
 * {-(2^M-1), ..., +(2^M-1)} times a scale that is folded into scale[k].  This is the direct
 * convolution with those integer weights:
 *     acc_s[n,k,oh,ow] = sum_{c,r,s} (2*q[k,r,s,c] - (2^M - 1)) * a_pad[...]
 * (for M = 1 the weights are -1/+1).  Returns 0, -1 on bad geometry, -2 on int32 overflow.
 */
int oracle_conv2d_signed_levels(const uint8_t *a, const uint8_t *q,
                                int N, int C, int H, int W, int K, int R, int S,
                                int stride, int pad, int M, int32_t *acc)
{
    int OH, OW;
    if (N <= 0 || C <= 0 || K <= 0 || R <= 0 || S <= 0 || pad < 0 || M < 1 || M > 8) return -1;
    if (oracle_out_dims(H, W, R, S, stride, pad, &OH, &OW)) return -1;
    const int top = (1 << M) - 1;
    int overflow = 0;
#pragma omp parallel for collapse(2) schedule(static) reduction(|:overflow)
    for (int n = 0; n < N; ++n)
        for (int oh = 0; oh < OH; ++oh)
            for (int ow = 0; ow < OW; ++ow)
                for (int k = 0; k < K; ++k) {
                    int64_t sum = 0;
                    for (int r = 0; r < R; ++r) {
                        int h = oh * stride + r - pad;
                        if (h < 0 || h >= H) continue;          /* zero padding: activation 0 */
                        for (int s = 0; s < S; ++s) {
                            int w = ow * stride + s - pad;
                            if (w < 0 || w >= W) continue;
                            const uint8_t *ap = a + (((size_t)n * H + h) * W + w) * C;
                            const uint8_t *qp = q + (((size_t)k * R + r) * S + s) * C;
                            for (int c = 0; c < C; ++c)
                                sum += (int64_t)(2 * (int)qp[c] - top) * (int64_t)ap[c];
                        }
                    }
                    if (sum > INT32_MAX || sum < INT32_MIN) overflow = 1;
                    acc[(((size_t)n * OH + oh) * OW + ow) * K + k] = (int32_t)sum;
                }
    return overflow ? -2 : 0;
}

/* A single output value (for sampled checks at sizes too big to run whole). */
int oracle_conv2d_point(const uint8_t *a, const uint8_t *q,
                        int N, int C, int H, int W, int K, int R, int S,
                        int stride, int pad, int n, int k, int oh, int ow,
                        int64_t *value)
{
    int OH, OW;
    if (oracle_out_dims(H, W, R, S, stride, pad, &OH, &OW)) return -1;
    if (n < 0 || n >= N || k < 0 || k >= K || oh < 0 || oh >= OH || ow < 0 || ow >= OW) return -1;
    *value = direct_point(a, q, C, H, W, R, S, stride, pad, n, k, oh, ow);
    return 0;
}

/*
 * Right-hand side of Eq. 2, literally: expand every level into its binary
 * digits c_m (weights, m < M) and c_k (activations, k < K) held as 0/1 BYTES,
 * form bitcount[AND(c_m(w), c_k(x))] by adding up the byte-wise ANDs over the
 * reduction index, and recombine with 2^(m+k).  Plane m is bit m (LSB is
 * plane 0), as in w = sum_m c_m 2^m.  Tiny inputs only.
 * If p_planes is not NULL it receives the intermediate P of Eq. 13 as
 * p[n][oh][ow][k][m][kk] (int32), i.e. the bit-plane partial products before
 * the power-of-two recombination.
 */
int oracle_bitplane_conv(const uint8_t *a, const uint8_t *q,
                         int N, int C, int H, int W, int K, int R, int S,
                         int stride, int pad, int M, int Kbits,
                         int32_t *acc, int32_t *p_planes)
{
    int OH, OW;
    if (M < 1 || M > 8 || Kbits < 1 || Kbits > 8) return -1;
    if (oracle_out_dims(H, W, R, S, stride, pad, &OH, &OW)) return -1;
    size_t na = (size_t)N * H * W * C, nq = (size_t)K * R * S * C;
    uint8_t *ca = (uint8_t *)malloc(na * (size_t)Kbits);   /* ca[kk][element] in {0,1} */
    uint8_t *cq = (uint8_t *)malloc(nq * (size_t)M);       /* cq[m][element]  in {0,1} */
    if (!ca || !cq) { free(ca); free(cq); return -3; }
    for (int kk = 0; kk < Kbits; ++kk)
        for (size_t e = 0; e < na; ++e) ca[(size_t)kk * na + e] = (uint8_t)((a[e] >> kk) & 1u);
    for (int m = 0; m < M; ++m)
        for (size_t e = 0; e < nq; ++e) cq[(size_t)m * nq + e] = (uint8_t)((q[e] >> m) & 1u);

    for (int n = 0; n < N; ++n)
      for (int oh = 0; oh < OH; ++oh)
        for (int ow = 0; ow < OW; ++ow)
          for (int k = 0; k < K; ++k) {
            int64_t total = 0;
            for (int m = 0; m < M; ++m)
              for (int kk = 0; kk < Kbits; ++kk) {
                int64_t bitcount = 0;
                for (int r = 0; r < R; ++r) {
                    int h = oh * stride + r - pad;
                    if (h < 0 || h >= H) continue;
                    for (int s = 0; s < S; ++s) {
                        int w = ow * stride + s - pad;
                        if (w < 0 || w >= W) continue;
                        size_t ea = (((size_t)n * H + h) * W + w) * C;
                        size_t eq = (((size_t)k * R + r) * S + s) * C;
                        for (int c = 0; c < C; ++c)
                            bitcount += cq[(size_t)m * nq + eq + c] & ca[(size_t)kk * na + ea + c];
                    }
                }
                size_t o = (((size_t)n * OH + oh) * OW + ow) * K + k;
                if (p_planes) p_planes[(o * M + m) * Kbits + kk] = (int32_t)bitcount;
                total += bitcount * ((int64_t)1 << (m + kk));
              }
            acc[(((size_t)n * OH + oh) * OW + ow) * K + k] = (int32_t)total;
          }
    free(ca); free(cq);
    return 0;
}

/*
 * Affine epilogue: out = scale[k] * acc + offset[k], evaluated in double and
 * rounded to float once.  per_channel == 0 uses scale[0] / offset[0] for every
 * channel.  offset may be NULL (zero).  n_pix = N*OH*OW, acc is [n_pix][K].
 */
void oracle_dequant(const int32_t *acc, size_t n_pix, int K,
                    const float *scale, const float *offset, int per_channel,
                    float *out)
{
    for (size_t p = 0; p < n_pix; ++p)
        for (int k = 0; k < K; ++k) {
            int idx = per_channel ? k : 0;
            double sc = (double)scale[idx];
            double of = offset ? (double)offset[idx] : 0.0;
            out[p * K + k] = (float)(sc * (double)acc[p * K + k] + of);
        }
}

/*
 * Fused re-quantisation: the NEXT layer's activation quantiser (Eq. 1b-1c: clip to
 * [0, alpha] - which includes the ReLU -, normalise, round half up to b bits) applied to
 * this layer's affine output x = scale[k]*acc + offset[k].  Returns integer levels.
 * A rounding decides an integer here, so the precision and the order of operations are
 * fixed (single precision, the kernel's):
 *     x  = fmaf((float)acc, scale, offset)
 *     z  = min(max(x, 0), alpha)
 *     qs = (float)(2^b - 1) / alpha                       (one IEEE division)
 *     level = (int) floorf(fmaf(z, qs, 0.5f))             (round half up)
 */
void oracle_requant_levels(const int32_t *acc, size_t n_pix, int K,
                           const float *scale, const float *offset, int per_channel,
                           float alpha, int bits, uint8_t *levels)
{
    const float qs = (float)((1 << bits) - 1) / alpha;
    for (size_t p = 0; p < n_pix; ++p)
        for (int k = 0; k < K; ++k) {
            int idx = per_channel ? k : 0;
            float of = offset ? offset[idx] : 0.0f;
            float x = fmaf((float)acc[p * K + k], scale[idx], of);
            float z = fminf(fmaxf(x, 0.0f), alpha);
            levels[p * K + k] = (uint8_t)(int)floorf(fmaf(z, qs, 0.5f));
        }
}

/*
 * Activation quantiser on real inputs (Eq. 1b-1c): clip to [0, alpha], normalise, round half up
 * to b bits; returns the integer level (the quantised value is alpha*level/(2^b - 1)).  The
 * rounding decides an integer, so precision and order are fixed as above (single precision):
 *     z = min(max(x, 0), alpha);  qs = (float)(2^b - 1) / alpha;  level = floorf(fmaf(z, qs, 0.5f))
 */
void oracle_activation_levels(const float *x, size_t count, float alpha, int bits, uint8_t *levels)
{
    const float qs = (float)((1 << bits) - 1) / alpha;
    for (size_t i = 0; i < count; ++i) {
        float z = fminf(fmaxf(x[i], 0.0f), alpha);
        levels[i] = (uint8_t)(int)floorf(fmaf(z, qs, 0.5f));
    }
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}
