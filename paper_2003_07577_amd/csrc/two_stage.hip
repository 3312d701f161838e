// The literal two-stage form of binary decomposition (Sec. 4.3), kept as a measured
// comparison with the fused kernel: stage 1 writes the partial products P of the binary
// convolution (Eq. 13, P = B_w B_x) to memory, stage 2 is the depthwise convolution with
// the power-of-two kernel delta_w^T delta_x of shape and stride (M, K) (Eq. 14).
//
// P is stored plane by plane: plane (m, k) is an int32 tensor [N][OH][OW][c_o], planes in
// the order m*k_a + k.  Entry p_(i*M+m, j*K+k) of the paper's (c_o M) x (n K) matrix is
// element (j, i) of plane (m, k): a window of the depthwise kernel is one element of every
// plane, so stage 2 reads k_w*k_a coalesced streams.
//
// This file holds the any-shape stage 1 (one thread per output) and stage 2; the tiled
// stage 1 is the MODE_PL instantiation of the tiled convolution kernel.
#include "ebs_internal.h"
#include "fastdiv.h"

namespace ebs {

struct PlaneGeom {
    int H, W, K, R, S, stride, pad, OH, OW, cw;
    long long total_pos;   // N*(H+2)*(W+2): bordered positions of the packed input [word][position][plane]
};

template <int KW, int KA>
__global__ void __launch_bounds__(256)
bd_planes_naive(const uint32_t *__restrict__ act, const uint32_t *__restrict__ wgt, const PlaneGeom g,
                int32_t *__restrict__ planes, long long total)
{
    long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    int k = (int)(idx % g.K);
    long long t = idx / g.K;
    int ow = (int)(t % g.OW);
    t /= g.OW;
    int oh = (int)(t % g.OH);
    long long n = t / g.OH;

    uint32_t p[KW][KA];
#pragma unroll
    for (int i = 0; i < KW; ++i)
#pragma unroll
        for (int j = 0; j < KA; ++j) p[i][j] = 0u;
    const int RS = g.R * g.S;
    const int cw = g.cw;
    const uint32_t *wk = wgt + ((long long)(k / kWgtGroup) * RS * cw * kWgtGroup + (k % kWgtGroup)) * KW;
    const int Hp = g.H + 2 * kActBorder, Wp = g.W + 2 * kActBorder;
    for (int r = 0; r < g.R; ++r) {
        int hp = oh * g.stride + r - g.pad + kActBorder;      // row in the bordered grid
        if (hp < 0 || hp >= Hp) continue;                    // beyond the stored zero ring: contributes 0
        for (int s = 0; s < g.S; ++s) {
            int wcol = ow * g.stride + s - g.pad + kActBorder;
            if (wcol < 0 || wcol >= Wp) continue;
            const long long apos = (n * Hp + hp) * Wp + wcol;
            const uint32_t *wp = wk + (long long)(r * g.S + s) * cw * kWgtGroup * KW;
            for (int word = 0; word < cw; ++word) {
#pragma unroll
                for (int i = 0; i < KW; ++i) {
                    const uint32_t q = wp[(long long)word * kWgtGroup * KW + i];
#pragma unroll
                    for (int j = 0; j < KA; ++j) p[i][j] += __builtin_popcount(q & act[(word * g.total_pos + apos) * KA + j]);
                }
            }
        }
    }
#pragma unroll
    for (int i = 0; i < KW; ++i)
#pragma unroll
        for (int j = 0; j < KA; ++j) planes[(long long)(i * KA + j) * total + idx] = (int32_t)p[i][j];
}

typedef int32_t i32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// Stage 2: o = sum_m sum_k p_(m,k) << (m + k), then the scale/offset epilogue.  VEC: four
// consecutive outputs per thread (needs plane_elems % 4 == 0 so that every plane stays
// 16-byte aligned).
template <int KW, int KA, bool VEC>
__global__ void __launch_bounds__(256)
pow2_depthwise(const int32_t *__restrict__ planes, uint32_t plane_elems, FastDiv div_k,
               const float *__restrict__ scale, const float *__restrict__ offset, int per_channel,
               int32_t *__restrict__ acc_out, float *__restrict__ out_f32)
{
    constexpr int PER = VEC ? 4 : 1;
    const uint32_t first = ((uint32_t)blockIdx.x * 256u + threadIdx.x) * PER;
    if (first >= plane_elems) return;
    const int K = (int)div_k.d;
    int32_t o[PER];
#pragma unroll
    for (int e = 0; e < PER; ++e) o[e] = 0;
#pragma unroll
    for (int m = 0; m < KW; ++m)
#pragma unroll
        for (int k = 0; k < KA; ++k) {
            const int32_t *src = planes + (size_t)(m * KA + k) * plane_elems + first;
            if constexpr (VEC) {
                const i32x4 v = *reinterpret_cast<const i32x4 *>(src);
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] += (int32_t)((uint32_t)v[e] << (m + k));
            } else {
                o[0] += (int32_t)((uint32_t)src[0] << (m + k));
            }
        }
    float f[PER];
    int ch = (int)(first - fd_div(first, div_k) * (uint32_t)K);      // channel of the first element
#pragma unroll
    for (int e = 0; e < PER; ++e) {
        const int ci = per_channel ? ch : 0;
        f[e] = fmaf((float)o[e], scale[ci], offset ? offset[ci] : 0.0f);
        if (++ch == K) ch = 0;
    }
    if constexpr (VEC) {
        *reinterpret_cast<i32x4 *>(acc_out + first) = i32x4{o[0], o[1], o[2], o[3]};
        if (out_f32) *reinterpret_cast<f32x4 *>(out_f32 + first) = f32x4{f[0], f[1], f[2], f[3]};
    } else {
        acc_out[first] = o[0];
        if (out_f32) out_f32[first] = f[0];
    }
}

template <int KW, int KA>
static int launch_planes(const ConvArgs &a)
{
    PlaneGeom g{a.H, a.W, a.K, a.R, a.S, a.stride, a.pad, a.OH, a.OW, a.cw,
                (long long)a.N * (a.H + 2 * kActBorder) * (a.W + 2 * kActBorder)};
    long long total = (long long)a.N * a.OH * a.OW * a.K;
    unsigned blocks = (unsigned)((total + 255) / 256);
    hipLaunchKernelGGL((bd_planes_naive<KW, KA>), dim3(blocks), dim3(256), 0, a.stream, a.act, a.wgt, g, a.acc, total);
    return hip_ok(hipGetLastError());
}

template <int KW, int KA>
static int launch_depthwise(const int32_t *planes, long long elems, int K, const float *scale, const float *offset,
                            int per_channel, int32_t *acc, float *out, hipStream_t st)
{
    const FastDiv dk = make_fastdiv((uint32_t)K);
    if (elems % 4 == 0) {
        unsigned blocks = (unsigned)((elems / 4 + 255) / 256);
        hipLaunchKernelGGL((pow2_depthwise<KW, KA, true>), dim3(blocks), dim3(256), 0, st, planes, (uint32_t)elems, dk,
                           scale, offset, per_channel, acc, out);
    } else {
        unsigned blocks = (unsigned)((elems + 255) / 256);
        hipLaunchKernelGGL((pow2_depthwise<KW, KA, false>), dim3(blocks), dim3(256), 0, st, planes, (uint32_t)elems, dk,
                           scale, offset, per_channel, acc, out);
    }
    return hip_ok(hipGetLastError());
}

#define EBS_ALL_PAIRS(X) \
    X(1, 1) X(1, 2) X(1, 3) X(1, 4) X(1, 5) X(2, 1) X(2, 2) X(2, 3) X(2, 4) X(2, 5) \
    X(3, 1) X(3, 2) X(3, 3) X(3, 4) X(3, 5) X(4, 1) X(4, 2) X(4, 3) X(4, 4) X(4, 5) \
    X(5, 1) X(5, 2) X(5, 3) X(5, 4) X(5, 5)

int launch_planes_naive(const ConvArgs &a)
{
#define EBS_CASE(w, x) case (w) * 8 + (x): return launch_planes<w, x>(a);
    switch (a.kw * 8 + a.ka) { EBS_ALL_PAIRS(EBS_CASE) }
#undef EBS_CASE
    return EBS_ERR_BITWIDTH;
}

int launch_pow2_depthwise(const int32_t *planes, long long elems, int K, int kw, int ka, const float *scale,
                          const float *offset, int per_channel, int32_t *acc, float *out, hipStream_t st)
{
#define EBS_CASE(w, x) case (w) * 8 + (x): return launch_depthwise<w, x>(planes, elems, K, scale, offset, per_channel, acc, out, st);
    switch (kw * 8 + ka) { EBS_ALL_PAIRS(EBS_CASE) }
#undef EBS_CASE
    return EBS_ERR_BITWIDTH;
}

}  // namespace ebs
