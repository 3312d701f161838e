// Fallback convolution: one thread per output value, no tiling.  Runs any
// valid shape; the tiled kernel is the fast path.  Per output it evaluates
// Eq. 2 over the packed words: for every reduction word and every plane pair
// (i, j) a bitwise AND and an accumulating bitcount into the accumulator of
// shift class i+j, then Eq. 14's recombination sum_s class_s << s.
#include "ebs_internal.h"
#include "requant.h"

namespace ebs {

struct NaiveGeom {
    int H, W, K, R, S, stride, pad, OH, OW, cw;
    int wtop;      // 0: unsigned weight levels; else 2^k_w - 1 (signed weights 2q - wtop)
    long long total_pos;   // N*(H+2)*(W+2): bordered positions of the packed input [word][position][plane]
};

template <int KW, int KA>
__device__ __forceinline__ int32_t naive_point(const uint32_t *__restrict__ act, const uint32_t *__restrict__ wgt,
                                               const NaiveGeom &g, long long n, int oh, int ow, int k)
{
    constexpr int NCLS = KW + KA - 1;
    uint32_t cls[NCLS];
#pragma unroll
    for (int c = 0; c < NCLS; ++c) cls[c] = 0u;
    uint32_t wsum[KA];
#pragma unroll
    for (int j = 0; j < KA; ++j) wsum[j] = 0u;
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
                uint32_t x[KA], q[KW];
#pragma unroll
                for (int j = 0; j < KA; ++j) x[j] = act[(word * g.total_pos + apos) * KA + j];
#pragma unroll
                for (int i = 0; i < KW; ++i) q[i] = wp[(long long)word * kWgtGroup * KW + i];
#pragma unroll
                for (int i = 0; i < KW; ++i)
#pragma unroll
                    for (int j = 0; j < KA; ++j) cls[i + j] += __builtin_popcount(q[i] & x[j]);
                if (g.wtop) {
#pragma unroll
                    for (int j = 0; j < KA; ++j) wsum[j] += __builtin_popcount(x[j]);
                }
            }
        }
    }
    uint32_t acc = 0;
#pragma unroll
    for (int c = 0; c < NCLS; ++c) acc += cls[c] << c;
    if (g.wtop) {
        uint32_t ws = 0;
#pragma unroll
        for (int j = 0; j < KA; ++j) ws += wsum[j] << j;
        return 2 * (int32_t)acc - g.wtop * (int32_t)ws;
    }
    return (int32_t)acc;
}

template <int KW, int KA>
__global__ void __launch_bounds__(256)
bd_conv_naive(const uint32_t *__restrict__ act, const uint32_t *__restrict__ wgt, const NaiveGeom g,
              const float *__restrict__ scale, const float *__restrict__ offset, int per_channel,
              int32_t *__restrict__ acc_out, float *__restrict__ out_f32, long long total)
{
    long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    int k = (int)(idx % g.K);
    long long t = idx / g.K;
    int ow = (int)(t % g.OW);
    t /= g.OW;
    int oh = (int)(t % g.OH);
    long long n = t / g.OH;
    const int32_t acc = naive_point<KW, KA>(act, wgt, g, n, oh, ow, k);
    acc_out[idx] = acc;
    if (out_f32) {
        int ci = per_channel ? k : 0;
        float of = offset ? offset[ci] : 0.0f;
        out_f32[idx] = fmaf((float)acc, scale[ci], of);
    }
}

// Fused re-quantisation, fallback form: one thread per (output position, 32-channel word of the
// next layer's packed activations).
template <int KW, int KA>
__global__ void __launch_bounds__(256)
bd_requant_naive(const uint32_t *__restrict__ act, const uint32_t *__restrict__ wgt, const NaiveGeom g,
                 const float *__restrict__ scale, const float *__restrict__ offset, int per_channel,
                 uint32_t *__restrict__ next, float alpha, float qs, int k_next, long long total /* positions*cwn */)
{
    long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const int cwn = (g.K + 31) / 32;
    int word = (int)(idx % cwn);
    long long t = idx / cwn;
    int ow = (int)(t % g.OW);
    long long tt = t / g.OW;
    int oh = (int)(tt % g.OH);
    long long n = tt / g.OH;
    uint32_t planes[kMaxBits] = {};
    for (int c = 0; c < 32; ++c) {
        const int k = word * 32 + c;
        if (k >= g.K) break;
        const int32_t acc = naive_point<KW, KA>(act, wgt, g, n, oh, ow, k);
        const int ci = per_channel ? k : 0;
        const uint32_t lv = requant_level(acc, scale[ci], offset ? offset[ci] : 0.0f, alpha, qs);
#pragma unroll
        for (int j = 0; j < kMaxBits; ++j) planes[j] |= ((lv >> j) & 1u) << c;
    }
    const long long pos = (n * (g.OH + 2 * kActBorder) + oh + kActBorder) * (g.OW + 2 * kActBorder) + ow + kActBorder;
    const long long total_next = (total / cwn) / ((long long)g.OH * g.OW) * (g.OH + 2 * kActBorder) * (g.OW + 2 * kActBorder);
    for (int j = 0; j < k_next; ++j) next[(word * total_next + pos) * k_next + j] = planes[j];
}

template <int KW, int KA>
static int launch(const ConvArgs &a)
{
    NaiveGeom g{a.H, a.W, a.K, a.R, a.S, a.stride, a.pad, a.OH, a.OW, a.cw, a.wtop,
                (long long)a.N * (a.H + 2 * kActBorder) * (a.W + 2 * kActBorder)};
    if (a.next) {
        long long total = (long long)a.N * a.OH * a.OW * ((a.K + 31) / 32);
        unsigned blocks = (unsigned)((total + 255) / 256);
        hipLaunchKernelGGL((bd_requant_naive<KW, KA>), dim3(blocks), dim3(256), 0, a.stream, a.act, a.wgt, g,
                           a.scale, a.offset, a.per_channel, a.next, a.alpha, requant_qs(a.alpha, a.k_next), a.k_next, total);
        return hip_ok(hipGetLastError());
    }
    long long total = (long long)a.N * a.OH * a.OW * a.K;
    unsigned blocks = (unsigned)((total + 255) / 256);
    hipLaunchKernelGGL((bd_conv_naive<KW, KA>), dim3(blocks), dim3(256), 0, a.stream,
                       a.act, a.wgt, g, a.scale, a.offset, a.per_channel, a.acc, a.out, total);
    return hip_ok(hipGetLastError());
}

static int dispatch(const ConvArgs &a)
{
#define EBS_CASE(w, x) case (w) * 8 + (x): return launch<w, x>(a);
    switch (a.kw * 8 + a.ka) {
        EBS_CASE(1, 1) EBS_CASE(1, 2) EBS_CASE(1, 3) EBS_CASE(1, 4) EBS_CASE(1, 5)
        EBS_CASE(2, 1) EBS_CASE(2, 2) EBS_CASE(2, 3) EBS_CASE(2, 4) EBS_CASE(2, 5)
        EBS_CASE(3, 1) EBS_CASE(3, 2) EBS_CASE(3, 3) EBS_CASE(3, 4) EBS_CASE(3, 5)
        EBS_CASE(4, 1) EBS_CASE(4, 2) EBS_CASE(4, 3) EBS_CASE(4, 4) EBS_CASE(4, 5)
        EBS_CASE(5, 1) EBS_CASE(5, 2) EBS_CASE(5, 3) EBS_CASE(5, 4) EBS_CASE(5, 5)
    }
#undef EBS_CASE
    return EBS_ERR_BITWIDTH;
}

int launch_conv_naive(const ConvArgs &a) { return dispatch(a); }
int launch_requant_naive(const ConvArgs &a) { return dispatch(a); }

// Zero ring of a packed activation tensor [word][N][H+2][W+2][plane]: one thread per ring dword.
__global__ void __launch_bounds__(256)
zero_border_kernel(uint32_t *__restrict__ packed, int H, int W, int planes, int wpp, long long per_image, long long total,
                   long long total_pos)
{
    long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const int Hp = H + 2 * kActBorder, Wp = W + 2 * kActBorder;
    long long n = idx / per_image;
    long long rem = idx - n * per_image;
    int dword = (int)(rem % wpp);             // (word, plane) of the position
    int b = (int)(rem / wpp);                 // ring position: top row, bottom row, then left/right columns
    int hp, wp;
    if (b < Wp) { hp = 0; wp = b; }
    else if (b < 2 * Wp) { hp = Hp - 1; wp = b - Wp; }
    else { int c = b - 2 * Wp; hp = 1 + c / 2; wp = (c & 1) ? Wp - 1 : 0; }
    const int word = dword / planes, j = dword - word * planes;
    packed[(word * total_pos + (n * Hp + hp) * Wp + wp) * planes + j] = 0u;
}

int launch_zero_border(uint32_t *packed, int N, int H, int W, int words, int planes, hipStream_t st)
{
    const int Wp = W + 2 * kActBorder;
    const int wpp = words * planes;
    long long ring = 2LL * Wp + 2LL * H;
    long long per_image = ring * wpp;
    long long total = per_image * N;
    unsigned blocks = (unsigned)((total + 255) / 256);
    hipLaunchKernelGGL(zero_border_kernel, dim3(blocks), dim3(256), 0, st, packed, H, W, planes, wpp, per_image, total,
                       (long long)N * (H + 2 * kActBorder) * Wp);
    return hip_ok(hipGetLastError());
}

}  // namespace ebs
