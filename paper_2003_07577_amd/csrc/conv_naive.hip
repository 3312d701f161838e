// Fallback convolution: one thread per output value, no tiling.  Runs any
// valid shape; the tiled kernel is the fast path.  Per output it evaluates
// Eq. 2 over the packed words: for every reduction word and every plane pair
// (i, j) a bitwise AND and an accumulating bitcount into the accumulator of
// shift class i+j, then Eq. 14's recombination sum_s class_s << s.
#include "ebs_internal.h"

namespace ebs {

template <int KW, int KA>
__global__ void __launch_bounds__(256)
bd_conv_naive(const uint32_t *__restrict__ act, const uint32_t *__restrict__ wgt,
              int H, int W, int K, int R, int S, int stride, int pad, int OH, int OW, int cw,
              const float *__restrict__ scale, const float *__restrict__ offset, int per_channel,
              int32_t *__restrict__ acc_out, float *__restrict__ out_f32, long long total)
{
    long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    int k = (int)(idx % K);
    long long t = idx / K;
    int ow = (int)(t % OW);
    t /= OW;
    int oh = (int)(t % OH);
    long long n = t / OH;
    constexpr int NCLS = KW + KA - 1;
    uint32_t cls[NCLS];
#pragma unroll
    for (int c = 0; c < NCLS; ++c) cls[c] = 0u;
    const int RS = R * S;
    const uint32_t *wk = wgt + ((long long)(k / kWgtGroup) * RS * cw * kWgtGroup + (k % kWgtGroup)) * KW;
    const int Hp = H + 2 * kActBorder, Wp = W + 2 * kActBorder;
    for (int r = 0; r < R; ++r) {
        int hp = oh * stride + r - pad + kActBorder;      // row in the bordered grid
        if (hp < 0 || hp >= Hp) continue;                // beyond the stored zero ring: contributes 0
        for (int s = 0; s < S; ++s) {
            int wcol = ow * stride + s - pad + kActBorder;
            if (wcol < 0 || wcol >= Wp) continue;
            const uint32_t *ap = act + (((n * Hp + hp) * Wp + wcol) * cw) * KA;
            const uint32_t *wp = wk + (long long)(r * S + s) * cw * kWgtGroup * KW;
            for (int word = 0; word < cw; ++word) {
                uint32_t x[KA], q[KW];
#pragma unroll
                for (int j = 0; j < KA; ++j) x[j] = ap[word * KA + j];
#pragma unroll
                for (int i = 0; i < KW; ++i) q[i] = wp[(long long)word * kWgtGroup * KW + i];
#pragma unroll
                for (int i = 0; i < KW; ++i)
#pragma unroll
                    for (int j = 0; j < KA; ++j) cls[i + j] += __builtin_popcount(q[i] & x[j]);
            }
        }
    }
    uint32_t acc = 0;
#pragma unroll
    for (int c = 0; c < NCLS; ++c) acc += cls[c] << c;
    acc_out[idx] = (int32_t)acc;
    if (out_f32) {
        int ci = per_channel ? k : 0;
        float of = offset ? offset[ci] : 0.0f;
        out_f32[idx] = fmaf((float)(int32_t)acc, scale[ci], of);
    }
}

template <int KW, int KA>
static int launch(const ConvArgs &a)
{
    long long total = (long long)a.N * a.OH * a.OW * a.K;
    unsigned blocks = (unsigned)((total + 255) / 256);
    hipLaunchKernelGGL((bd_conv_naive<KW, KA>), dim3(blocks), dim3(256), 0, a.stream,
                       a.act, a.wgt, a.H, a.W, a.K, a.R, a.S, a.stride, a.pad, a.OH, a.OW, a.cw,
                       a.scale, a.offset, a.per_channel, a.acc, a.out, total);
    return hip_ok(hipGetLastError());
}

int launch_conv_naive(const ConvArgs &a)
{
#define EBS_CASE(w, x) case (w) * 8 + (x): return launch<w, x>(a);
    switch (a.kw * 8 + a.ka) {
        EBS_CASE(1, 1) EBS_CASE(1, 2) EBS_CASE(1, 3) EBS_CASE(1, 4)
        EBS_CASE(2, 1) EBS_CASE(2, 2) EBS_CASE(2, 3) EBS_CASE(2, 4)
        EBS_CASE(3, 1) EBS_CASE(3, 2) EBS_CASE(3, 3) EBS_CASE(3, 4)
        EBS_CASE(4, 1) EBS_CASE(4, 2) EBS_CASE(4, 3) EBS_CASE(4, 4)
    }
#undef EBS_CASE
    return EBS_ERR_BITWIDTH;
}

}  // namespace ebs
