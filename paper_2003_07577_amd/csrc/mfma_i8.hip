// Measured comparison only: the same integer convolution taken directly on the
// unpacked levels with int8 matrix instructions (v_mfma_i32_32x32x32_i8), i.e.
// WITHOUT binary decomposition.  It exists to report, on the same layers, what
// the matrix cores deliver for the product that Sec. 3 Eq. 2 evaluates with
// AND + bitcount; it is not on the default path.
//
// Implicit GEMM: rows = output positions t = (n*OH+oh)*OW+ow, columns = output
// channels, reduction = (r, s, c) with c innermost (NHWC activations and KRSC
// weights are both contiguous in c).  A wave owns MT x NT blocks of 32 x 32
// outputs; per reduction step of 32 channels each lane loads 16 bytes per
// block row / column straight from global memory (operands are re-read through
// L1/L2 by neighbouring waves).  Needs C % 32 == 0 and levels < 128.
#include "ebs_internal.h"

namespace ebs {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

template <int MT, int NT>
__global__ void __launch_bounds__(256)
mfma_i8_conv(const uint8_t *__restrict__ act, const uint8_t *__restrict__ wgt,
             int N, int C, int H, int W, int K, int R, int S, int stride, int pad, int OH, int OW,
             const float *__restrict__ scale, const float *__restrict__ offset, int per_channel,
             int32_t *__restrict__ acc_out, float *__restrict__ out_f32, int total)
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int row = lane & 31;          // row of A / column of B this lane supplies
    const int half = lane >> 5;         // which 16 of the 32 reduction bytes of a step
    const int t0 = (blockIdx.x * 4 + wave) * (32 * MT);
    const int k0 = blockIdx.y * (32 * NT);
    if (t0 >= total) return;

    // positions of this lane's A rows
    int pn[MT], ph[MT], pw[MT];
#pragma unroll
    for (int mi = 0; mi < MT; ++mi) {
        int t = t0 + mi * 32 + row;
        if (t > total - 1) t = total - 1;
        const int ow = t % OW;
        const int tt = t / OW;
        pw[mi] = ow * stride - pad;
        ph[mi] = (tt % OH) * stride - pad;
        pn[mi] = tt / OH;
    }
    // weight rows of this lane's B columns (clamped: columns beyond K are never stored)
    const uint8_t *wrow[NT];
#pragma unroll
    for (int ni = 0; ni < NT; ++ni) {
        int k = k0 + ni * 32 + row;
        if (k > K - 1) k = K - 1;
        wrow[ni] = wgt + (size_t)k * R * S * C + half * 16;
    }

    v16i acc[MT][NT];
#pragma unroll
    for (int mi = 0; mi < MT; ++mi)
#pragma unroll
        for (int ni = 0; ni < NT; ++ni)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0;

    for (int r = 0; r < R; ++r) {
        for (int s = 0; s < S; ++s) {
            const uint8_t *arow[MT];
            bool ok[MT];
#pragma unroll
            for (int mi = 0; mi < MT; ++mi) {
                const int h = ph[mi] + r, w = pw[mi] + s;
                ok[mi] = h >= 0 && h < H && w >= 0 && w < W;
                arow[mi] = act + (((size_t)pn[mi] * H + (ok[mi] ? h : 0)) * W + (ok[mi] ? w : 0)) * C + half * 16;
            }
            const size_t wtap = (size_t)(r * S + s) * C;
            for (int c = 0; c < C; c += 32) {
                v4i a[MT], b[NT];
#pragma unroll
                for (int mi = 0; mi < MT; ++mi) {
                    a[mi] = *reinterpret_cast<const v4i *>(arow[mi] + c);
                    if (!ok[mi]) a[mi] = v4i{0, 0, 0, 0};            // zero padding
                }
#pragma unroll
                for (int ni = 0; ni < NT; ++ni) b[ni] = *reinterpret_cast<const v4i *>(wrow[ni] + wtap + c);
#pragma unroll
                for (int mi = 0; mi < MT; ++mi)
#pragma unroll
                    for (int ni = 0; ni < NT; ++ni)
                        acc[mi][ni] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[mi], b[ni], acc[mi][ni], 0, 0, 0);
            }
        }
    }

    // accumulator v of a lane: output row 8*(v/4) + 4*half + v%4, column `row`
#pragma unroll
    for (int ni = 0; ni < NT; ++ni) {
        const int k = k0 + ni * 32 + row;
        if (k >= K) continue;
        const int ci = per_channel ? k : 0;
        const float sc = scale[ci];
        const float of = offset ? offset[ci] : 0.0f;
#pragma unroll
        for (int mi = 0; mi < MT; ++mi)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int t = t0 + mi * 32 + 8 * (v / 4) + 4 * half + (v % 4);
                if (t < total) {
                    const size_t o = (size_t)t * K + k;
                    const int val = acc[mi][ni][v];
                    acc_out[o] = val;
                    if (out_f32) out_f32[o] = fmaf((float)val, sc, of);
                }
            }
    }
}

int launch_conv_mfma_i8(const uint8_t *act, const uint8_t *wgt, const ConvArgs &a)
{
    if (a.C % 32 != 0) return EBS_ERR_UNSUPPORTED;
    const int total = a.N * a.OH * a.OW;
    constexpr int MT = 2;
    const bool wide = a.K > 64;
    const int nt = wide ? 4 : 2;
    const long long gx = ((long long)total + 4 * 32 * MT - 1) / (4 * 32 * MT);
    const long long gy = ((long long)a.K + 32 * nt - 1) / (32 * nt);
    if (gx > 0x7fffffffLL || gy > 65535) return EBS_ERR_UNSUPPORTED;
    dim3 grid((unsigned)gx, (unsigned)gy);
    if (wide)
        hipLaunchKernelGGL((mfma_i8_conv<MT, 4>), grid, dim3(256), 0, a.stream, act, wgt, a.N, a.C, a.H, a.W, a.K, a.R, a.S,
                           a.stride, a.pad, a.OH, a.OW, a.scale, a.offset, a.per_channel, a.acc, a.out, total);
    else
        hipLaunchKernelGGL((mfma_i8_conv<MT, 2>), grid, dim3(256), 0, a.stream, act, wgt, a.N, a.C, a.H, a.W, a.K, a.R, a.S,
                           a.stride, a.pad, a.OH, a.OW, a.scale, a.offset, a.per_channel, a.acc, a.out, total);
    return hip_ok(hipGetLastError());
}

}  // namespace ebs
