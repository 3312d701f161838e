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
// L1/L2 by neighbouring waves).  Needs C % 32 == 0 and levels < 128.  For C % 64 == 0 an
// LDS-tiled version (below) is used instead.
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

// ---- LDS-tiled version for C % 64 == 0: a work-group owns 64*MB output positions x 64*NB
// channels; per reduction step (one filter tap, 32*KK input channels) the A tile (activation
// levels, zero where the tap leaves the image) and the B tile (weight levels) are copied with
// coalesced 16-byte loads into LDS (next step's data waits in registers during the matrix work),
// and each of the 2 x 2 waves runs MB x NB x KK matrix instructions on its 32*MB x 32*NB sub-tile.
template <int MB, int NB, int KK>
__global__ void __launch_bounds__(256)
mfma_i8_conv_tiled(const uint8_t *__restrict__ act, const uint8_t *__restrict__ wgt,
                   int N, int C, int H, int W, int K, int R, int S, int stride, int pad, int OH, int OW,
                   const float *__restrict__ scale, const float *__restrict__ offset, int per_channel,
                   int32_t *__restrict__ acc_out, float *__restrict__ out_f32, int total)
{
    constexpr int BM = 64 * MB, BN = 64 * NB, BK = 32 * KK, PITCH = BK + 16;   // bytes per LDS row, padded
    constexpr int CPR = BK / 16;                                // 16-byte pieces per row
    constexpr int A_LOADS = BM * CPR / 256, B_LOADS = BN * CPR / 256;
    constexpr int A_BYTES = BM * PITCH;
    __shared__ __attribute__((aligned(16))) uint8_t lds[(BM + BN) * PITCH];
    uint8_t *const la = lds;
    uint8_t *const lb = lds + A_BYTES;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave & 1, wn = wave >> 1;
    const int row = lane & 31, half = lane >> 5;
    const int t0 = blockIdx.x * BM;
    const int k0 = blockIdx.y * BN;

    // global -> LDS assignment: piece q = tid + 256*i; row = q / CPR, 16-byte column = q % CPR
    int an[A_LOADS], ah[A_LOADS], aw[A_LOADS];
#pragma unroll
    for (int i = 0; i < A_LOADS; ++i) {
        int t = t0 + (tid + 256 * i) / CPR;
        if (t > total - 1) t = total - 1;
        const int ow = t % OW;
        const int tt = t / OW;
        aw[i] = ow * stride - pad;
        ah[i] = (tt % OH) * stride - pad;
        an[i] = tt / OH;
    }
    const uint8_t *brow[B_LOADS];
#pragma unroll
    for (int i = 0; i < B_LOADS; ++i) {
        int k = k0 + (tid + 256 * i) / CPR;
        if (k > K - 1) k = K - 1;
        brow[i] = wgt + (size_t)k * R * S * C + ((tid + 256 * i) % CPR) * 16;
    }
    const int csteps = C / BK;
    const int nsteps = R * S * csteps;

    v4i ra[A_LOADS], rb[B_LOADS];
    auto gload = [&](int step) {
        const int tap = step / csteps;
        const int c0 = (step - tap * csteps) * BK;
        const int r = tap / S, s = tap - r * S;
#pragma unroll
        for (int i = 0; i < A_LOADS; ++i) {
            const int h = ah[i] + r, w = aw[i] + s;
            const bool ok = h >= 0 && h < H && w >= 0 && w < W;
            ra[i] = v4i{0, 0, 0, 0};
            if (ok)
                ra[i] = *reinterpret_cast<const v4i *>(act + (((size_t)an[i] * H + h) * W + w) * C + c0 +
                                                      ((tid + 256 * i) % CPR) * 16);
        }
#pragma unroll
        for (int i = 0; i < B_LOADS; ++i) rb[i] = *reinterpret_cast<const v4i *>(brow[i] + (size_t)tap * C + c0);
    };
    auto lstore = [&]() {
#pragma unroll
        for (int i = 0; i < A_LOADS; ++i)
            *reinterpret_cast<v4i *>(la + ((tid + 256 * i) / CPR) * PITCH + ((tid + 256 * i) % CPR) * 16) = ra[i];
#pragma unroll
        for (int i = 0; i < B_LOADS; ++i)
            *reinterpret_cast<v4i *>(lb + ((tid + 256 * i) / CPR) * PITCH + ((tid + 256 * i) % CPR) * 16) = rb[i];
    };

    v16i acc[MB][NB];
#pragma unroll
    for (int mi = 0; mi < MB; ++mi)
#pragma unroll
        for (int ni = 0; ni < NB; ++ni)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0;

    gload(0);
    lstore();
    __syncthreads();
    const uint8_t *pa = la + (wm * 32 * MB + row) * PITCH + half * 16;
    const uint8_t *pb = lb + (wn * 32 * NB + row) * PITCH + half * 16;
    for (int step = 0; step < nsteps; ++step) {
        if (step + 1 < nsteps) gload(step + 1);                 // in flight during the matrix work
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
            v4i a[MB], b[NB];
#pragma unroll
            for (int mi = 0; mi < MB; ++mi) a[mi] = *reinterpret_cast<const v4i *>(pa + mi * 32 * PITCH + kk * 32);
#pragma unroll
            for (int ni = 0; ni < NB; ++ni) b[ni] = *reinterpret_cast<const v4i *>(pb + ni * 32 * PITCH + kk * 32);
#pragma unroll
            for (int mi = 0; mi < MB; ++mi)
#pragma unroll
                for (int ni = 0; ni < NB; ++ni)
                    acc[mi][ni] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[mi], b[ni], acc[mi][ni], 0, 0, 0);
        }
        __syncthreads();                                        // everyone has read this step's tiles
        if (step + 1 < nsteps) lstore();
        __syncthreads();
    }

#pragma unroll
    for (int ni = 0; ni < NB; ++ni) {
        const int k = k0 + wn * 32 * NB + ni * 32 + row;
        if (k >= K) continue;
        const int ci = per_channel ? k : 0;
        const float sc = scale[ci];
        const float of = offset ? offset[ci] : 0.0f;
#pragma unroll
        for (int mi = 0; mi < MB; ++mi)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int t = t0 + wm * 32 * MB + mi * 32 + 8 * (v / 4) + 4 * half + (v % 4);
                if (t < total) {
                    const size_t o = (size_t)t * K + k;
                    const int val = acc[mi][ni][v];
                    acc_out[o] = val;
                    if (out_f32) out_f32[o] = fmaf((float)val, sc, of);
                }
            }
    }
}

template <int MB, int NB, int KK>
static int launch_mfma_tiled(const uint8_t *act, const uint8_t *wgt, const ConvArgs &a, int total)
{
    const long long bx = ((long long)total + 64 * MB - 1) / (64 * MB);
    const long long by = ((long long)a.K + 64 * NB - 1) / (64 * NB);
    if (bx > 0x7fffffffLL || by > 65535) return EBS_ERR_UNSUPPORTED;
    hipLaunchKernelGGL((mfma_i8_conv_tiled<MB, NB, KK>), dim3((unsigned)bx, (unsigned)by), dim3(256), 0, a.stream, act, wgt,
                       a.N, a.C, a.H, a.W, a.K, a.R, a.S, a.stride, a.pad, a.OH, a.OW, a.scale, a.offset, a.per_channel,
                       a.acc, a.out, total);
    return hip_ok(hipGetLastError());
}

int launch_conv_mfma_i8(const uint8_t *act, const uint8_t *wgt, const ConvArgs &a)
{
    if (a.C % 32 != 0) return EBS_ERR_UNSUPPORTED;
    const int total = a.N * a.OH * a.OW;
    if (a.C % 64 == 0) {
        // tile choice: wide channel tile when the layer has the channels, deep reduction steps when
        // C allows, and the smaller position tile when the larger one would leave compute units idle
        // 128-channel tiles only where they still leave at least two work-groups per compute unit
        const bool nb2 = a.K > 64 && (((long long)total + 63) / 64) * (((long long)a.K + 127) / 128) >= 512;
        const bool kk4 = a.C % 128 == 0;
        const long long big_blocks = (((long long)total + 127) / 128) * (((long long)a.K + (nb2 ? 127 : 63)) / (nb2 ? 128 : 64));
        const bool mb2 = big_blocks >= 1024;
        int rc;
#define EBS_MF(mb, nb, kk) rc = launch_mfma_tiled<mb, nb, kk>(act, wgt, a, total)
        if (mb2) { if (nb2) { if (kk4) EBS_MF(2, 2, 4); else EBS_MF(2, 2, 2); } else { if (kk4) EBS_MF(2, 1, 4); else EBS_MF(2, 1, 2); } }
        else     { if (nb2) { if (kk4) EBS_MF(1, 2, 4); else EBS_MF(1, 2, 2); } else { if (kk4) EBS_MF(1, 1, 4); else EBS_MF(1, 1, 2); } }
#undef EBS_MF
        if (rc != EBS_ERR_UNSUPPORTED) return rc;
    }
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
