// Bit-plane packing: levels -> binary matrices B_w / B_x (paper Sec. 3, the
// expansion w = sum_m c_m 2^m; Sec. 4.3, Eq. 12 and 15), channel bits packed
// into 32-bit words.
//
// Activations: uint32 [pixel = (n*H+h)*W+w][word][plane], word = c / 32, bit
// c % 32 of the word of plane j is digit j of channel c.  Channel bits beyond C
// are zero.  Keeping the k_a planes of one word adjacent lets the convolution
// fetch all planes of a reduction word with a single wide load.
//
// Weights: uint32 [k / 16][tap = r*S+s][word][k % 16][plane]; output channels
// beyond K (up to the next multiple of 16) are zero.  One reduction step of a
// 16-channel group is k_w*16 consecutive words, which a wave can fetch with
// scalar loads.
#include "ebs_internal.h"

namespace ebs {

// 32 channels of one pixel -> k planes.  Generic path: any C, byte loads.
template <int BITS>
__global__ void __launch_bounds__(256)
pack_act_generic(const uint8_t *__restrict__ levels, uint32_t *__restrict__ packed,
                 long long n_items /* pixels*cw */, int C, int cw)
{
    long long item = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (item >= n_items) return;
    long long pix = item / cw;
    int word = (int)(item - pix * cw);
    int c0 = word * 32;
    const uint8_t *src = levels + pix * C + c0;
    int nvalid = C - c0 < 32 ? C - c0 : 32;
    uint32_t planes[BITS];
#pragma unroll
    for (int j = 0; j < BITS; ++j) planes[j] = 0u;
    for (int c = 0; c < nvalid; ++c) {
        uint32_t lv = src[c];
#pragma unroll
        for (int j = 0; j < BITS; ++j) planes[j] |= ((lv >> j) & 1u) << c;
    }
#pragma unroll
    for (int j = 0; j < BITS; ++j) packed[item * BITS + j] = planes[j];
}

template <int BITS>
__global__ void __launch_bounds__(256)
pack_wgt_generic(const uint8_t *__restrict__ levels, uint32_t *__restrict__ packed,
                 int K, int C, int RS, int cw, long long n_items /* Kpad*RS*cw */)
{
    long long item = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (item >= n_items) return;
    // item enumerates the OUTPUT layout: ((kg*RS + tap)*cw + word)*16 + kl
    int kl = (int)(item % kWgtGroup);
    long long t = item / kWgtGroup;
    int word = (int)(t % cw);
    t /= cw;
    int tap = (int)(t % RS);
    int kg = (int)(t / RS);
    int k = kg * kWgtGroup + kl;
    uint32_t planes[BITS];
#pragma unroll
    for (int i = 0; i < BITS; ++i) planes[i] = 0u;
    if (k < K) {
        int c0 = word * 32;
        int nvalid = C - c0 < 32 ? C - c0 : 32;
        const uint8_t *src = levels + ((long long)k * RS + tap) * C + c0;
        for (int c = 0; c < nvalid; ++c) {
            uint32_t lv = src[c];
#pragma unroll
            for (int i = 0; i < BITS; ++i) planes[i] |= ((lv >> i) & 1u) << c;
        }
    }
#pragma unroll
    for (int i = 0; i < BITS; ++i) packed[item * BITS + i] = planes[i];
}

__global__ void clear_flag_kernel(int32_t *flag) { *flag = 0; }

__global__ void __launch_bounds__(256)
check_levels_kernel(const uint8_t *__restrict__ levels, size_t count, unsigned limit, int32_t *flag)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t step = (size_t)gridDim.x * blockDim.x;
    int bad = 0;
    for (; i < count; i += step) bad |= levels[i] >= limit;
    if (bad) atomicOr(flag, 1);
}

template <int BITS>
static int launch_pack_act(const uint8_t *levels, uint32_t *packed, long long pixels, int C, hipStream_t st)
{
    int cw = words_per_pixel(C);
    long long items = pixels * cw;
    unsigned blocks = (unsigned)((items + 255) / 256);
    hipLaunchKernelGGL(pack_act_generic<BITS>, dim3(blocks), dim3(256), 0, st, levels, packed, items, C, cw);
    return hip_ok(hipGetLastError());
}

template <int BITS>
static int launch_pack_wgt(const uint8_t *levels, uint32_t *packed, int K, int C, int RS, hipStream_t st)
{
    int cw = words_per_pixel(C);
    long long kpad = (long long)((K + kWgtGroup - 1) / kWgtGroup) * kWgtGroup;
    long long items = kpad * RS * cw;
    unsigned blocks = (unsigned)((items + 255) / 256);
    hipLaunchKernelGGL(pack_wgt_generic<BITS>, dim3(blocks), dim3(256), 0, st, levels, packed, K, C, RS, cw, items);
    return hip_ok(hipGetLastError());
}

int pack_activations(const uint8_t *levels, uint32_t *packed, long long pixels, int C, int bits, hipStream_t st)
{
    switch (bits) {
        case 1: return launch_pack_act<1>(levels, packed, pixels, C, st);
        case 2: return launch_pack_act<2>(levels, packed, pixels, C, st);
        case 3: return launch_pack_act<3>(levels, packed, pixels, C, st);
        case 4: return launch_pack_act<4>(levels, packed, pixels, C, st);
    }
    return EBS_ERR_BITWIDTH;
}

int pack_weights(const uint8_t *levels, uint32_t *packed, int K, int C, int RS, int bits, hipStream_t st)
{
    switch (bits) {
        case 1: return launch_pack_wgt<1>(levels, packed, K, C, RS, st);
        case 2: return launch_pack_wgt<2>(levels, packed, K, C, RS, st);
        case 3: return launch_pack_wgt<3>(levels, packed, K, C, RS, st);
        case 4: return launch_pack_wgt<4>(levels, packed, K, C, RS, st);
    }
    return EBS_ERR_BITWIDTH;
}

int check_levels(const uint8_t *levels, size_t count, int bits, int32_t *flag, hipStream_t st)
{
    hipLaunchKernelGGL(clear_flag_kernel, dim3(1), dim3(1), 0, st, flag);
    size_t want = (count + 255) / 256;
    unsigned blocks = (unsigned)(want < 4096 ? (want ? want : 1) : 4096);
    hipLaunchKernelGGL(check_levels_kernel, dim3(blocks), dim3(256), 0, st, levels, count, 1u << bits, flag);
    return hip_ok(hipGetLastError());
}

}  // namespace ebs
