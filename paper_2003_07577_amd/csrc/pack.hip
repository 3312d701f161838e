// Bit-plane packing: levels -> binary matrices B_w / B_x (paper Sec. 3, the
// expansion w = sum_m c_m 2^m; Sec. 4.3, Eq. 12 and 15), channel bits packed
// into 32-bit words.
//
// Activations: uint32 [word][n][h+1][w+1][plane] over a (H+2) x (W+2) grid per
// image whose outer ring of positions is all zero (activation level 0 is the
// real value 0, so the ring is the convolution's zero padding); word = c / 32,
// bit c % 32 of the word of plane j is digit j of channel c.  Channel bits
// beyond C are zero.  Keeping the k_a planes of one word adjacent lets the
// convolution fetch all planes of a reduction word with a single wide load;
// keeping the positions of one word adjacent makes the run of input positions
// a filter row touches, for one reduction word, one contiguous piece of memory
// (what a wave can fetch with scalar loads, and what a tile stages as a copy).
//
// Weights: uint32 [k / 16][tap = r*S+s][word][k % 16][plane]; output channels
// beyond K (up to the next multiple of 16) are zero.  One reduction step of a
// 16-channel group is k_w*16 consecutive words, which a wave can fetch with
// scalar loads.  3x3 layers with C <= 16 carry a second section behind it with
// two taps per word (pack_wgt_pairs).
#include "ebs_internal.h"
#include "fastdiv.h"

namespace ebs {

// 32 channels of one position -> k planes.  Generic path: any C, byte loads.
// One thread per (bordered position, word); border positions store zeros.
template <int BITS>
__global__ void __launch_bounds__(256)
pack_act_generic(const uint8_t *__restrict__ levels, uint32_t *__restrict__ packed,
                 long long n_items /* N*(H+2)*(W+2)*cw */, int H, int W, int C, int cw)
{
    long long item = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (item >= n_items) return;
    long long pos = item / cw;
    int word = (int)(item - pos * cw);
    const int Wp = W + 2 * kActBorder, Hp = H + 2 * kActBorder;
    int wp = (int)(pos % Wp);
    long long t = pos / Wp;
    int hp = (int)(t % Hp);
    long long n = t / Hp;
    int h = hp - kActBorder, w = wp - kActBorder;
    uint32_t planes[BITS];
#pragma unroll
    for (int j = 0; j < BITS; ++j) planes[j] = 0u;
    if (h >= 0 && h < H && w >= 0 && w < W) {
        int c0 = word * 32;
        const uint8_t *src = levels + ((n * H + h) * W + w) * C + c0;
        int nvalid = C - c0 < 32 ? C - c0 : 32;
        for (int c = 0; c < nvalid; ++c) {
            uint32_t lv = src[c];
#pragma unroll
            for (int j = 0; j < BITS; ++j) planes[j] |= ((lv >> j) & 1u) << c;
        }
    }
    const long long total_pos = n_items / cw;
#pragma unroll
    for (int j = 0; j < BITS; ++j) packed[((long long)word * total_pos + pos) * BITS + j] = planes[j];
}

// ---- fast path for C % 32 == 0: 32 one-byte levels -> BITS plane words in registers.
//
// d[0..7] hold channels 4i..4i+3 (one byte each).  After masking to the low
// nibble, d[2m] | d[2m+1] << 4 puts channel 8m+r in the low nibble and channel
// 8m+4+r in the high nibble of byte r: a 4(byte r) x 4(digit j) bit matrix in
// each nibble column.  Two delta swaps transpose r <-> j, so that byte j holds
// digit j of the 8 channels; a 4x4 byte transpose over the four groups then
// yields one 32-bit word per digit.
__device__ __forceinline__ uint32_t swap_rj(uint32_t v)
{
    uint32_t t = (v ^ (v >> 7)) & 0x00AA00AAu;     // (r0=0, j0=1) <-> (r0=1, j0=0): distance 8-1
    v ^= t | (t << 7);
    t = (v ^ (v >> 14)) & 0x0000CCCCu;             // (r1=0, j1=1) <-> (r1=1, j1=0): distance 16-2
    v ^= t | (t << 14);
    return v;
}

__device__ __forceinline__ void planes_of_32(const uint32_t (&d)[8], uint32_t (&plane)[4])
{
    uint32_t v[4];
#pragma unroll
    for (int m = 0; m < 4; ++m)
        v[m] = swap_rj((d[2 * m] & 0x0F0F0F0Fu) | ((d[2 * m + 1] & 0x0F0F0F0Fu) << 4));
    // byte j of v[m] = digit j of channels 8m..8m+7  ->  word j = bytes j of v[0..3]
    const uint32_t lo01 = __builtin_amdgcn_perm(v[1], v[0], 0x05010400u);   // v0.b0 v1.b0 v0.b1 v1.b1
    const uint32_t hi01 = __builtin_amdgcn_perm(v[1], v[0], 0x07030602u);   // v0.b2 v1.b2 v0.b3 v1.b3
    const uint32_t lo23 = __builtin_amdgcn_perm(v[3], v[2], 0x05010400u);
    const uint32_t hi23 = __builtin_amdgcn_perm(v[3], v[2], 0x07030602u);
    plane[0] = __builtin_amdgcn_perm(lo23, lo01, 0x05040100u);             // lo01.b0 lo01.b1 lo23.b0 lo23.b1
    plane[1] = __builtin_amdgcn_perm(lo23, lo01, 0x07060302u);
    plane[2] = __builtin_amdgcn_perm(hi23, hi01, 0x05040100u);
    plane[3] = __builtin_amdgcn_perm(hi23, hi01, 0x07060302u);
}

// Digit 4 of the same 32 levels: bit 4 of byte r of d[i] is channel 4i+r.  The multiply gathers the
// four bits (at 0, 8, 16, 24 after the shift and mask) into bits 24..27; no two partial products meet.
__device__ __forceinline__ uint32_t fifth_plane_of_32(const uint32_t (&d)[8])
{
    uint32_t p = 0u;
#pragma unroll
    for (int i = 0; i < 8; ++i) p |= ((((d[i] >> 4) & 0x01010101u) * 0x01020408u) >> 24 & 0xFu) << (4 * i);
    return p;
}

template <int BITS>
__global__ void __launch_bounds__(256)
pack_act_c32(const uint8_t *__restrict__ levels, uint32_t *__restrict__ packed,
             int H, int W, int C, int cw, int items_per_image, FastDiv div_cw, FastDiv div_wp)
{
    const int item = blockIdx.x * 256 + threadIdx.x;          // (bordered position, word) inside image blockIdx.y
    if (item >= items_per_image) return;
    const int n = blockIdx.y;
    const int Wp = W + 2 * kActBorder;
    const int pos = (int)fd_div((uint32_t)item, div_cw);
    const int word = item - pos * cw;
    const int hp = (int)fd_div((uint32_t)pos, div_wp);
    const int wp = pos - hp * Wp;
    const int h = hp - kActBorder, w = wp - kActBorder;
    uint32_t plane[5] = {0u, 0u, 0u, 0u, 0u};
    if (h >= 0 && h < H && w >= 0 && w < W) {
        const uint4 *src = reinterpret_cast<const uint4 *>(levels + (((size_t)n * H + h) * W + w) * C + word * 32);
        const uint4 a = src[0], b = src[1];
        const uint32_t d[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
        uint32_t low[4];
        planes_of_32(d, low);
#pragma unroll
        for (int j = 0; j < 4; ++j) plane[j] = low[j];
        if (BITS == 5) plane[4] = fifth_plane_of_32(d);
    }
    const size_t pos_per_image = (size_t)(H + 2 * kActBorder) * Wp;
    uint32_t *dst = packed + (((size_t)word * gridDim.y + n) * pos_per_image + pos) * BITS;
#pragma unroll
    for (int j = 0; j < BITS; ++j) dst[j] = plane[j];
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

// Second section of the packed weights of 3x3 layers with C <= 16: two taps per word, five words per
// plane, uint32 [k][word][plane] for k < ceil16(K) (zero beyond K):
//   word 0..2 = taps (r,0) | (r,1) << 16 for r = 0..2, word 3 = taps (0,2) | (1,2) << 16, word 4 = tap (2,2).
// One thread per (k, word).
template <int BITS>
__global__ void __launch_bounds__(256)
pack_wgt_pairs(const uint8_t *__restrict__ levels, uint32_t *__restrict__ pairs, int K, int C, int n_items /* Kpad*5 */)
{
    const int item = blockIdx.x * blockDim.x + threadIdx.x;
    if (item >= n_items) return;
    const int k = item / 5, t5 = item - k * 5;
    const int tap_lo = t5 < 3 ? 3 * t5 : (t5 == 3 ? 2 : 8);
    const int tap_hi = t5 < 3 ? 3 * t5 + 1 : (t5 == 3 ? 5 : -1);
    uint32_t planes[BITS];
#pragma unroll
    for (int i = 0; i < BITS; ++i) planes[i] = 0u;
    if (k < K) {
        for (int half = 0; half < 2; ++half) {
            const int tap = half ? tap_hi : tap_lo;
            if (tap < 0) continue;
            const uint8_t *src = levels + ((long long)k * 9 + tap) * C;
            for (int c = 0; c < C; ++c) {
                const uint32_t lv = src[c];
#pragma unroll
                for (int i = 0; i < BITS; ++i) planes[i] |= ((lv >> i) & 1u) << (c + 16 * half);
            }
        }
    }
#pragma unroll
    for (int i = 0; i < BITS; ++i) pairs[(size_t)item * BITS + i] = planes[i];
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
static int launch_pack_act(const uint8_t *levels, uint32_t *packed, int N, int H, int W, int C, hipStream_t st)
{
    int cw = words_per_pixel(C);
    long long per_image = (long long)(H + 2 * kActBorder) * (W + 2 * kActBorder) * cw;
    if (C % 32 == 0 && N <= 65535 && per_image < (1LL << 30)) {
        unsigned bx = (unsigned)((per_image + 255) / 256);
        hipLaunchKernelGGL(pack_act_c32<BITS>, dim3(bx, (unsigned)N), dim3(256), 0, st, levels, packed, H, W, C, cw,
                           (int)per_image, make_fastdiv((uint32_t)cw), make_fastdiv((uint32_t)(W + 2 * kActBorder)));
        return hip_ok(hipGetLastError());
    }
    long long items = (long long)N * per_image;
    unsigned blocks = (unsigned)((items + 255) / 256);
    hipLaunchKernelGGL(pack_act_generic<BITS>, dim3(blocks), dim3(256), 0, st, levels, packed, items, H, W, C, cw);
    return hip_ok(hipGetLastError());
}

template <int BITS>
static int launch_pack_wgt(const uint8_t *levels, uint32_t *packed, int K, int C, int R, int S, hipStream_t st)
{
    const int RS = R * S;
    int cw = words_per_pixel(C);
    long long kpad = (long long)((K + kWgtGroup - 1) / kWgtGroup) * kWgtGroup;
    long long items = kpad * RS * cw;
    unsigned blocks = (unsigned)((items + 255) / 256);
    hipLaunchKernelGGL(pack_wgt_generic<BITS>, dim3(blocks), dim3(256), 0, st, levels, packed, K, C, RS, cw, items);
    if (has_pair_section(C, R, S)) {
        const int n_items = (int)kpad * 5;
        hipLaunchKernelGGL(pack_wgt_pairs<BITS>, dim3((unsigned)((n_items + 255) / 256)), dim3(256), 0, st, levels,
                           packed + items * BITS, K, C, n_items);
    }
    return hip_ok(hipGetLastError());
}

int pack_activations(const uint8_t *levels, uint32_t *packed, int N, int H, int W, int C, int bits, hipStream_t st)
{
    switch (bits) {
        case 1: return launch_pack_act<1>(levels, packed, N, H, W, C, st);
        case 2: return launch_pack_act<2>(levels, packed, N, H, W, C, st);
        case 3: return launch_pack_act<3>(levels, packed, N, H, W, C, st);
        case 4: return launch_pack_act<4>(levels, packed, N, H, W, C, st);
        case 5: return launch_pack_act<5>(levels, packed, N, H, W, C, st);
    }
    return EBS_ERR_BITWIDTH;
}

int pack_weights(const uint8_t *levels, uint32_t *packed, int K, int C, int R, int S, int bits, hipStream_t st)
{
    switch (bits) {
        case 1: return launch_pack_wgt<1>(levels, packed, K, C, R, S, st);
        case 2: return launch_pack_wgt<2>(levels, packed, K, C, R, S, st);
        case 3: return launch_pack_wgt<3>(levels, packed, K, C, R, S, st);
        case 4: return launch_pack_wgt<4>(levels, packed, K, C, R, S, st);
        case 5: return launch_pack_wgt<5>(levels, packed, K, C, R, S, st);
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
