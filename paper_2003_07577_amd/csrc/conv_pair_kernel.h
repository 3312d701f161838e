// AND + bitcount convolution for 3x3 layers with at most 16 input channels: two filter taps per
// 32-bit word (paper Sec. 3 Eq. 2; Sec. 4.3 Eq. 13-14 in one kernel, and the complexity count of
// Sec. 4.3, which is in real bits).
//
// With C <= 16 a packed word carries 16 channel bits and 16 zeros, and the one-word-per-tap
// kernels spend half of every AND + bitcount on the zeros.  Here the nine taps of a 3x3 filter
// are paired into five words per plane:
//     word 0..2 : taps (r,0) | (r,1) << 16        for filter row r = 0..2
//     word 3    : taps (0,2) | (1,2) << 16
//     word 4    : tap  (2,2)                      (upper half zero)
// The weights are stored like this once (a second section of the packed weights, written by
// ebs_pack_weights).  The matching activation words are built while a work-group stages its input
// tile into LDS, from the ordinary packed activations: for every staged position u of the
// zero-bordered grid
//     H[u] = x[u] | x[u + 1]  << 16               (horizontal neighbour)
//     V[u] = x[u] | x[u + Wp] << 16               (vertical neighbour, Wp = row length)
// so that the five words of the output whose top-left tap sits at u are H[u], H[u+Wp], H[u+2Wp],
// V[u+2] and H[u+2Wp+2] (the upper half of the last one meets the zero half of weight word 4).
//
// Mapping (CDNA4, 64-wide waves): a lane owns ONE (output position, output channel) pair at a
// time: the KP = 16 or 32 lanes of a group share a position and differ in the channel, a wave
// covers 64 / KP consecutive positions per step.  Both operands of v_and_b32 are vector
// registers: the lane's five weight words per plane stay in registers for the whole kernel, the
// activation words come from LDS (all lanes of a group read the same address).  A wave's 64
// results of a step are consecutive in the NHWC output when K == KP: one full 256-byte store.
// The fused re-quantising form ballots the level bits of a group into the next layer's packed word.
#pragma once
#include "ebs_internal.h"
#include "fastdiv.h"
#include "requant.h"
#include "tile_geometry.h"

namespace ebs {

constexpr int kPairWords = 5;      // words per plane of the paired 3x3 taps

struct PairShape {
    int K, OH, OW, Hp, Wp, stride, origin;
    int total;          // N * OH * OW output positions
    int total_pos;      // N * Hp * Wp positions of the packed input
    int ucap;           // staged positions the LDS allocation holds
    int per_channel;
    int nblocks;
    FastDiv div_ow, div_ohow;
    // fused re-quantisation: next layer's quantiser and packed layout (one word per position: K <= 32)
    float alpha, qs;
    int k_next, OHn, OWn, total_next;
    int ring_total, ring_per_image;
    int wtop;           // signed weights: 2^k_w - 1 (else 0)
};

__device__ __forceinline__ uint32_t pair_bcnt_acc(uint32_t x, uint32_t acc)
{
    uint32_t d;
    asm("v_bcnt_u32_b32 %0, %1, %2" : "=v"(d) : "v"(x), "v"(acc));
    return d;
}
// bitcount alone, for the first product of an accumulator (no clearing)
__device__ __forceinline__ uint32_t pair_bcnt_first(uint32_t x)
{
    uint32_t d;
    asm("v_bcnt_u32_b32 %0, %1, 0" : "=v"(d) : "v"(x));
    return d;
}

// TP: output positions per work-group.  SGN: signed weights (Eq. 1a): the levels q stand for the integers
// 2q - wtop, so the result is 2 * sum(q*a) - wtop * sum(a) with the window sum of the activation levels.
template <int KW, int KA, int KP, bool REQ, int TP, bool SGN>
__global__ void __launch_bounds__(256)
bd_conv_pair(const uint32_t *__restrict__ act, const uint32_t *__restrict__ wpair,
             const float *__restrict__ scale, const float *__restrict__ offset,
             int32_t *__restrict__ acc_out, float *__restrict__ out_f32, uint32_t *__restrict__ packed_next,
             const PairShape sh)
{
    constexpr int NCLS = KW + KA - 1;
    constexpr int G = 64 / KP;                  // positions of a wave per step
    constexpr int kPairTile = TP;
    constexpr int TPW = kPairTile / 4;          // positions of a wave
    constexpr int STEPS = TPW / G;
    static_assert(STEPS % 2 == 0, "the loop takes two steps per trip");
    // LDS: per output position of the tile {offset of its first word in H, its position in the next layer's
    // bordered grid}, its window sum of activation levels (signed weights), then H [ucap][KA], then V [ucap][KA]
    extern __shared__ __attribute__((aligned(16))) uint32_t lds_all[];
    uint2 *tab = reinterpret_cast<uint2 *>(lds_all);
    uint32_t *wsum_tab = lds_all + 2 * kPairTile;
    uint32_t *lds = lds_all + 3 * kPairTile;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int c = lane % KP;                    // output channel of this lane
    const int g = lane / KP;                    // its position inside a step

    const int t_first = blockIdx.x * kPairTile;
    int t_last = t_first + kPairTile - 1;
    if (t_last > sh.total - 1) t_last = sh.total - 1;
    // flat index, in the zero-bordered input grid, of the top-left tap of output t
    auto base_of = [&](int t, int &n, int &oh, int &ow) {
        n = (int)fd_div((uint32_t)t, sh.div_ohow);
        const int rem = t - n * (int)sh.div_ohow.d;
        oh = (int)fd_div((uint32_t)rem, sh.div_ow);
        ow = rem - oh * sh.OW;
        return (n * sh.Hp + oh * sh.stride + sh.origin) * sh.Wp + ow * sh.stride + sh.origin;
    };
    int n_, oh_, ow_;
    const int u_lo = base_of(t_first, n_, oh_, ow_);
    int u_hi = base_of(t_last, n_, oh_, ow_) + 2 * sh.Wp + 2;
    if (u_hi > u_lo + sh.ucap - 1) u_hi = u_lo + sh.ucap - 1;       // never beyond the LDS allocation
    const int n_pos = u_hi - u_lo + 1;

    // ---- staging: the pair words of every position the tile's taps start at.  The neighbours of the last
    //      positions of the whole tensor are clamped: their halves only ever meet zero weight bits.
    {
        const int last = sh.total_pos - 1;
        for (int u = tid; u < n_pos; u += 256) {
            const int ua = u_lo + u;
            const int u1 = ua + 1 < last ? ua + 1 : last;
            const int uw = ua + sh.Wp < last ? ua + sh.Wp : last;
#pragma unroll
            for (int j = 0; j < KA; ++j) {
                const uint32_t a0 = act[(size_t)ua * KA + j];
                const uint32_t a1 = act[(size_t)u1 * KA + j];
                const uint32_t aw = act[(size_t)uw * KA + j];
                lds[u * KA + j] = a0 | (a1 << 16);
                lds[(sh.ucap + u) * KA + j] = a0 | (aw << 16);
            }
        }
    }

    // LDS dword offsets of the five words relative to H[u][0]
    const int row1 = sh.Wp * KA, row2 = 2 * sh.Wp * KA;
    const int vofs = (sh.ucap + 2) * KA;

    // ---- where each output position of the tile reads and writes: worked out once per position here, not
    //      once per lane and step in the loop (positions past the end repeat the last one; they are not stored)
    if constexpr (SGN) __syncthreads();          // the window sums read the staged words
    if (tid < kPairTile) {
        const int t = t_first + tid;
        int n, oh, ow;
        const int b = base_of(t < sh.total ? t : sh.total - 1, n, oh, ow);
        uint2 e;
        e.x = (uint32_t)((b - u_lo) * KA);
        e.y = REQ ? (uint32_t)((n * sh.OHn + oh + kActBorder) * sh.OWn + ow + kActBorder) : 0u;
        tab[tid] = e;
        if constexpr (SGN) {
            uint32_t ws = 0;
#pragma unroll
            for (int j = 0; j < KA; ++j) {
                const uint32_t cnt = __builtin_popcount(lds[e.x + j]) + __builtin_popcount(lds[e.x + row1 + j]) +
                                     __builtin_popcount(lds[e.x + row2 + j]) + __builtin_popcount(lds[e.x + vofs + j]) +
                                     __builtin_popcount(lds[e.x + row2 + 2 * KA + j] & 0xFFFFu);
                ws += cnt << j;
            }
            wsum_tab[tid] = ws;
        }
    }

    // ---- this lane's weights (five words per plane) and affine parameters
    const int kc = c < sh.K ? c : sh.K - 1;
    uint32_t wq[kPairWords][KW];
#pragma unroll
    for (int t5 = 0; t5 < kPairWords; ++t5)
#pragma unroll
        for (int i = 0; i < KW; ++i) wq[t5][i] = wpair[(kc * kPairWords + t5) * KW + i];
    const int ci = sh.per_channel ? kc : 0;
    const float sc = scale[ci];
    const float of = offset ? offset[ci] : 0.0f;
    __syncthreads();

    const int p_wave = wave * TPW + g;            // this lane's position of step 0 inside the tile

    struct Pos { int t; uint32_t li, next, wsum; };
    auto locate = [&](int step) {
        const int p = p_wave + step * G;
        const uint2 e = tab[p];
        Pos r;
        r.t = t_first + p;
        r.li = e.x;
        r.next = e.y;
        r.wsum = SGN ? wsum_tab[p] : 0u;
        return r;
    };
    auto load_x = [&](uint32_t li, uint32_t (&x)[kPairWords][KA]) {
#pragma unroll
        for (int j = 0; j < KA; ++j) {
            x[0][j] = lds[li + j];
            x[1][j] = lds[li + row1 + j];
            x[2][j] = lds[li + row2 + j];
            x[3][j] = lds[li + vofs + j];
            x[4][j] = lds[li + row2 + 2 * KA + j];
        }
    };
    // Eq. 2 / Eq. 13 on the five words, one accumulator per shift class i + j (each class is first written
    // at word 0 with its smallest i), then Eq. 14
    auto product = [&](const uint32_t (&x)[kPairWords][KA]) {
        uint32_t cls[NCLS];
#pragma unroll
        for (int t5 = 0; t5 < kPairWords; ++t5)
#pragma unroll
            for (int i = 0; i < KW; ++i)
#pragma unroll
                for (int j = 0; j < KA; ++j) {
                    const uint32_t v = wq[t5][i] & x[t5][j];
                    if (t5 == 0 && (i == 0 || j == KA - 1)) cls[i + j] = pair_bcnt_first(v);
                    else cls[i + j] = pair_bcnt_acc(v, cls[i + j]);
                }
        uint32_t v = cls[0];
#pragma unroll
        for (int s = 1; s < NCLS; ++s) v += cls[s] << s;
        return (int32_t)v;
    };
    auto emit = [&](const Pos &p, int32_t acc) {
        if constexpr (SGN) acc = 2 * acc - sh.wtop * (int32_t)p.wsum;
        if constexpr (REQ) {
            const uint32_t lv = c < sh.K ? requant_level(acc, sc, of, sh.alpha, sh.qs) : 0u;
            uint32_t *dst = packed_next + (size_t)p.next * sh.k_next;
#pragma unroll
            for (int j = 0; j < kMaxBits; ++j) {
                if (j < sh.k_next) {
                    const unsigned long long m = __ballot((lv >> j) & 1u);
                    const uint32_t word = KP == 32 ? (uint32_t)(m >> (32 * g)) : ((uint32_t)(m >> (16 * g)) & 0xFFFFu);
                    if (c == 0 && p.t < sh.total) dst[j] = word;
                }
            }
        } else {
            if (p.t < sh.total && c < sh.K) {
                const size_t o = (size_t)p.t * sh.K + c;
                acc_out[o] = acc;
                if (out_f32) out_f32[o] = fmaf((float)acc, sc, of);
            }
        }
    };

    // two steps per trip; the next step's words are read from LDS before the current ones are multiplied
    uint32_t xa[kPairWords][KA], xb[kPairWords][KA];
    Pos pa = locate(0), pb;
    load_x(pa.li, xa);
    for (int step = 0; step < STEPS; step += 2) {
        pb = locate(step + 1);
        load_x(pb.li, xb);
        emit(pa, product(xa));
        pa = locate(step + 2 < STEPS ? step + 2 : step + 1);
        load_x(pa.li, xa);
        emit(pb, product(xb));
    }

    if constexpr (REQ) {
        // zero ring of the next layer's tensor, dealt evenly to the work-groups: top row, bottom row,
        // then the left/right columns of every image (one word per position)
        const int kmax = sh.k_next;
        for (int idx = blockIdx.x * 256 + tid; idx < sh.ring_total; idx += sh.nblocks * 256) {
            const int n = idx / sh.ring_per_image;
            const int rem = idx - n * sh.ring_per_image;
            const int b = rem / kmax;
            const int j = rem - b * kmax;
            int hp, wp;
            if (b < sh.OWn) { hp = 0; wp = b; }
            else if (b < 2 * sh.OWn) { hp = sh.OHn - 1; wp = b - sh.OWn; }
            else { const int cc = b - 2 * sh.OWn; hp = 1 + (cc >> 1); wp = (cc & 1) ? sh.OWn - 1 : 0; }
            packed_next[(((size_t)n * sh.OHn + hp) * sh.OWn + wp) * kmax + j] = 0u;
        }
    }
}

// Dwords of the ordinary section of the packed weights of a C <= 32 layer (the pair section follows it).
inline size_t pair_section_offset(int K, int RS, int kw)
{
    return (size_t)((K + kWgtGroup - 1) / kWgtGroup) * kWgtGroup * RS * kw;
}

template <int KW, int KA, int KP, bool REQ, int TP, bool SGN>
static int launch_pair_cfg(const ConvArgs &a)
{
    constexpr int kPairTile = TP;
    PairShape sh{};
    sh.K = a.K; sh.OH = a.OH; sh.OW = a.OW;
    sh.Hp = a.H + 2 * kActBorder; sh.Wp = a.W + 2 * kActBorder;
    sh.stride = a.stride; sh.origin = kActBorder - a.pad;
    sh.total = a.N * a.OH * a.OW;
    sh.total_pos = a.N * sh.Hp * sh.Wp;
    sh.per_channel = a.per_channel;
    sh.wtop = a.wtop;
    sh.div_ow = make_fastdiv((uint32_t)a.OW);
    sh.div_ohow = make_fastdiv((uint32_t)(a.OH * a.OW));
    TileGeom geo{a.H, a.W, 3, 3, a.stride, a.pad, a.OH, a.OW, kActBorder};
    const long long tp = kPairTile < sh.total ? kPairTile : sh.total;
    const long long ucap = geo.extent_bound(tp);
    const size_t lds_bytes = ((size_t)ucap * 2 * KA + 3 * kPairTile) * sizeof(uint32_t);
    if (lds_bytes > 64 * 1024) return EBS_ERR_UNSUPPORTED;
    sh.ucap = (int)ucap;
    sh.nblocks = (sh.total + kPairTile - 1) / kPairTile;
    if (REQ) {
        sh.alpha = a.alpha;
        sh.k_next = a.k_next;
        sh.qs = requant_qs(a.alpha, a.k_next);
        sh.OHn = a.OH + 2 * kActBorder;
        sh.OWn = a.OW + 2 * kActBorder;
        sh.total_next = a.N * sh.OHn * sh.OWn;
        const long long per_image = (2LL * sh.OWn + 2LL * a.OH) * a.k_next;
        if (per_image * a.N > (1LL << 30)) return EBS_ERR_UNSUPPORTED;
        sh.ring_per_image = (int)per_image;
        sh.ring_total = (int)(per_image * a.N);
    }
    const DeviceShape *dev = device_shape();
    if (!dev) return EBS_ERR_HIP;
    if (!dev->gfx950) return EBS_ERR_UNSUPPORTED;       // tile and LDS budget are gfx950's
    const uint32_t *wpair = a.wgt + pair_section_offset(a.K, 9, KW);
    hipLaunchKernelGGL((bd_conv_pair<KW, KA, KP, REQ, TP, SGN>), dim3((unsigned)sh.nblocks), dim3(256), lds_bytes, a.stream,
                       a.act, wpair, a.scale, a.offset, a.acc, a.out, a.next, sh);
    return hip_ok(hipGetLastError());
}

// Whether the pair kernel can run the request at all (shape part; bitwidths are the instantiated pairs).
inline bool pair_shape_ok(const ConvArgs &a)
{
    return a.C <= 16 && a.R == 3 && a.S == 3 && a.pad <= kActBorder && a.stride >= 1 && a.stride <= 2 && a.K <= 32 &&
           (long long)a.N * a.OH * a.OW < (1LL << 30);
}

// Tiles of 128 positions where that still gives every compute unit several work-groups, else 32 (16->32
// stride 2 on 32x32 images, batch 128: 8.8 -> 7.1 us; the large layers take the same time with either).
template <int KW, int KA, int KP, bool REQ, bool SGN>
static int launch_pair_tile(const ConvArgs &a)
{
    const long long total = (long long)a.N * a.OH * a.OW;
    if (total >= 128 * 1024) return launch_pair_cfg<KW, KA, KP, REQ, 128, SGN>(a);
    return launch_pair_cfg<KW, KA, KP, REQ, 32, SGN>(a);
}

template <int KW, int KA, int KP, bool REQ>
static int launch_pair_sign(const ConvArgs &a)
{
    if (a.wtop) return launch_pair_tile<KW, KA, KP, REQ, true>(a);
    return launch_pair_tile<KW, KA, KP, REQ, false>(a);
}

template <int KW, int KA>
static int launch_pair_impl(const ConvArgs &a)
{
    if (!pair_shape_ok(a)) return EBS_ERR_UNSUPPORTED;
    if (a.next) {
        if (a.K <= 16) return launch_pair_sign<KW, KA, 16, true>(a);
        return launch_pair_sign<KW, KA, 32, true>(a);
    }
    if (a.K <= 16) return launch_pair_sign<KW, KA, 16, false>(a);
    return launch_pair_sign<KW, KA, 32, false>(a);
}

template <int KW, int KA> int launch_pair_pair(const ConvArgs &a);

#define EBS_DEFINE_PAIR_PAIR(KWV, KAV)                                  \
    template <> int launch_pair_pair<KWV, KAV>(const ConvArgs &a)      \
    {                                                                   \
        return launch_pair_impl<KWV, KAV>(a);                           \
    }

}  // namespace ebs
