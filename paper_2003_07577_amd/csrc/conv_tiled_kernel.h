// Tiled AND + bitcount convolution with fused shift-accumulate and scale/offset
// epilogue (paper Sec. 3 Eq. 2; Sec. 4.3 Eq. 13-14, both stages in one kernel:
// the bit-plane partial products P live in registers only).
//
// Mapping (CDNA4, 64-wide waves):
//  * a lane owns PIX output positions, a wave a tile of 64*PIX positions x KT
//    output channels.  Output positions are numbered t = (n*OH+oh)*OW+ow, so a
//    tile is any run of consecutive positions and may cross rows and images.
//  * weight words are wave-uniform: they are fetched with scalar loads and used
//    as the scalar operand of v_and_b32; activations are per-lane vector
//    operands.  The inner body per (word, plane pair) is exactly v_and_b32 +
//    accumulating v_bcnt_u32_b32; one accumulator per shift class i+j, so the
//    2^(i+j) recombination is paid once per output in the epilogue.
//  * the packed activations a work-group needs are staged in LDS as one
//    contiguous run of the flat zero-padded input (see tile_geometry.h): image
//    borders are resolved once at staging time and every filter tap becomes a
//    wave-uniform LDS offset r*Wp + s.
//  * SPLIT = 4 lets the four waves of a work-group share one position tile and
//    split the reduction words among them (for layers with few output
//    positions and a long reduction); partial sums meet in LDS.
#pragma once
#include "ebs_internal.h"
#include "tile_geometry.h"

namespace ebs {

struct TiledShape {
    int N, H, W, K, R, S, stride, pad, OH, OW, cw, Hp, Wp, RS;
    int total;        // N*OH*OW output positions
    int nchunks;      // ceil(cw / CH) reduction chunks staged one at a time
    int ktiles;       // ceil(K / KT)
    int kiters;       // channel tiles handled by one work-group (blockIdx.y selects the group)
    int per_channel;
    int ucap;         // staged positions that fit the LDS allocation
    int wgroups;      // 16-channel groups present in the packed weights
};

template <int N> struct UVec;
template <> struct UVec<1> { typedef uint32_t type; };
template <> struct UVec<2> { typedef uint32_t type __attribute__((ext_vector_type(2))); };
template <> struct UVec<4> { typedef uint32_t type __attribute__((ext_vector_type(4))); };

template <int KW, int KA, int PIX, int KT, int CH, int SPLIT>
struct Cfg {
    static constexpr int NCLS = KW + KA - 1;
    static constexpr int KAP = (KA == 3) ? 4 : KA;   // planes per staged word, padded to a power of two
    static constexpr int WAVES = 4;
    static constexpr int WPX = WAVES / SPLIT;        // waves along the position axis
    static constexpr int TPW = 64 * PIX;             // positions per wave
    static constexpr int TP = WPX * TPW;             // positions per work-group
    static constexpr int POSW = CH * KAP;            // LDS dwords per staged position
    static constexpr int WSTEP = CH / SPLIT;         // reduction words per wave per tap per chunk
    static constexpr int KG = (KT + kWgtGroup - 1) / kWgtGroup;   // 16-channel weight groups per tile
    static constexpr int KTG = KT < kWgtGroup ? KT : kWgtGroup;   // channels taken from one group
    static_assert(CH % SPLIT == 0, "chunk must divide among the waves");
    static_assert(KT % 4 == 0 && (KT <= 16 ? 16 % KT == 0 : KT % 16 == 0), "channel tile vs weight group");
};

template <int KW, int KA, int PIX, int KT, int CH, int SPLIT>
__global__ void __launch_bounds__(256)
bd_conv_tiled(const uint32_t *__restrict__ act, const uint32_t *__restrict__ wgt,
              const float *__restrict__ scale, const float *__restrict__ offset,
              int32_t *__restrict__ acc_out, float *__restrict__ out_f32, const TiledShape sh)
{
    using C = Cfg<KW, KA, PIX, KT, CH, SPLIT>;
    extern __shared__ __attribute__((aligned(16))) uint32_t lds[];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wpx = SPLIT == 1 ? wave : 0;        // which position sub-tile this wave owns
    const int wred = SPLIT == 1 ? 0 : wave;       // which share of the reduction words

    // ---- tile of output positions and the flat padded-input range it reads
    const int t_first = blockIdx.x * C::TP;
    int t_last = t_first + C::TP - 1;
    if (t_last > sh.total - 1) t_last = sh.total - 1;
    const int ohow = sh.OH * sh.OW;
    auto base_of = [&](int t) {
        int n = t / ohow;
        int rem = t - n * ohow;
        int oh = rem / sh.OW;
        int ow = rem - oh * sh.OW;
        return (n * sh.Hp + oh * sh.stride) * sh.Wp + ow * sh.stride;
    };
    const int u_lo = base_of(t_first);
    int u_hi = base_of(t_last) + (sh.R - 1) * sh.Wp + (sh.S - 1);
    if (u_hi > u_lo + sh.ucap - 1) u_hi = u_lo + sh.ucap - 1;   // never beyond the LDS allocation

    int my_t[PIX];
    int my_lds[PIX];          // LDS dword index of the lane's positions (tap 0, word 0)
#pragma unroll
    for (int p = 0; p < PIX; ++p) {
        int t = t_first + wpx * C::TPW + p * 64 + lane;
        my_t[p] = t;
        int tc = t < sh.total ? t : sh.total - 1;
        my_lds[p] = (base_of(tc) - u_lo) * C::POSW;
    }

    // ---- staging of one reduction chunk: rows of the flat padded input
    const int row_lo = u_lo / sh.Wp;
    const int row_hi = u_hi / sh.Wp;
    auto stage = [&](int chunk) {
        const int w0 = chunk * CH;
        for (int row = row_lo + wave; row <= row_hi; row += C::WAVES) {
            const int n = row / sh.Hp;
            const int h = row - n * sh.Hp - sh.pad;
            const bool row_ok = (h >= 0) && (h < sh.H) && (n < sh.N);
            const int src_row = (n * sh.H + h) * sh.W;
            for (int x = lane; x < sh.Wp * CH; x += 64) {
                const int wp = x / CH;
                const int w = x - wp * CH;
                const int u = row * sh.Wp + wp;
                if (u < u_lo || u > u_hi) continue;
                const int col = wp - sh.pad;
                const bool ok = row_ok && (col >= 0) && (col < sh.W) && (w0 + w < sh.cw);
                uint32_t v[C::KAP];
#pragma unroll
                for (int j = 0; j < C::KAP; ++j) v[j] = 0u;
                if (ok) {
                    const uint32_t *src = act + ((size_t)(src_row + col) * sh.cw + (w0 + w)) * KA;
#pragma unroll
                    for (int j = 0; j < KA; ++j) v[j] = src[j];
                }
                typedef typename UVec<C::KAP>::type vec_t;
                vec_t vv;
                if constexpr (C::KAP == 1) {
                    vv = v[0];
                } else {
#pragma unroll
                    for (int j = 0; j < C::KAP; ++j) vv[j] = v[j];
                }
                *reinterpret_cast<vec_t *>(lds + (size_t)(u - u_lo) * C::POSW + w * C::KAP) = vv;
            }
        }
    };

    const int kt_begin = blockIdx.y * sh.kiters;
    int kt_end = kt_begin + sh.kiters;
    if (kt_end > sh.ktiles) kt_end = sh.ktiles;

    if (sh.nchunks == 1) {
        stage(0);
        __syncthreads();
    }

    for (int kt = kt_begin; kt < kt_end; ++kt) {
        const int k0 = kt * KT;
        uint32_t cls[PIX][KT][C::NCLS];
#pragma unroll
        for (int p = 0; p < PIX; ++p)
#pragma unroll
            for (int c = 0; c < KT; ++c)
#pragma unroll
                for (int s = 0; s < C::NCLS; ++s) cls[p][c][s] = 0u;

        for (int chunk = 0; chunk < sh.nchunks; ++chunk) {
            if (sh.nchunks > 1) {
                __syncthreads();      // everyone is done with the previous chunk
                stage(chunk);
                __syncthreads();
            }
            // weight words of this tile: [k/16][tap][word][k%16][plane]
            const int g0 = k0 / kWgtGroup;
            const uint32_t *wchunk = wgt + (size_t)chunk * CH * (kWgtGroup * KW) + (k0 % kWgtGroup) * KW;
            int tap_off = 0;          // (r*Wp + s) * POSW, maintained incrementally
            int s_col = 0;
            for (int tap = 0; tap < sh.RS; ++tap) {
#pragma unroll
                for (int ws = 0; ws < C::WSTEP; ++ws) {
                    const int w = ws * SPLIT + wred;        // word inside the chunk
                    if (chunk * CH + w < sh.cw) {
                        // ---- scalar (wave-uniform) weight words q[channel][plane]
                        uint32_t q[KT][KW];
#pragma unroll
                        for (int g = 0; g < C::KG; ++g) {
                            // a tile may reach past the last packed group (its channels are never stored): re-read the last one
                            const int gi = g0 + g < sh.wgroups ? g0 + g : sh.wgroups - 1;
                            const uint32_t *wp = wchunk + (((size_t)gi * sh.RS + tap) * sh.cw + w) * (kWgtGroup * KW);
#pragma unroll
                            for (int c = 0; c < C::KTG; ++c)
#pragma unroll
                                for (int i = 0; i < KW; ++i) q[g * kWgtGroup + c][i] = wp[c * KW + i];
                        }
                        // ---- per-lane activation words x[position][plane] from LDS
                        uint32_t x[PIX][KA];
#pragma unroll
                        for (int p = 0; p < PIX; ++p) {
                            typedef typename UVec<C::KAP>::type vec_t;
                            const vec_t v = *reinterpret_cast<const vec_t *>(lds + my_lds[p] + tap_off + w * C::KAP);
                            if constexpr (C::KAP == 1) {
                                x[p][0] = v;
                            } else {
#pragma unroll
                                for (int j = 0; j < KA; ++j) x[p][j] = v[j];
                            }
                        }
                        // ---- Eq. 2 / Eq. 13: AND + accumulating bitcount per plane pair
#pragma unroll
                        for (int p = 0; p < PIX; ++p)
#pragma unroll
                            for (int c = 0; c < KT; ++c)
#pragma unroll
                                for (int i = 0; i < KW; ++i)
#pragma unroll
                                    for (int j = 0; j < KA; ++j)
                                        cls[p][c][i + j] += __builtin_popcount(q[c][i] & x[p][j]);
                    }
                }
                // next tap
                ++s_col;
                tap_off += C::POSW;
                if (s_col == sh.S) {
                    s_col = 0;
                    tap_off += (sh.Wp - sh.S) * C::POSW;
                }
            }
        }

        // ---- Eq. 14: recombine the shift classes, then the affine epilogue
        int32_t acc[PIX][KT];
#pragma unroll
        for (int p = 0; p < PIX; ++p)
#pragma unroll
            for (int c = 0; c < KT; ++c) {
                uint32_t v = 0;
#pragma unroll
                for (int s = 0; s < C::NCLS; ++s) v += cls[p][c][s] << s;
                acc[p][c] = (int32_t)v;
            }

        if constexpr (SPLIT > 1) {
            // partial sums of the four waves meet in LDS (after the staged data is dead)
            __syncthreads();
            int32_t *red = reinterpret_cast<int32_t *>(lds);     // [PIX][KT][64]
            if (wave == 0) {
#pragma unroll
                for (int p = 0; p < PIX; ++p)
#pragma unroll
                    for (int c = 0; c < KT; ++c) red[(p * KT + c) * 64 + lane] = acc[p][c];
            }
            __syncthreads();
            if (wave != 0) {
#pragma unroll
                for (int p = 0; p < PIX; ++p)
#pragma unroll
                    for (int c = 0; c < KT; ++c) atomicAdd(&red[(p * KT + c) * 64 + lane], acc[p][c]);
            }
            __syncthreads();
            // wave w finishes channels [w*KT/4, (w+1)*KT/4)
            constexpr int KQ = KT / SPLIT;
#pragma unroll
            for (int p = 0; p < PIX; ++p) {
                if (my_t[p] < sh.total) {
#pragma unroll
                    for (int cc = 0; cc < KQ; ++cc) {
                        const int c = wave * KQ + cc;
                        const int k = k0 + c;
                        if (k < sh.K) {
                            const int32_t v = red[(p * KT + c) * 64 + lane];
                            const size_t o = (size_t)my_t[p] * sh.K + k;
                            acc_out[o] = v;
                            if (out_f32) {
                                const int ci = sh.per_channel ? k : 0;
                                const float of = offset ? offset[ci] : 0.0f;
                                out_f32[o] = fmaf((float)v, scale[ci], of);
                            }
                        }
                    }
                }
            }
            if (sh.nchunks == 1 && kt + 1 < kt_end) {   // the staged data was overwritten by the reduction
                __syncthreads();
                stage(0);
                __syncthreads();
            }
        } else {
            const bool full = (k0 + KT <= sh.K) && ((sh.K & 3) == 0);
            float sc[KT], of[KT];
            if (out_f32) {
#pragma unroll
                for (int c = 0; c < KT; ++c) {
                    const int k = k0 + c < sh.K ? k0 + c : sh.K - 1;
                    const int ci = sh.per_channel ? k : 0;
                    sc[c] = scale[ci];
                    of[c] = offset ? offset[ci] : 0.0f;
                }
            }
#pragma unroll
            for (int p = 0; p < PIX; ++p) {
                if (my_t[p] >= sh.total) continue;
                const size_t o = (size_t)my_t[p] * sh.K + k0;
                if (full) {
                    typedef int32_t i4 __attribute__((ext_vector_type(4)));
                    typedef float f4 __attribute__((ext_vector_type(4)));
#pragma unroll
                    for (int c = 0; c < KT; c += 4) {
                        i4 v = {acc[p][c], acc[p][c + 1], acc[p][c + 2], acc[p][c + 3]};
                        *reinterpret_cast<i4 *>(acc_out + o + c) = v;
                    }
                    if (out_f32) {
#pragma unroll
                        for (int c = 0; c < KT; c += 4) {
                            f4 v = {fmaf((float)acc[p][c], sc[c], of[c]), fmaf((float)acc[p][c + 1], sc[c + 1], of[c + 1]),
                                    fmaf((float)acc[p][c + 2], sc[c + 2], of[c + 2]), fmaf((float)acc[p][c + 3], sc[c + 3], of[c + 3])};
                            *reinterpret_cast<f4 *>(out_f32 + o + c) = v;
                        }
                    }
                } else {
#pragma unroll
                    for (int c = 0; c < KT; ++c) {
                        if (k0 + c < sh.K) {
                            acc_out[o + c] = acc[p][c];
                            if (out_f32) out_f32[o + c] = fmaf((float)acc[p][c], sc[c], of[c]);
                        }
                    }
                }
            }
        }
    }
}

// (PIX, KT) per accumulator budget and number of shift classes.
template <int BUDGET, int NCLS> struct TileOf;
#define EBS_TILE(b, n, p, k) template <> struct TileOf<b, n> { static constexpr int PIX = p, KT = k; };
EBS_TILE(128, 1, 4, 32) EBS_TILE(128, 2, 4, 16) EBS_TILE(128, 3, 4, 8) EBS_TILE(128, 4, 4, 8)
EBS_TILE(128, 5, 4, 4)  EBS_TILE(128, 6, 4, 4)  EBS_TILE(128, 7, 4, 4)
EBS_TILE(64, 1, 4, 16)  EBS_TILE(64, 2, 4, 8)   EBS_TILE(64, 3, 2, 8)  EBS_TILE(64, 4, 2, 8)
EBS_TILE(64, 5, 2, 4)   EBS_TILE(64, 6, 2, 4)   EBS_TILE(64, 7, 2, 4)
EBS_TILE(32, 1, 2, 16)  EBS_TILE(32, 2, 2, 8)   EBS_TILE(32, 3, 1, 8)  EBS_TILE(32, 4, 1, 8)
EBS_TILE(32, 5, 1, 4)   EBS_TILE(32, 6, 1, 4)   EBS_TILE(32, 7, 1, 4)
#undef EBS_TILE

static constexpr size_t kMaxLdsBytes = 64 * 1024;

template <int KW, int KA, int BUDGET, int CH, int SPLIT>
static int launch_cfg(const ConvArgs &a)
{
    constexpr int PIX = TileOf<BUDGET, KW + KA - 1>::PIX;
    constexpr int KT = TileOf<BUDGET, KW + KA - 1>::KT;
    using C = Cfg<KW, KA, PIX, KT, CH, SPLIT>;
    TiledShape sh{};
    sh.N = a.N; sh.H = a.H; sh.W = a.W; sh.K = a.K; sh.R = a.R; sh.S = a.S;
    sh.stride = a.stride; sh.pad = a.pad; sh.OH = a.OH; sh.OW = a.OW; sh.cw = a.cw;
    sh.Hp = a.H + 2 * a.pad; sh.Wp = a.W + 2 * a.pad; sh.RS = a.R * a.S;
    sh.total = a.N * a.OH * a.OW;
    sh.nchunks = (a.cw + CH - 1) / CH;
    sh.ktiles = (a.K + KT - 1) / KT;
    sh.per_channel = a.per_channel;
    sh.wgroups = (a.K + kWgtGroup - 1) / kWgtGroup;

    TileGeom g{a.H, a.W, a.R, a.S, a.stride, a.pad, a.OH, a.OW};
    long long tp = C::TP < sh.total ? C::TP : sh.total;
    long long ucap = g.extent_bound(tp);
    size_t lds_bytes = (size_t)ucap * C::POSW * sizeof(uint32_t);
    if (SPLIT > 1) {
        size_t red = (size_t)PIX * KT * 64 * sizeof(int32_t);
        if (red > lds_bytes) lds_bytes = red;
    }
    if (lds_bytes > kMaxLdsBytes || ucap > (1 << 30)) return EBS_ERR_UNSUPPORTED;
    sh.ucap = (int)ucap;

    long long ptiles = ((long long)sh.total + C::TP - 1) / C::TP;
    // Channel tiles per work-group: when the whole reduction is staged once, let a
    // work-group reuse it for several channel tiles, but keep >= ~4 waves per SIMD.
    int kiters = 1;
    if (sh.nchunks == 1 && SPLIT == 1) {
        while (kiters * 2 <= sh.ktiles && ptiles * ((sh.ktiles + kiters * 2 - 1) / (kiters * 2)) >= 2048) kiters *= 2;
    }
    sh.kiters = kiters;
    long long kgroups = (sh.ktiles + kiters - 1) / kiters;
    if (ptiles > 0x7fffffffLL || kgroups > 65535) return EBS_ERR_UNSUPPORTED;

    hipLaunchKernelGGL((bd_conv_tiled<KW, KA, PIX, KT, CH, SPLIT>), dim3((unsigned)ptiles, (unsigned)kgroups), dim3(256),
                       lds_bytes, a.stream, a.act, a.wgt, a.scale, a.offset, a.acc, a.out, sh);
    return hip_ok(hipGetLastError());
}


// Variant table: (accumulator budget, words per staged chunk, reduction split).
struct TiledVariant { const char *name; int budget, ch, split; };
#define EBS_TILED_VARIANTS(X) \
    X(0, 128, 2, 1) X(1, 128, 1, 1) X(2, 128, 4, 1) \
    X(3, 64, 2, 1)  X(4, 64, 1, 1)  X(5, 64, 4, 1)  \
    X(6, 32, 2, 1)  X(7, 32, 1, 1)  X(8, 32, 4, 1)  \
    X(9, 64, 4, 4)  X(10, 32, 4, 4)
constexpr int kNumTiledVariants = 11;

template <int KW, int KA>
static int launch_bits(const ConvArgs &a, int v)
{
    switch (v) {
#define EBS_X(idx, b, ch, sp) case idx: return launch_cfg<KW, KA, b, ch, sp>(a);
        EBS_TILED_VARIANTS(EBS_X)
#undef EBS_X
    }
    return EBS_ERR_UNSUPPORTED;
}

// One translation unit per weight bitwidth instantiates these.
template <int KW> int launch_tiled_kw(const ConvArgs &a, int v);

#define EBS_DEFINE_TILED_KW(KWV)                                            \
    template <> int launch_tiled_kw<KWV>(const ConvArgs &a, int v)          \
    {                                                                       \
        switch (a.ka) {                                                     \
            case 1: return launch_bits<KWV, 1>(a, v);                       \
            case 2: return launch_bits<KWV, 2>(a, v);                       \
            case 3: return launch_bits<KWV, 3>(a, v);                       \
            case 4: return launch_bits<KWV, 4>(a, v);                       \
        }                                                                   \
        return EBS_ERR_BITWIDTH;                                            \
    }

}  // namespace ebs
