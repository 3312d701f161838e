// Tiled AND + bitcount convolution with fused shift-accumulate and scale/offset
// epilogue (paper Sec. 3 Eq. 2; Sec. 4.3 Eq. 13-14, both stages in one kernel:
// the bit-plane partial products P live in registers only).
//
// Mapping (CDNA4, 64-wide waves, 4 waves per work-group):
//  * a lane owns PIX output positions, a wave a tile of 64*PIX positions x KT
//    output channels.  Output positions are numbered t = (n*OH+oh)*OW+ow, so a
//    tile is any run of consecutive positions and may cross rows and images.
//  * weight words are wave-uniform: they are fetched with scalar loads and used
//    as the scalar operand of v_and_b32; activations are per-lane vector
//    operands.  The inner body per (word, plane pair) is exactly v_and_b32 +
//    accumulating v_bcnt_u32_b32; one accumulator per shift class i+j, so the
//    2^(i+j) recombination is paid once per output in the epilogue.  Operands
//    of the next reduction step are requested before the current step's
//    arithmetic starts.
//  * the packed activations a work-group needs are staged in LDS as one
//    contiguous run of the flat zero-bordered input (see tile_geometry.h): the
//    staging is a plain copy, image borders need no test and every filter tap
//    is a wave-uniform LDS offset r*Wp + s.  Needs pad <= the stored border.
//    LDS layout is [word][position][plane], so the lanes of a wave (consecutive
//    positions) read consecutive addresses whatever the chunk size.
//  * the four waves of a work-group either take four position sub-tiles of one
//    channel tile (MODE_P4), four channel tiles of one position tile (MODE_K4:
//    the staged activations serve 4*KT channels and the output rows a
//    work-group writes are 4*KT channels wide), or four shares of the reduction
//    words of one tile (MODE_R4, for layers with few outputs and a long
//    reduction; the partial sums meet in LDS).
//  * the epilogue goes through LDS: accumulators are laid out [position][channel]
//    and written back by all 256 threads as 16-byte pieces of consecutive
//    addresses, so global stores cover whole runs of each NHWC output row.
#pragma once
#include "ebs_internal.h"
#include "tile_geometry.h"
#include <cstdlib>

namespace ebs {

enum { MODE_P4 = 0, MODE_K4 = 1, MODE_R4 = 2 };

// Experiment builds (-DEBS_EXPERIMENT) can switch phases of the kernel off through the
// EBS_EXP_DBG environment variable to time them; production builds compile this away.
#ifdef EBS_EXPERIMENT
#define EBS_DBG(bit) (sh.dbg & (bit))
#else
#define EBS_DBG(bit) false
#endif

struct TiledShape {
    int N, H, W, K, R, S, stride, pad, OH, OW, cw, Hp, Wp, RS;   // Hp, Wp: bordered grid
    int total;        // N*OH*OW output positions
    int nchunks;      // ceil(cw / CH) reduction chunks staged one at a time
    int per_channel;
    int ucap;         // staged positions that fit the LDS allocation
    int wgroups;      // 16-channel groups present in the packed weights
    int stage_dwords; // LDS dwords reserved for staged activations (the output tile follows)
    int dbg;          // experiment switches; only read in EBS_EXPERIMENT builds
};

template <int N> struct UVec;
template <> struct UVec<1> { typedef uint32_t type; };
template <> struct UVec<2> { typedef uint32_t type __attribute__((ext_vector_type(2))); };
template <> struct UVec<4> { typedef uint32_t type __attribute__((ext_vector_type(4))); };

// acc + bitcount(x) in ONE instruction: v_bcnt_u32_b32 adds its second operand.  Spelled
// out because the optimiser otherwise regroups sums of bitcounts into separate
// count and three-operand-add instructions, which costs an extra VALU slot per pair.
__device__ __forceinline__ uint32_t bcnt_acc(uint32_t x, uint32_t acc)
{
    uint32_t d;
    asm("v_bcnt_u32_b32 %0, %1, %2" : "=v"(d) : "v"(x), "v"(acc));
    return d;
}

typedef int32_t i32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

template <int KW, int KA, int PIX, int KT, int CH, int MODE>
struct Cfg {
    static constexpr int NCLS = KW + KA - 1;
    static constexpr int KAP = (KA == 3) ? 4 : KA;   // planes per staged word, padded to a power of two
    static constexpr int WAVES = 4;
    static constexpr int WPX = MODE == MODE_P4 ? 4 : 1;          // waves along the position axis
    static constexpr int WK = MODE == MODE_K4 ? 4 : 1;           // waves along the channel axis
    static constexpr int WRED = MODE == MODE_R4 ? 4 : 1;         // waves sharing one reduction
    static constexpr int TPW = 64 * PIX;             // positions per wave
    static constexpr int TP = WPX * TPW;             // positions per work-group
    static constexpr int KB = WK * KT;               // channels per work-group
    static constexpr int POSW = CH * KAP;            // LDS dwords per staged position (all words of the chunk)
    static constexpr int WSTEP = CH / WRED;          // reduction words per wave per tap per chunk
    static constexpr int KG = (KT + kWgtGroup - 1) / kWgtGroup;   // 16-channel weight groups per tile
    static constexpr int KTG = KT < kWgtGroup ? KT : kWgtGroup;   // channels taken from one group
    // output tile of one epilogue pass, [row = position][col = channel], padded pitch
    static constexpr int OROWS = WPX * 64;
    static constexpr int OCOLS = KB;
    static constexpr int OPITCH = OCOLS + 4;
    static constexpr int OUT_DWORDS = OROWS * OPITCH;
    static_assert(CH % WRED == 0, "chunk must divide among the waves");
    static_assert(KT % 4 == 0 && (KT <= 16 ? 16 % KT == 0 : KT % 16 == 0), "channel tile vs weight group");
    static_assert(256 % (OCOLS / 4) == 0, "write-back assumes a fixed column group per thread");
};

template <int KW, int KA, int PIX, int KT, int CH, int MODE>
__global__ void __launch_bounds__(256)
bd_conv_tiled(const uint32_t *__restrict__ act, const uint32_t *__restrict__ wgt,
              const float *__restrict__ scale, const float *__restrict__ offset,
              int32_t *__restrict__ acc_out, float *__restrict__ out_f32, const TiledShape sh)
{
    using C = Cfg<KW, KA, PIX, KT, CH, MODE>;
    extern __shared__ __attribute__((aligned(16))) uint32_t lds[];
    int32_t *otile = reinterpret_cast<int32_t *>(lds + sh.stage_dwords);

#ifdef EBS_EXPERIMENT
    const unsigned long long exp_t0 = wall_clock64();
#endif
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wpx = MODE == MODE_P4 ? wave : 0;     // position sub-tile of this wave
    const int wk = MODE == MODE_K4 ? wave : 0;      // channel sub-tile of this wave
    const int wred = MODE == MODE_R4 ? wave : 0;    // share of the reduction words

    // ---- tile of output positions and the flat bordered-input range it reads
    const int t_first = blockIdx.x * C::TP;
    int t_last = t_first + C::TP - 1;
    if (t_last > sh.total - 1) t_last = sh.total - 1;
    const int ohow = sh.OH * sh.OW;
    auto base_of = [&](int t) {
        int n = t / ohow;
        int rem = t - n * ohow;
        int oh = rem / sh.OW;
        int ow = rem - oh * sh.OW;
        return (n * sh.Hp + oh * sh.stride + kActBorder - sh.pad) * sh.Wp + ow * sh.stride + kActBorder - sh.pad;
    };
    const int u_lo = base_of(t_first);
    int u_hi = base_of(t_last) + (sh.R - 1) * sh.Wp + (sh.S - 1);
    if (u_hi > u_lo + sh.ucap - 1) u_hi = u_lo + sh.ucap - 1;   // never beyond the LDS allocation

    int my_lds[PIX];          // LDS dword index of the lane's positions (tap 0, word 0)
#pragma unroll
    for (int p = 0; p < PIX; ++p) {
        int t = t_first + wpx * C::TPW + p * 64 + lane;
        int tc = t < sh.total ? t : sh.total - 1;
        my_lds[p] = (base_of(tc) - u_lo) * C::KAP;
    }

    // ---- staging of one reduction chunk: positions [u_lo, u_hi] of the bordered
    //      input are contiguous in memory; copy CH words (x KA planes) of each
    const int n_stage = (u_hi - u_lo + 1) * CH;
    auto stage = [&](int chunk) {
        const int w0 = chunk * CH;
        for (int x = tid; x < n_stage; x += 256) {
            const int u = x / CH;
            const int w = x - u * CH;
            uint32_t v[C::KAP];
#pragma unroll
            for (int j = 0; j < C::KAP; ++j) v[j] = 0u;
            if (w0 + w < sh.cw) {
                const uint32_t *src = act + ((size_t)(u_lo + u) * sh.cw + (w0 + w)) * KA;
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
            *reinterpret_cast<vec_t *>(lds + (size_t)(w * sh.ucap + u) * C::KAP) = vv;
        }
    };

    const int kb0 = blockIdx.y * C::KB;       // first channel of the work-group
    const int k0 = kb0 + wk * KT;             // first channel of this wave
    const int g0 = k0 / kWgtGroup;

    uint32_t cls[PIX][KT][C::NCLS];
#pragma unroll
    for (int p = 0; p < PIX; ++p)
#pragma unroll
        for (int c = 0; c < KT; ++c)
#pragma unroll
            for (int s = 0; s < C::NCLS; ++s) cls[p][c][s] = 0u;

    for (int chunk = 0; chunk < sh.nchunks; ++chunk) {
        if (chunk > 0) __syncthreads();       // everyone is done with the previous chunk
        stage(chunk);
        __syncthreads();

        // weight words of this tile: [k/16][tap][word][k%16][plane]; per 16-channel group a
        // wave-uniform base pointer, plus one running offset over (tap, word)
        const uint32_t *wg[C::KG];
#pragma unroll
        for (int g = 0; g < C::KG; ++g) {
            // a tile may reach past the last packed group (its channels are never stored): re-read the last one
            const int gi = g0 + g < sh.wgroups ? g0 + g : sh.wgroups - 1;
            wg[g] = wgt + ((size_t)gi * sh.RS * sh.cw + (size_t)chunk * CH + wred) * (kWgtGroup * KW)
                        + (k0 % kWgtGroup) * KW;
        }
        constexpr int QSTEP = C::WRED * kWgtGroup * KW;                           // next word of this wave
        const int q_wrap = (sh.cw - (C::WSTEP - 1) * C::WRED) * (kWgtGroup * KW);  // first word of the next tap

        auto fetch_q = [&](int qoff, uint32_t (&q)[KT][KW]) {
#pragma unroll
            for (int g = 0; g < C::KG; ++g)
#pragma unroll
                for (int c = 0; c < C::KTG; ++c)
#pragma unroll
                    for (int i = 0; i < KW; ++i) q[g * kWgtGroup + c][i] = wg[g][qoff + c * KW + i];
        };
        auto fetch_x = [&](int off, uint32_t (&x)[PIX][KA]) {     // off: LDS dwords from the lane's position
#pragma unroll
            for (int p = 0; p < PIX; ++p) {
                typedef typename UVec<C::KAP>::type vec_t;
                const vec_t v = *reinterpret_cast<const vec_t *>(lds + my_lds[p] + off);
                if constexpr (C::KAP == 1) {
                    x[p][0] = v;
                } else {
#pragma unroll
                    for (int j = 0; j < KA; ++j) x[p][j] = v[j];
                }
            }
        };

        if (!EBS_DBG(2)) {
            uint32_t xc[PIX][KA], qc[KT][KW];
            const int wstride = sh.ucap * C::KAP;  // LDS dwords between consecutive words of a position
            const int w_first = wred * wstride;    // LDS dword offset of this wave's first word
            int tap_off = 0;                       // (r*Wp + s) * KAP of the current tap
            int s_col = 0;
            int qoff = 0;
            fetch_q(0, qc);
            fetch_x(w_first, xc);
            for (int tap = 0; tap < sh.RS; ++tap) {
                // LDS offset of the next tap
                int next_off = tap_off + C::KAP;
                int next_col = s_col + 1;
                if (next_col == sh.S) {
                    next_col = 0;
                    next_off += (sh.Wp - sh.S) * C::KAP;
                }
                const bool more_taps = tap + 1 < sh.RS;
#pragma unroll
                for (int ws = 0; ws < C::WSTEP; ++ws) {
                    const bool wrap = ws + 1 == C::WSTEP;      // known at compile time after unrolling
                    // request the operands of the following step first ...
                    uint32_t xn[PIX][KA], qn[KT][KW];
                    const bool have_next = !wrap || more_taps;
                    // The current operands were requested a whole step ago: wait for them BEFORE
                    // the next requests go out (LDS and scalar loads share one counter that can
                    // only be waited to zero, so a wait placed later would also cover the new ones).
                    __builtin_amdgcn_s_waitcnt(0xC07F);     // lgkmcnt(0) only
                    if (have_next) {
                        qoff += wrap ? q_wrap : QSTEP;
                        fetch_q(qoff, qn);
                        fetch_x(wrap ? next_off + w_first : tap_off + w_first + (ws + 1) * C::WRED * wstride, xn);
                    }
                    // ... then Eq. 2 / Eq. 13 on the current ones: AND + accumulating bitcount per plane pair
#pragma unroll
                    for (int p = 0; p < PIX; ++p)
#pragma unroll
                        for (int c = 0; c < KT; ++c)
#pragma unroll
                            for (int i = 0; i < KW; ++i)
#pragma unroll
                                for (int j = 0; j < KA; ++j)
                                    cls[p][c][i + j] = bcnt_acc(qc[c][i] & xc[p][j], cls[p][c][i + j]);
                    if (have_next) {
#pragma unroll
                        for (int p = 0; p < PIX; ++p)
#pragma unroll
                            for (int j = 0; j < KA; ++j) xc[p][j] = xn[p][j];
#pragma unroll
                        for (int c = 0; c < KT; ++c)
#pragma unroll
                            for (int i = 0; i < KW; ++i) qc[c][i] = qn[c][i];
                    }
                }
                tap_off = next_off;
                s_col = next_col;
            }
        }
    }

    // ---- Eq. 14: recombine the shift classes
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

    // ---- epilogue through LDS: [position][channel] tile, then coalesced write-back
    constexpr int CG = C::OCOLS / 4;              // 16-byte column groups per row
    constexpr int RSTEP = 256 / CG;               // rows covered by one sweep of the work-group
    const int cg = tid % CG;                      // this thread's column group (fixed)
    const int kq = kb0 + cg * 4;                  // its first channel
    float sc[4], of[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int k = kq + e < sh.K ? kq + e : sh.K - 1;
        const int ci = sh.per_channel ? k : 0;
        sc[e] = scale[ci];
        of[e] = offset ? offset[ci] : 0.0f;
    }
    const bool vec_ok = ((sh.K & 3) == 0) && (kq + 3 < sh.K);
    const int my_row = wpx * 64 + lane;
    const int my_col = wk * KT;

#pragma unroll
    for (int p = 0; p < PIX; ++p) {
        if (p > 0) __syncthreads();               // the previous pass has been written back
        if constexpr (MODE == MODE_R4) {
            // partial sums of the four waves meet in the tile
            if (wave == 0) {
#pragma unroll
                for (int c = 0; c < KT; c += 4) {
                    i32x4 v = {acc[p][c], acc[p][c + 1], acc[p][c + 2], acc[p][c + 3]};
                    *reinterpret_cast<i32x4 *>(otile + my_row * C::OPITCH + c) = v;
                }
            }
            __syncthreads();
            if (wave != 0) {
#pragma unroll
                for (int c = 0; c < KT; ++c) atomicAdd(&otile[my_row * C::OPITCH + c], acc[p][c]);
            }
        } else {
#pragma unroll
            for (int c = 0; c < KT; c += 4) {
                i32x4 v = {acc[p][c], acc[p][c + 1], acc[p][c + 2], acc[p][c + 3]};
                *reinterpret_cast<i32x4 *>(otile + my_row * C::OPITCH + my_col + c) = v;
            }
        }
        __syncthreads();
        if (EBS_DBG(1)) continue;
        // rows of this pass: row r of sub-tile w is position t_first + w*TPW + p*64 + r
#pragma unroll
        for (int r0 = 0; r0 < C::OROWS; r0 += RSTEP) {
            const int row = r0 + tid / CG;
            const int t = t_first + (row >> 6) * C::TPW + p * 64 + (row & 63);
            if (row < C::OROWS && t < sh.total && kq < sh.K) {
                const i32x4 v = *reinterpret_cast<const i32x4 *>(otile + row * C::OPITCH + cg * 4);
                const size_t o = (size_t)t * sh.K + kq;
                if (vec_ok) {
                    *reinterpret_cast<i32x4 *>(acc_out + o) = v;
                    if (out_f32 && !EBS_DBG(8)) {
                        f32x4 f = {fmaf((float)v[0], sc[0], of[0]), fmaf((float)v[1], sc[1], of[1]),
                                   fmaf((float)v[2], sc[2], of[2]), fmaf((float)v[3], sc[3], of[3])};
                        *reinterpret_cast<f32x4 *>(out_f32 + o) = f;
                    }
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        if (kq + e < sh.K) {
                            acc_out[o + e] = v[e];
                            if (out_f32 && !EBS_DBG(8)) out_f32[o + e] = fmaf((float)v[e], sc[e], of[e]);
                        }
                    }
                }
            }
        }
    }
#ifdef EBS_EXPERIMENT
    if (EBS_DBG(8) && out_f32 && tid == 0) {
        unsigned long long *tr = reinterpret_cast<unsigned long long *>(out_f32) + 2 * ((size_t)blockIdx.y * gridDim.x + blockIdx.x);
        tr[0] = exp_t0;
        tr[1] = wall_clock64();
    }
#endif
}

// ------------------------------------------------------------------ launch

// (PIX, KT) per accumulator budget and number of shift classes.
template <int BUDGET, int NCLS> struct TileOf;
#define EBS_TILE(b, n, p, k) template <> struct TileOf<b, n> { static constexpr int PIX = p, KT = k; };
EBS_TILE(128, 1, 4, 32) EBS_TILE(128, 2, 4, 16) EBS_TILE(128, 3, 4, 8) EBS_TILE(128, 4, 4, 8)
EBS_TILE(128, 5, 4, 4)  EBS_TILE(128, 6, 4, 4)  EBS_TILE(128, 7, 4, 4)
EBS_TILE(64, 1, 4, 16)  EBS_TILE(64, 2, 4, 8)   EBS_TILE(64, 3, 2, 8)  EBS_TILE(64, 4, 2, 8)
EBS_TILE(64, 5, 2, 4)   EBS_TILE(64, 6, 2, 4)   EBS_TILE(64, 7, 2, 4)
EBS_TILE(32, 1, 2, 16)  EBS_TILE(32, 2, 2, 8)   EBS_TILE(32, 3, 1, 8)  EBS_TILE(32, 4, 1, 8)
EBS_TILE(32, 5, 1, 4)   EBS_TILE(32, 6, 1, 4)   EBS_TILE(32, 7, 1, 4)
EBS_TILE(16, 1, 1, 16)  EBS_TILE(16, 2, 1, 8)   EBS_TILE(16, 3, 1, 4)  EBS_TILE(16, 4, 1, 4)
EBS_TILE(16, 5, 1, 4)   EBS_TILE(16, 6, 1, 4)   EBS_TILE(16, 7, 1, 4)
#undef EBS_TILE

static constexpr size_t kMaxLdsBytes = 64 * 1024;

template <int KW, int KA, int BUDGET, int CH, int MODE>
static int launch_cfg(const ConvArgs &a)
{
    constexpr int PIX = TileOf<BUDGET, KW + KA - 1>::PIX;
    constexpr int KT = TileOf<BUDGET, KW + KA - 1>::KT;
    using C = Cfg<KW, KA, PIX, KT, CH, MODE>;
    if (a.pad > kActBorder) return EBS_ERR_UNSUPPORTED;   // taps would leave the stored zero ring
    if (a.cw % CH != 0) return EBS_ERR_UNSUPPORTED;       // chunks are whole: no ragged last chunk
    TiledShape sh{};
    sh.N = a.N; sh.H = a.H; sh.W = a.W; sh.K = a.K; sh.R = a.R; sh.S = a.S;
    sh.stride = a.stride; sh.pad = a.pad; sh.OH = a.OH; sh.OW = a.OW; sh.cw = a.cw;
    sh.Hp = a.H + 2 * kActBorder; sh.Wp = a.W + 2 * kActBorder; sh.RS = a.R * a.S;
    sh.total = a.N * a.OH * a.OW;
    sh.nchunks = (a.cw + CH - 1) / CH;
    sh.per_channel = a.per_channel;
    sh.wgroups = (a.K + kWgtGroup - 1) / kWgtGroup;

    TileGeom g{a.H, a.W, a.R, a.S, a.stride, a.pad, a.OH, a.OW, kActBorder};
    long long tp = C::TP < sh.total ? C::TP : sh.total;
    long long ucap = g.extent_bound(tp);
    long long stage_dwords = (ucap * C::POSW + 3) / 4 * 4;
    size_t lds_bytes = (size_t)(stage_dwords + C::OUT_DWORDS) * sizeof(uint32_t);
    if (lds_bytes > kMaxLdsBytes || ucap > (1 << 28)) return EBS_ERR_UNSUPPORTED;
    sh.ucap = (int)ucap;
    sh.stage_dwords = (int)stage_dwords;
#ifdef EBS_EXPERIMENT
    if (const char *e = getenv("EBS_EXP_DBG")) sh.dbg = atoi(e);
#endif

    long long ptiles = ((long long)sh.total + C::TP - 1) / C::TP;
    long long kblocks = ((long long)a.K + C::KB - 1) / C::KB;
    if (ptiles > 0x7fffffffLL || kblocks > 65535) return EBS_ERR_UNSUPPORTED;

    hipLaunchKernelGGL((bd_conv_tiled<KW, KA, PIX, KT, CH, MODE>), dim3((unsigned)ptiles, (unsigned)kblocks), dim3(256),
                       lds_bytes, a.stream, a.act, a.wgt, a.scale, a.offset, a.acc, a.out, sh);
    return hip_ok(hipGetLastError());
}

// Variant table: (index, accumulator budget, words per staged chunk, wave arrangement).
#define EBS_TILED_VARIANTS(X)                                               \
    X(0, 128, 2, MODE_P4)  X(1, 128, 1, MODE_P4)  X(2, 128, 4, MODE_P4)     \
    X(3, 64, 2, MODE_P4)   X(4, 64, 1, MODE_P4)   X(5, 64, 4, MODE_P4)      \
    X(6, 32, 2, MODE_P4)   X(7, 32, 1, MODE_P4)   X(8, 32, 4, MODE_P4)      \
    X(9, 128, 2, MODE_K4)  X(10, 128, 1, MODE_K4) X(11, 128, 4, MODE_K4)    \
    X(12, 64, 2, MODE_K4)  X(13, 64, 1, MODE_K4)  X(14, 64, 4, MODE_K4)     \
    X(15, 32, 2, MODE_K4)  X(16, 32, 1, MODE_K4)  X(17, 32, 4, MODE_K4)     \
    X(18, 128, 4, MODE_R4) X(19, 64, 4, MODE_R4)  X(20, 32, 4, MODE_R4)     \
    X(21, 16, 2, MODE_K4)  X(22, 16, 1, MODE_K4)  X(23, 16, 4, MODE_K4)     \
    X(24, 16, 4, MODE_R4)
constexpr int kNumTiledVariants = 25;

template <int KW, int KA>
static int launch_bits(const ConvArgs &a, int v)
{
    switch (v) {
#define EBS_X(idx, b, ch, mode) case idx: return launch_cfg<KW, KA, b, ch, mode>(a);
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
