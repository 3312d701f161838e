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
//  * SGN adds, for the signed-weight form (integer weights 2q - (2^k_w - 1), Eq. 1a), the
//    bitcounts of the activation planes alone (window sum of the levels) and folds
//    2*acc - (2^k_w - 1)*window_sum into the epilogue; REQ replaces the int32/fp32 write-back
//    by the next layer's quantiser and bit-plane packing.
//  * MODE_PL (waves arranged as in MODE_K4) is stage 1 of the literal two-stage form of
//    Sec. 4.3 alone: one accumulator per plane pair (m, k) instead of per shift class, no
//    recombination; the k_w*k_a partial-product planes P are written out as int32 tensors.
//  * FS = 3 instantiates the 3x3 filter with the taps of a filter row unrolled
//    (tap offsets become instruction immediates); FS = 0 is the generic filter.
//  * the epilogue goes through LDS: accumulators are laid out [position][channel]
//    and written back by all 256 threads as 16-byte pieces of consecutive
//    addresses, so global stores cover whole runs of each NHWC output row.
//  * work-groups are numbered so that the eight accelerator dies (work-groups
//    are dealt to them round-robin) each take one contiguous eighth of the
//    position tiles: a die's L2 then only ever sees its own part of the input.
#pragma once
#include "ebs_internal.h"
#include "fastdiv.h"
#include "requant.h"
#include "tile_geometry.h"

namespace ebs {

enum { MODE_P4 = 0, MODE_K4 = 1, MODE_R4 = 2, MODE_PL = 3 };

struct TiledShape {
    int K, R, S, stride, pad, OW, cw, Hp, Wp, RS;   // Hp, Wp: bordered grid
    int total;        // N*OH*OW output positions
    int total_pos;    // N*Hp*Wp bordered input positions (packed input: [word][position][plane])
    int total_next;   // REQ: N*OHn*OWn bordered positions of the next layer's packed tensor
    int nchunks;      // cw / CH reduction chunks staged one at a time
    int per_channel;
    int ucap;         // staged positions that fit the LDS allocation
    int wgroups;      // 16-channel groups present in the packed weights
    int stage_dwords; // LDS dwords reserved for staged activations (the output tile follows)
    int kblocks;      // channel blocks per position tile
    int nblocks;      // position tiles * channel blocks
    int xcd_chunk;    // ceil(nblocks / 8): logical blocks handled by one die
    FastDiv div_ow, div_ohow, div_kblocks;
    // fused re-quantisation (REQ kernels only): next layer's quantiser and packed layout
    float alpha, qs;
    int k_next, OHn, OWn, cwn;     // bordered output grid (OH+2, OW+2), words per position of the next layer
    int ring_total, ring_per_image;  // dwords of the zero ring of the next layer's packed tensor (all images / one)
    int wtop;         // 0: unsigned weight levels; else 2^k_w - 1 (signed weights 2q - wtop, Eq. 1a)
    int gather;       // 1x1 filter without padding: stage exactly the tile's own positions (no halo, no ring)
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
    static constexpr bool PLN = MODE == MODE_PL;     // keep the plane pairs apart (stage 1 of Sec. 4.3 only)
    static constexpr int NCLS = PLN ? KW * KA : KW + KA - 1;     // accumulators per output
    // Staged planes per (position, word): padded to a power of two so that one LDS access fetches
    // them.  The fifth plane of five-bit activations lives in a second region, [word][position],
    // behind the four-plane one (a single eight-dword slot would put the lanes of a wave on one
    // bank in eight).
    static constexpr int KAP = (KA == 3 || KA == 5) ? 4 : KA;
    static constexpr int XTRA = KA == 5 ? 1 : 0;
    static constexpr int WAVES = 4;
    static constexpr int WPX = MODE == MODE_P4 ? 4 : 1;          // waves along the position axis
    static constexpr int WK = (MODE == MODE_K4 || PLN) ? 4 : 1;           // waves along the channel axis
    static constexpr int WRED = MODE == MODE_R4 ? 4 : 1;         // waves sharing one reduction
    static constexpr int TPW = 64 * PIX;             // positions per wave
    static constexpr int TP = WPX * TPW;             // positions per work-group
    static constexpr int KB = WK * KT;               // channels per work-group
    static constexpr int POSW = CH * (KAP + XTRA);   // LDS dwords per staged position (all words of the chunk)
    static constexpr int WSTEP = CH / WRED;          // reduction words per wave per tap per chunk
    static constexpr int WPS = (NCLS <= 2 && WSTEP % 2 == 0) ? 2 : 1;   // words per pipelined step (3x3 path)
    static constexpr int KG = (KT + kWgtGroup - 1) / kWgtGroup;   // 16-channel weight groups per tile
    static constexpr int KTG = KT < kWgtGroup ? KT : kWgtGroup;   // channels taken from one group
    // output tile of one epilogue pass, [row = position][col = channel], padded pitch
    static constexpr int OROWS = WPX * 64;
    static constexpr int OCOLS = KB;
    static constexpr int OPITCH = OCOLS + 4;
    static constexpr int OUT_DWORDS = OROWS * OPITCH;
    // fused re-quantisation: bit pieces of the next layer's words, bytes [position][plane][8-channel group]
    static constexpr int REQ_NG = KB / 8;                  // 8-channel groups of a work-group (4 per packed word)
    static constexpr int REQ_ROWB = kMaxBits * REQ_NG;     // bytes per position
    static constexpr int REQ_DWORDS = (TP * REQ_ROWB + 3) / 4;
    static_assert(CH % WRED == 0, "chunk must divide among the waves");
    static_assert(KT % 4 == 0 && (KT <= 16 ? 16 % KT == 0 : KT % 16 == 0), "channel tile vs weight group");
    static_assert(256 % (OCOLS / 4) == 0, "write-back assumes a fixed column group per thread");
};

template <int KW, int KA, int PIX, int KT, int CH, int MODE, int FS, bool REQ, bool SGN>
__global__ void __launch_bounds__(256)
bd_conv_tiled(const uint32_t *__restrict__ act, const uint32_t *__restrict__ wgt,
              const float *__restrict__ scale, const float *__restrict__ offset,
              int32_t *__restrict__ acc_out, float *__restrict__ out_f32, uint32_t *__restrict__ packed_next,
              const TiledShape sh)
{
    using C = Cfg<KW, KA, PIX, KT, CH, MODE>;
    extern __shared__ __attribute__((aligned(16))) uint32_t lds[];
    int32_t *otile = reinterpret_cast<int32_t *>(lds + sh.stage_dwords);

    // ---- which (position tile, channel block): dies take contiguous runs of logical blocks
    const int die = blockIdx.x & 7;
    const int slot = blockIdx.x >> 3;
    const int logical = die * sh.xcd_chunk + slot;
    if (slot >= sh.xcd_chunk || logical >= sh.nblocks) return;       // uniform for the whole work-group
    const int ptile = (int)fd_div((uint32_t)logical, sh.div_kblocks);
    const int kblock = logical - ptile * sh.kblocks;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wpx = MODE == MODE_P4 ? wave : 0;     // position sub-tile of this wave
    const int wk = (MODE == MODE_K4 || MODE == MODE_PL) ? wave : 0;      // channel sub-tile of this wave
    const int wred = MODE == MODE_R4 ? wave : 0;    // share of the reduction words
    const int R = FS > 0 ? FS : sh.R;
    const int S = FS > 0 ? FS : sh.S;
    const int RS = FS > 0 ? FS * FS : sh.RS;

    // ---- tile of output positions and the flat bordered-input range it reads
    const int t_first = ptile * C::TP;
    int t_last = t_first + C::TP - 1;
    if (t_last > sh.total - 1) t_last = sh.total - 1;
    const int origin = kActBorder - sh.pad;
    auto base_of = [&](int t) {
        const int n = (int)fd_div((uint32_t)t, sh.div_ohow);
        const int rem = t - n * (int)sh.div_ohow.d;
        const int oh = (int)fd_div((uint32_t)rem, sh.div_ow);
        const int ow = rem - oh * sh.OW;
        return (n * sh.Hp + oh * sh.stride + origin) * sh.Wp + ow * sh.stride + origin;
    };
    // 1x1 filters read one input position per output: the staged run is then indexed by the position's
    // number inside the tile, and the zero ring between rows and images is never copied
    const bool gather = FS == 0 && sh.gather;
    const int u_lo = base_of(t_first);
    int u_hi = base_of(t_last) + (R - 1) * sh.Wp + (S - 1);
    if (u_hi > u_lo + sh.ucap - 1) u_hi = u_lo + sh.ucap - 1;   // never beyond the LDS allocation

    int my_lds[PIX];          // LDS dword index of the lane's positions (tap 0, word 0)
#pragma unroll
    for (int p = 0; p < PIX; ++p) {
        int t = t_first + wpx * C::TPW + p * 64 + lane;
        int tc = t < sh.total ? t : sh.total - 1;
        my_lds[p] = (gather ? tc - t_first : base_of(tc) - u_lo) * C::KAP;
    }

    const int xtra_base = sh.ucap * CH * C::KAP;      // start of the fifth-plane region (five-bit activations)
    (void)xtra_base;

    // ---- staging of one reduction chunk: for every word, positions [u_lo, u_hi] of the bordered input
    //      are contiguous in memory (packed input [word][position][plane]); the 256 threads split into
    //      CH groups, one per word of the chunk, each copying its word's run with consecutive lanes on
    //      consecutive positions (interleaving the words over the lanes instead was up to 30 % slower on
    //      the deep stride-2 layers)
    const int n_pos = gather ? t_last - t_first + 1 : u_hi - u_lo + 1;
    constexpr int SG = 256 / CH;                 // threads per word
    static_assert(256 % CH == 0, "chunk words must divide the work-group");
    auto stage = [&](int chunk) {
        const int w = tid / SG;
        const uint32_t *srcw = act + ((size_t)(chunk * CH + w) * (unsigned)sh.total_pos + (unsigned)u_lo) * KA;
        for (int u = tid % SG; u < n_pos; u += SG) {
            const unsigned rel = gather ? (unsigned)(base_of(t_first + u) - u_lo) : (unsigned)u;
            const uint32_t *src = srcw + (size_t)rel * KA;
            uint32_t *dst = lds + (w * sh.ucap + u) * C::KAP;
            if constexpr (KA == 5) {
                const UVec<4>::type v4 = {src[0], src[1], src[2], src[3]};
                *reinterpret_cast<UVec<4>::type *>(dst) = v4;
                lds[xtra_base + w * sh.ucap + u] = src[4];
            } else {
                typedef typename UVec<C::KAP>::type vec_t;
                vec_t vv;
                if constexpr (C::KAP == 1) {
                    vv = src[0];
                } else {
#pragma unroll
                    for (int j = 0; j < C::KAP; ++j) vv[j] = j < KA ? src[j] : 0u;
                }
                *reinterpret_cast<vec_t *>(dst) = vv;
            }
        }
    };

    const int kb0 = kblock * C::KB;           // first channel of the work-group
    const int k0 = kb0 + wk * KT;             // first channel of this wave
    const int g0 = k0 / kWgtGroup;

    uint32_t cls[PIX][KT][C::NCLS];
#pragma unroll
    for (int p = 0; p < PIX; ++p)
#pragma unroll
        for (int c = 0; c < KT; ++c)
#pragma unroll
            for (int s = 0; s < C::NCLS; ++s) cls[p][c][s] = 0u;

    // signed weights only: bitcounts of the activation planes alone (the window sum of the levels)
    uint32_t wsum_cls[PIX][KA];
#pragma unroll
    for (int p = 0; p < PIX; ++p)
#pragma unroll
        for (int j = 0; j < KA; ++j) wsum_cls[p][j] = 0u;

    const int wstride = sh.ucap * C::KAP;     // LDS dwords between consecutive words of a position
    const int rowstride = sh.Wp * C::KAP;     // LDS dwords between filter rows

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
            wg[g] = wgt + ((size_t)gi * RS * sh.cw + (size_t)chunk * CH + wred) * (kWgtGroup * KW)
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
        auto load_x = [&](int idx, uint32_t (&x)[KA]) {          // idx: LDS dword index
            if constexpr (KA == 5) {
                const UVec<4>::type v = *reinterpret_cast<const UVec<4>::type *>(lds + idx);
#pragma unroll
                for (int j = 0; j < 4; ++j) x[j] = v[j];
                x[4] = lds[xtra_base + (idx >> 2)];
            } else {
                typedef typename UVec<C::KAP>::type vec_t;
                const vec_t v = *reinterpret_cast<const vec_t *>(lds + idx);
                if constexpr (C::KAP == 1) {
                    x[0] = v;
                } else {
#pragma unroll
                    for (int j = 0; j < KA; ++j) x[j] = v[j];
                }
            }
        };
        // Eq. 2 / Eq. 13 on one reduction word: AND + accumulating bitcount per plane pair
        auto mac = [&](const uint32_t (&x)[PIX][KA], const uint32_t (&q)[KT][KW]) {
#pragma unroll
            for (int p = 0; p < PIX; ++p)
#pragma unroll
                for (int c = 0; c < KT; ++c)
#pragma unroll
                    for (int i = 0; i < KW; ++i)
#pragma unroll
                        for (int j = 0; j < KA; ++j)
                        {
                            const int a_idx = C::PLN ? i * KA + j : i + j;
                            cls[p][c][a_idx] = bcnt_acc(q[c][i] & x[p][j], cls[p][c][a_idx]);
                        }
            if constexpr (SGN) {
#pragma unroll
                for (int p = 0; p < PIX; ++p)
#pragma unroll
                    for (int j = 0; j < KA; ++j) wsum_cls[p][j] = bcnt_acc(x[p][j], wsum_cls[p][j]);
            }
        };
        auto rotate = [&](uint32_t (&xc)[PIX][KA], uint32_t (&qc)[KT][KW],
                          const uint32_t (&xn)[PIX][KA], const uint32_t (&qn)[KT][KW]) {
#pragma unroll
            for (int p = 0; p < PIX; ++p)
#pragma unroll
                for (int j = 0; j < KA; ++j) xc[p][j] = xn[p][j];
#pragma unroll
            for (int c = 0; c < KT; ++c)
#pragma unroll
                for (int i = 0; i < KW; ++i) qc[c][i] = qn[c][i];
        };

        int qoff = 0;

        if constexpr (FS > 0) {
            // ---- fixed FS x FS filter: per filter row one LDS address per (position, word);
            //      the taps of the row are instruction immediates.  A step covers WPS words:
            //      two for the low bit products, whose single-word steps are too short to
            //      cover the operand latency when few waves share a SIMD.
            constexpr int WPS = C::WPS;
            constexpr int NGRP = C::WSTEP / WPS;       // steps per tap
            const int q_wrap_g = (sh.cw - (C::WSTEP - WPS) * C::WRED) * (kWgtGroup * KW);
            uint32_t xg[WPS][PIX][KA], qg[WPS][KT][KW];
            int addr[PIX][C::WSTEP];
#pragma unroll
            for (int p = 0; p < PIX; ++p)
#pragma unroll
                for (int ws = 0; ws < C::WSTEP; ++ws) addr[p][ws] = my_lds[p] + (ws * C::WRED + wred) * wstride;
#pragma unroll
            for (int u = 0; u < WPS; ++u) {
                fetch_q(u * QSTEP, qg[u]);
#pragma unroll
                for (int p = 0; p < PIX; ++p) load_x(addr[p][u], xg[u][p]);
            }
            for (int r = 0; r < FS; ++r) {
                const bool more_rows = r + 1 < FS;
#pragma unroll
                for (int s = 0; s < FS; ++s) {
#pragma unroll
                    for (int g = 0; g < NGRP; ++g) {
                        const bool wrap = g + 1 == NGRP;               // next step starts a new tap
                        const bool last_in_row = (s + 1 == FS) && wrap;
                        const bool have_next = !last_in_row || more_rows;
                        // The current operands were requested a whole step ago: wait for them BEFORE
                        // the next requests go out (LDS and scalar loads share one counter that can
                        // only be waited to zero, so a wait placed later would also cover the new ones).
                        __builtin_amdgcn_s_waitcnt(0xC07F);     // lgkmcnt(0) only
                        uint32_t xn[WPS][PIX][KA], qn[WPS][KT][KW];
                        if (have_next) {
                            qoff += wrap ? q_wrap_g : WPS * QSTEP;
                            const int nws = wrap ? 0 : (g + 1) * WPS;
                            const int noff = last_in_row ? rowstride : (wrap ? (s + 1) * C::KAP : s * C::KAP);
#pragma unroll
                            for (int u = 0; u < WPS; ++u) {
                                fetch_q(qoff + u * QSTEP, qn[u]);
#pragma unroll
                                for (int p = 0; p < PIX; ++p) load_x(addr[p][nws + u] + noff, xn[u][p]);
                            }
                        }
#pragma unroll
                        for (int u = 0; u < WPS; ++u) mac(xg[u], qg[u]);
                        if (have_next) {
#pragma unroll
                            for (int u = 0; u < WPS; ++u) rotate(xg[u], qg[u], xn[u], qn[u]);
                        }
                    }
                }
#pragma unroll
                for (int p = 0; p < PIX; ++p)
#pragma unroll
                    for (int ws = 0; ws < C::WSTEP; ++ws) addr[p][ws] += rowstride;
            }
        } else {
            // ---- generic filter: one LDS offset per tap, maintained incrementally
            const int w_first = wred * wstride;    // LDS dword offset of this wave's first word
            int tap_off = 0;                       // (r*Wp + s) * KAP of the current tap
            int s_col = 0;
            uint32_t xc[PIX][KA], qc[KT][KW];
            fetch_q(0, qc);
#pragma unroll
            for (int p = 0; p < PIX; ++p) load_x(my_lds[p] + w_first, xc[p]);
            for (int tap = 0; tap < RS; ++tap) {
                int next_off = tap_off + C::KAP;
                int next_col = s_col + 1;
                if (next_col == S) {
                    next_col = 0;
                    next_off += (sh.Wp - S) * C::KAP;
                }
                const bool more_taps = tap + 1 < RS;
#pragma unroll
                for (int ws = 0; ws < C::WSTEP; ++ws) {
                    const bool wrap = ws + 1 == C::WSTEP;      // known at compile time after unrolling
                    const bool have_next = !wrap || more_taps;
                    __builtin_amdgcn_s_waitcnt(0xC07F);        // lgkmcnt(0) only, see above
                    uint32_t xn[PIX][KA], qn[KT][KW];
                    if (have_next) {
                        qoff += wrap ? q_wrap : QSTEP;
                        fetch_q(qoff, qn);
                        const int off = wrap ? next_off + w_first : tap_off + w_first + (ws + 1) * C::WRED * wstride;
#pragma unroll
                        for (int p = 0; p < PIX; ++p) load_x(my_lds[p] + off, xn[p]);
                    }
                    mac(xc, qc);
                    if (have_next) rotate(xc, qc, xn, qn);
                }
                tap_off = next_off;
                s_col = next_col;
            }
        }
    }

    if constexpr (REQ) {
        // ---- fused re-quantisation (Eq. 1b-1c) and bit-plane packing of the next layer's activations.
        //      A lane holds KT channels of its positions: it quantises them and builds for every plane the
        //      KT-bit piece "bit j of the levels".  K4: the pieces go to LDS, bytes [position][plane][group of
        //      8 channels]; the four pieces of a 32-channel word are then one aligned dword, which the
        //      write-out copies to the packed tensor.  R4: the partial sums of the four waves first meet in
        //      LDS; the work-group owns 8 channels, one byte of each word, which wave 0 stores directly.
        //      P4 (layers with fewer than 32 output channels): every wave stores the bytes of its own positions.
        //      Every work-group also clears its share of the zero ring.
        static_assert(!REQ || (MODE == MODE_K4 && KT % 8 == 0 && C::KB % 32 == 0) ||
                          ((MODE == MODE_R4 || MODE == MODE_P4) && KT == 8 && PIX == 1),
                      "re-quantising kernels own whole bytes of the packed words");
        constexpr bool BYTES = MODE == MODE_R4 || MODE == MODE_P4;    // a wave's 8 channels are one byte of a word
        const int kmax = sh.k_next;
        int32_t sums[PIX][KT];
#pragma unroll
        for (int p = 0; p < PIX; ++p) {
            uint32_t ws = 0;
            if constexpr (SGN) {
#pragma unroll
                for (int j = 0; j < KA; ++j) ws += wsum_cls[p][j] << j;
            }
#pragma unroll
            for (int c = 0; c < KT; ++c) {
                uint32_t v = 0;
#pragma unroll
                for (int sft = 0; sft < C::NCLS; ++sft) v += cls[p][c][sft] << sft;       // Eq. 14
                sums[p][c] = (int32_t)v;
                if constexpr (SGN) sums[p][c] = 2 * sums[p][c] - sh.wtop * (int32_t)ws;   // linear: also for partial sums
            }
        }
        if constexpr (MODE == MODE_R4) {
            if (wave == 0) {
#pragma unroll
                for (int c = 0; c < KT; c += 4) {
                    i32x4 v = {sums[0][c], sums[0][c + 1], sums[0][c + 2], sums[0][c + 3]};
                    *reinterpret_cast<i32x4 *>(otile + lane * C::OPITCH + c) = v;
                }
            }
            __syncthreads();
            if (wave != 0) {
#pragma unroll
                for (int c = 0; c < KT; ++c) atomicAdd(&otile[lane * C::OPITCH + c], sums[0][c]);
            }
            __syncthreads();
            if (wave == 0) {
#pragma unroll
                for (int c = 0; c < KT; c += 4) {
                    const i32x4 v = *reinterpret_cast<const i32x4 *>(otile + lane * C::OPITCH + c);
                    sums[0][c] = v[0]; sums[0][c + 1] = v[1]; sums[0][c + 2] = v[2]; sums[0][c + 3] = v[3];
                }
            }
        }
        uint8_t *pieces = reinterpret_cast<uint8_t *>(otile);
        if (MODE != MODE_R4 || wave == 0) {
#pragma unroll
            for (int p = 0; p < PIX; ++p) {
                uint32_t piece[kMaxBits];
#pragma unroll
                for (int j = 0; j < kMaxBits; ++j) piece[j] = 0u;
#pragma unroll
                for (int c = 0; c < KT; ++c) {
                    const int k = k0 + c;                      // wave-uniform: scalar loads
                    const int kc = k < sh.K ? k : sh.K - 1;
                    const int ci = sh.per_channel ? kc : 0;
                    const uint32_t lv = k < sh.K ? requant_level(sums[p][c], scale[ci], offset ? offset[ci] : 0.0f, sh.alpha, sh.qs) : 0u;
#pragma unroll
                    for (int j = 0; j < kMaxBits; ++j) piece[j] |= ((lv >> j) & 1u) << c;
                }
                const int row = wpx * C::TPW + p * 64 + lane;
                if constexpr (BYTES) {
                    const int t = t_first + row;
                    if (t < sh.total) {
                        const int n = (int)fd_div((uint32_t)t, sh.div_ohow);
                        const int rem = t - n * (int)sh.div_ohow.d;
                        const int oh = (int)fd_div((uint32_t)rem, sh.div_ow);
                        const int ow = rem - oh * sh.OW;
                        const size_t pos = ((size_t)n * sh.OHn + oh + kActBorder) * sh.OWn + ow + kActBorder;
                        const int byte = (kb0 >> 3) & 3;
                        uint8_t *dstb = reinterpret_cast<uint8_t *>(packed_next + ((size_t)(kb0 >> 5) * sh.total_next + pos) * kmax) + byte;
                        const int fill = kb0 + 8 >= sh.K ? 3 - byte : 0;     // the last channel block also clears the rest of its word
#pragma unroll
                        for (int j = 0; j < kMaxBits; ++j) {
                            if (j < kmax) {
                                dstb[4 * j] = (uint8_t)piece[j];
                                for (int z = 1; z <= fill; ++z) dstb[4 * j + z] = 0;
                            }
                        }
                    }
                } else {
                    uint8_t *dst = pieces + row * C::REQ_ROWB + wk * (KT / 8);
#pragma unroll
                    for (int j = 0; j < kMaxBits; ++j) {
                        if (j < kmax) {
                            if constexpr (KT == 8) dst[j * C::REQ_NG] = (uint8_t)piece[j];
                            else *reinterpret_cast<uint16_t *>(dst + j * C::REQ_NG) = (uint16_t)piece[j];
                        }
                    }
                }
            }
        }
        if constexpr (!BYTES) {
            __syncthreads();
            constexpr int WPB = C::KB / 32;                // packed words of a position this work-group owns
            const int word0 = kb0 >> 5;
            const int items = C::TP * WPB;
            for (int it = tid; it < items; it += 256) {
                const int row = it / WPB;
                const int wd = it - row * WPB;
                const int t = t_first + row;
                if (t >= sh.total || word0 + wd >= sh.cwn) continue;
                const int n = (int)fd_div((uint32_t)t, sh.div_ohow);
                const int rem = t - n * (int)sh.div_ohow.d;
                const int oh = (int)fd_div((uint32_t)rem, sh.div_ow);
                const int ow = rem - oh * sh.OW;
                const size_t pos = ((size_t)n * sh.OHn + oh + kActBorder) * sh.OWn + ow + kActBorder;
                uint32_t *dstw = packed_next + ((size_t)(word0 + wd) * sh.total_next + pos) * kmax;
                const uint8_t *src = pieces + row * C::REQ_ROWB + wd * 4;
                for (int j = 0; j < kmax; ++j) dstw[j] = *reinterpret_cast<const uint32_t *>(src + j * C::REQ_NG);
            }
        }
        // zero ring of the next layer's tensor, dealt evenly to the work-groups: top row, bottom row,
        // then the left/right columns of every image
        const int wpp = sh.cwn * kmax;
        for (int idx = logical * 256 + tid; idx < sh.ring_total; idx += sh.nblocks * 256) {
            const int n = idx / sh.ring_per_image;
            const int rem = idx - n * sh.ring_per_image;
            const int b = rem / wpp;
            const int word = rem - b * wpp;
            int hp, wp;
            if (b < sh.OWn) { hp = 0; wp = b; }
            else if (b < 2 * sh.OWn) { hp = sh.OHn - 1; wp = b - sh.OWn; }
            else { const int cc = b - 2 * sh.OWn; hp = 1 + (cc >> 1); wp = (cc & 1) ? sh.OWn - 1 : 0; }
            const int wd = word / kmax, j = word - wd * kmax;
            packed_next[((size_t)wd * sh.total_next + ((size_t)n * sh.OHn + hp) * sh.OWn + wp) * kmax + j] = 0u;
        }
        return;
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
        sc[e] = C::PLN ? 0.0f : scale[ci];                   // the plane kernels take no scales
        of[e] = (!C::PLN && offset) ? offset[ci] : 0.0f;
    }
    const bool vec_ok = ((sh.K & 3) == 0) && (kq + 3 < sh.K);
    const int my_row = wpx * 64 + lane;
    const int my_col = wk * KT;

    // one pass per partial-product plane (stage 1 of Sec. 4.3 alone), else a single pass
    constexpr int NPL = C::PLN ? KW * KA : 1;
#pragma unroll
    for (int pl = 0; pl < NPL; ++pl) {
        int32_t *__restrict__ dst_acc = acc_out + (C::PLN ? (size_t)pl * (size_t)sh.total * (size_t)sh.K : 0);
        // ---- Eq. 14: recombine the shift classes
        int32_t acc[PIX][KT];
#pragma unroll
        for (int p = 0; p < PIX; ++p)
#pragma unroll
            for (int c = 0; c < KT; ++c) {
                uint32_t v = 0;
                if constexpr (C::PLN) {
                    v = cls[p][c][pl];                 // stage 1 only: plane pair pl = m*k_a + k as it is
                } else {
#pragma unroll
                    for (int s = 0; s < C::NCLS; ++s) v += cls[p][c][s] << s;
                }
                acc[p][c] = (int32_t)v;
            }
        if constexpr (SGN) {
            // integer weights 2q - wtop: 2 * sum(q*a) - wtop * sum(a); linear, so it also holds for the
            // partial sums of a reduction split among waves
#pragma unroll
            for (int p = 0; p < PIX; ++p) {
                uint32_t ws = 0;
#pragma unroll
                for (int j = 0; j < KA; ++j) ws += wsum_cls[p][j] << j;
#pragma unroll
                for (int c = 0; c < KT; ++c) acc[p][c] = 2 * acc[p][c] - sh.wtop * (int32_t)ws;
            }
        }

#pragma unroll
        for (int p = 0; p < PIX; ++p) {
            if (p > 0 || pl > 0) __syncthreads();     // the previous pass has been written back
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
            // rows of this pass: row r of sub-tile w is position t_first + w*TPW + p*64 + r
            {
#pragma unroll
            for (int r0 = 0; r0 < C::OROWS; r0 += RSTEP) {
                const int row = r0 + tid / CG;
                const int t = t_first + (row >> 6) * C::TPW + p * 64 + (row & 63);
                if (row < C::OROWS && t < sh.total && kq < sh.K) {
                    const i32x4 v = *reinterpret_cast<const i32x4 *>(otile + row * C::OPITCH + cg * 4);
                    const size_t o = (size_t)t * sh.K + kq;
                    if (vec_ok) {
                        *reinterpret_cast<i32x4 *>(dst_acc + o) = v;
                        if (!C::PLN && out_f32) {
                            f32x4 f = {fmaf((float)v[0], sc[0], of[0]), fmaf((float)v[1], sc[1], of[1]),
                                       fmaf((float)v[2], sc[2], of[2]), fmaf((float)v[3], sc[3], of[3])};
                            *reinterpret_cast<f32x4 *>(out_f32 + o) = f;
                        }
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            if (kq + e < sh.K) {
                                dst_acc[o + e] = v[e];
                                if (!C::PLN && out_f32) out_f32[o + e] = fmaf((float)v[e], sc[e], of[e]);
                            }
                        }
                    }
                }
            }
            }
        }
    }
}

// ------------------------------------------------------------------ launch

// (PIX, KT) per accumulator budget and number of shift classes.
template <int BUDGET, int NCLS> struct TileOf;
#define EBS_TILE(b, n, p, k) template <> struct TileOf<b, n> { static constexpr int PIX = p, KT = k; };
EBS_TILE(64, 1, 4, 16)  EBS_TILE(64, 2, 4, 8)   EBS_TILE(64, 3, 2, 8)  EBS_TILE(64, 4, 2, 8)
EBS_TILE(64, 5, 2, 4)   EBS_TILE(64, 6, 2, 4)   EBS_TILE(64, 7, 2, 4)   EBS_TILE(64, 8, 2, 4)  EBS_TILE(64, 9, 2, 4)
EBS_TILE(32, 1, 2, 16)  EBS_TILE(32, 2, 2, 8)   EBS_TILE(32, 3, 1, 8)  EBS_TILE(32, 4, 1, 8)
EBS_TILE(32, 5, 1, 4)   EBS_TILE(32, 6, 1, 4)   EBS_TILE(32, 7, 1, 4)   EBS_TILE(32, 8, 1, 4)  EBS_TILE(32, 9, 1, 4)
EBS_TILE(16, 1, 1, 16)  EBS_TILE(16, 2, 1, 8)   EBS_TILE(16, 3, 1, 4)  EBS_TILE(16, 4, 1, 4)
EBS_TILE(16, 5, 1, 4)   EBS_TILE(16, 6, 1, 4)   EBS_TILE(16, 7, 1, 4)   EBS_TILE(16, 8, 1, 4)  EBS_TILE(16, 9, 1, 4)
// budget 8: tiles of the re-quantising kernels (>= 8 channels per wave, so that the four waves of a
// work-group hold whole 32-channel words of the next layer's packed activations)
EBS_TILE(8, 1, 1, 16)   EBS_TILE(8, 2, 1, 8)    EBS_TILE(8, 3, 1, 8)   EBS_TILE(8, 4, 1, 8)
EBS_TILE(8, 5, 1, 8)    EBS_TILE(8, 6, 1, 8)    EBS_TILE(8, 7, 1, 8)    EBS_TILE(8, 8, 1, 8)   EBS_TILE(8, 9, 1, 8)
// budget 7: re-quantising kernels that split the reduction among the waves (MODE_R4): a work-group
// owns 8 channels, one byte of each packed word of the next layer
EBS_TILE(7, 1, 1, 8)    EBS_TILE(7, 2, 1, 8)    EBS_TILE(7, 3, 1, 8)   EBS_TILE(7, 4, 1, 8)
EBS_TILE(7, 5, 1, 8)    EBS_TILE(7, 6, 1, 8)    EBS_TILE(7, 7, 1, 8)    EBS_TILE(7, 8, 1, 8)   EBS_TILE(7, 9, 1, 8)
#undef EBS_TILE

// Tile of a (budget, k_w, k_a) kernel.  Budget 4 is the plane-pair kernel (MODE_PL): one
// position per lane and as many channels as k_w*k_a accumulators per output (<= 64 per lane)
// and the weight words per channel (<= 32 scalar registers per operand buffer) allow.
template <int BUDGET, int KW, int KA> struct TileSel {
    static constexpr int PIX = TileOf<BUDGET, KW + KA - 1>::PIX;
    static constexpr int KT = TileOf<BUDGET, KW + KA - 1>::KT;
};
// Five-bit activations with up to three weight bits: eight channels per wave (the shift-class table
// above would give four; the weight words are few here, and more channels share each activation fetch).
template <int KW> struct TileSelA5 {
    static constexpr int PIX = 1;
    static constexpr int KT = KW <= 3 ? 8 : 4;
};
template <> struct TileSel<16, 1, 5> : TileSelA5<1> {};
template <> struct TileSel<16, 2, 5> : TileSelA5<2> {};
template <> struct TileSel<16, 3, 5> : TileSelA5<3> {};
template <> struct TileSel<32, 1, 5> : TileSelA5<1> {};
template <> struct TileSel<32, 2, 5> : TileSelA5<2> {};
template <> struct TileSel<32, 3, 5> : TileSelA5<3> {};
// Budget 48 ("wide"): one position per lane, 8 channels per wave (16 for one shift class).  For 1x1 layers with
// a very short reduction, which are bound by their output writes: a work-group then writes 128-byte pieces of
// each output row instead of 64-byte ones, and each wave carries twice the arithmetic per set-up.
template <int KW, int KA> struct TileSel<48, KW, KA> {
    static constexpr int PIX = 1;
    static constexpr int KT = (KW + KA - 1 == 1) ? 16 : 8;
};
template <int KW, int KA> struct TileSel<4, KW, KA> {
    static constexpr int PIX = 1;
    static constexpr int KT_ACC = KW * KA <= 4 ? 16 : (KW * KA <= 8 ? 8 : 4);
    static constexpr int QW = KW * (KW * KA <= 2 ? 2 : 1);     // weight words per channel and step (two-word steps)
    static constexpr int KT_SGPR = 32 / QW >= 16 ? 16 : (32 / QW >= 8 ? 8 : 4);
    static constexpr int KT = KT_ACC < KT_SGPR ? KT_ACC : KT_SGPR;
};

static constexpr size_t kMaxLdsBytes = 64 * 1024;       // per work-group (dynamic LDS without opt-in)
static constexpr size_t kLdsPerCu = 160 * 1024;         // gfx950

template <int KW, int KA, int BUDGET, int CH, int MODE, int FS, bool REQ = false, bool SGN = false>
static int launch_cfg(const ConvArgs &a)
{
    if ((a.wtop != 0) != SGN) return EBS_ERR_UNSUPPORTED;
    constexpr int PIX = TileSel<BUDGET, KW, KA>::PIX;
    constexpr int KT = TileSel<BUDGET, KW, KA>::KT;
    using C = Cfg<KW, KA, PIX, KT, CH, MODE>;
    if (a.pad > kActBorder) return EBS_ERR_UNSUPPORTED;   // taps would leave the stored zero ring
    if (a.cw % CH != 0) return EBS_ERR_UNSUPPORTED;       // chunks are whole: no ragged last chunk
    if (FS > 0 && (a.R != FS || a.S != FS)) return EBS_ERR_UNSUPPORTED;
    TiledShape sh{};
    sh.K = a.K; sh.R = a.R; sh.S = a.S;
    sh.stride = a.stride; sh.pad = a.pad; sh.OW = a.OW; sh.cw = a.cw;
    sh.Hp = a.H + 2 * kActBorder; sh.Wp = a.W + 2 * kActBorder; sh.RS = a.R * a.S;
    sh.total = a.N * a.OH * a.OW;
    sh.total_pos = a.N * sh.Hp * sh.Wp;
    sh.nchunks = a.cw / CH;
    sh.per_channel = a.per_channel;
    sh.wgroups = (a.K + kWgtGroup - 1) / kWgtGroup;
    sh.div_ow = make_fastdiv((uint32_t)a.OW);
    sh.div_ohow = make_fastdiv((uint32_t)(a.OH * a.OW));
    sh.wtop = a.wtop;
    if (REQ) {
        sh.alpha = a.alpha;
        sh.k_next = a.k_next;
        sh.qs = requant_qs(a.alpha, a.k_next);
        sh.OHn = a.OH + 2 * kActBorder;
        sh.OWn = a.OW + 2 * kActBorder;
        sh.cwn = words_per_pixel(a.K);
        sh.total_next = a.N * sh.OHn * sh.OWn;
        const long long ring_pos = 2LL * sh.OWn + 2LL * a.OH;          // ring positions of one image
        const long long per_image = ring_pos * sh.cwn * a.k_next;
        if (per_image * a.N > (1LL << 30)) return EBS_ERR_UNSUPPORTED;
        sh.ring_per_image = (int)per_image;
        sh.ring_total = (int)(per_image * a.N);
    }

    TileGeom g{a.H, a.W, a.R, a.S, a.stride, a.pad, a.OH, a.OW, kActBorder};
    long long tp = C::TP < sh.total ? C::TP : sh.total;
    // worth its extra index arithmetic only where the ring is at least as large as the image (tiny images, and
    // a fully-connected layer given as a 1x1 convolution on 1x1 images): measured -12..35 % there, +8 % on 56x56
    sh.gather = (FS == 0 && a.R == 1 && a.S == 1 && a.pad == 0 &&
                 (long long)(a.H + 2 * kActBorder) * (a.W + 2 * kActBorder) >= 2LL * a.H * a.W) ? 1 : 0;
    long long ucap = sh.gather ? tp : g.extent_bound(tp);
    long long stage_dwords = (ucap * C::POSW + 3) / 4 * 4;
    size_t lds_bytes = (size_t)(stage_dwords + ((REQ && MODE == MODE_K4) ? C::REQ_DWORDS : C::OUT_DWORDS)) * sizeof(uint32_t);
    if (lds_bytes > kMaxLdsBytes || ucap > (1 << 28)) return EBS_ERR_UNSUPPORTED;
    sh.ucap = (int)ucap;
    sh.stage_dwords = (int)stage_dwords;

    long long ptiles = ((long long)sh.total + C::TP - 1) / C::TP;
    long long kblocks = ((long long)a.K + C::KB - 1) / C::KB;
    long long nblocks = ptiles * kblocks;
    if (nblocks > (1LL << 30)) return EBS_ERR_UNSUPPORTED;
    sh.kblocks = (int)kblocks;
    sh.nblocks = (int)nblocks;
    sh.xcd_chunk = (int)((nblocks + 7) / 8);
    sh.div_kblocks = make_fastdiv((uint32_t)kblocks);

    // A grid that fits the machine in one go is dealt unevenly to the compute units; asking
    // for more LDS than needed caps the work-groups per unit at ceil(nblocks / units).
    const DeviceShape *dev = device_shape();
    if (!dev) return EBS_ERR_HIP;
    if (!dev->gfx950) return EBS_ERR_UNSUPPORTED;       // tile sizes, LDS budget and die numbering are gfx950's
    long long per_cu = (nblocks + dev->cus - 1) / dev->cus;
    if (per_cu >= 2 && per_cu < 8) {
        size_t want = kLdsPerCu / (size_t)(per_cu + 1) + 512;
        if (want > kMaxLdsBytes) want = kMaxLdsBytes;
        if (want > lds_bytes) lds_bytes = want;
    }

    hipLaunchKernelGGL((bd_conv_tiled<KW, KA, PIX, KT, CH, MODE, FS, REQ, SGN>), dim3((unsigned)(sh.xcd_chunk * 8)), dim3(256),
                       lds_bytes, a.stream, a.act, a.wgt, a.scale, a.offset, a.acc, a.out, a.next, sh);
    return hip_ok(hipGetLastError());
}

// Variant table: (index, accumulator budget, words per staged chunk, wave arrangement).
#define EBS_TILED_VARIANTS(X)                                               \
    X(0, 64, 2, MODE_P4)   X(1, 64, 1, MODE_P4)   X(2, 64, 4, MODE_P4)      \
    X(3, 32, 2, MODE_P4)   X(4, 32, 1, MODE_P4)   X(5, 32, 4, MODE_P4)      \
    X(6, 64, 2, MODE_K4)   X(7, 64, 1, MODE_K4)   X(8, 64, 4, MODE_K4)      \
    X(9, 32, 2, MODE_K4)   X(10, 32, 1, MODE_K4)  X(11, 32, 4, MODE_K4)     \
    X(12, 16, 2, MODE_K4)  X(13, 16, 1, MODE_K4)  X(14, 16, 4, MODE_K4)     \
    X(15, 64, 4, MODE_R4)  X(16, 32, 4, MODE_R4)  X(17, 16, 4, MODE_R4)
// variants 18-20 ("wide", budget 48, chunks of 2 / 1 / 4 words) exist for the generic filter only (FS = 0):
// they serve 1x1 layers with very short reductions
constexpr int kNumTiledVariants = 21;

template <int KW, int KA, int FS>
static int launch_bits(const ConvArgs &a, int v)
{
    if (a.wtop) {
        // signed weights: only the variants the shape heuristic uses are instantiated
        switch (v) {
#define EBS_X(idx, b, ch, mode) case idx: return launch_cfg<KW, KA, b, ch, mode, FS, false, true>(a);
            EBS_X(3, 32, 2, MODE_P4)   EBS_X(4, 32, 1, MODE_P4)   EBS_X(5, 32, 4, MODE_P4)
            EBS_X(9, 32, 2, MODE_K4)   EBS_X(10, 32, 1, MODE_K4)  EBS_X(11, 32, 4, MODE_K4)
            EBS_X(12, 16, 2, MODE_K4)  EBS_X(13, 16, 1, MODE_K4)  EBS_X(14, 16, 4, MODE_K4)
            EBS_X(16, 32, 4, MODE_R4)  EBS_X(17, 16, 4, MODE_R4)
#undef EBS_X
        }
        return EBS_ERR_UNSUPPORTED;
    }
    if constexpr (KW == 5 || KA == 5) {
        // five-bit operands (the top of the paper's search space): the heuristic's variants only
        switch (v) {
#define EBS_X(idx, b, ch, mode) case idx: return launch_cfg<KW, KA, b, ch, mode, FS>(a);
            EBS_X(3, 32, 2, MODE_P4)   EBS_X(4, 32, 1, MODE_P4)   EBS_X(5, 32, 4, MODE_P4)
            EBS_X(9, 32, 2, MODE_K4)   EBS_X(10, 32, 1, MODE_K4)  EBS_X(11, 32, 4, MODE_K4)
            EBS_X(12, 16, 2, MODE_K4)  EBS_X(13, 16, 1, MODE_K4)  EBS_X(14, 16, 4, MODE_K4)
            EBS_X(17, 16, 4, MODE_R4)
#undef EBS_X
        }
        return EBS_ERR_UNSUPPORTED;
    } else {
        switch (v) {
#define EBS_X(idx, b, ch, mode) case idx: return launch_cfg<KW, KA, b, ch, mode, FS>(a);
            EBS_TILED_VARIANTS(EBS_X)
#undef EBS_X
        }
        if constexpr (FS == 0) {
            switch (v) {
                case 18: return launch_cfg<KW, KA, 48, 2, MODE_K4, FS>(a);
                case 19: return launch_cfg<KW, KA, 48, 1, MODE_K4, FS>(a);
                case 20: return launch_cfg<KW, KA, 48, 4, MODE_K4, FS>(a);
            }
        }
        return EBS_ERR_UNSUPPORTED;
    }
}

// Re-quantising kernels: K4 arrangement with chunk sizes 2 / 1 / 4 (variants 0 / 1 / 2), and the
// reduction-split arrangement for layers with few positions and a long reduction (variant 3), and the
// position-split arrangement with 8-channel work-groups for layers with few output channels (4 / 5:
// chunks of 2 / 1 words).
template <int KW, int KA, int FS, bool SGN>
static int launch_bits_req_sgn(const ConvArgs &a, int v)
{
    switch (v) {
        case 0: return launch_cfg<KW, KA, 8, 2, MODE_K4, FS, true, SGN>(a);
        case 1: return launch_cfg<KW, KA, 8, 1, MODE_K4, FS, true, SGN>(a);
        case 2: return launch_cfg<KW, KA, 8, 4, MODE_K4, FS, true, SGN>(a);
        case 3: return launch_cfg<KW, KA, 7, 4, MODE_R4, FS, true, SGN>(a);
        case 4: return launch_cfg<KW, KA, 7, 2, MODE_P4, FS, true, SGN>(a);
        case 5: return launch_cfg<KW, KA, 7, 1, MODE_P4, FS, true, SGN>(a);
    }
    return EBS_ERR_UNSUPPORTED;
}

template <int KW, int KA, int FS>
static int launch_bits_req(const ConvArgs &a, int v)
{
    return a.wtop ? launch_bits_req_sgn<KW, KA, FS, true>(a, v) : launch_bits_req_sgn<KW, KA, FS, false>(a, v);
}

// Plane-pair kernels (stage 1 of the two-stage form): chunk sizes 1 / 4 (variant 0 / 1); the
// planes are written where ConvArgs::acc points.
template <int KW, int KA, int FS>
static int launch_bits_planes(const ConvArgs &a, int v)
{
    if (a.wtop) return EBS_ERR_UNSUPPORTED;
    switch (v) {
        case 0: return launch_cfg<KW, KA, 4, 1, MODE_PL, FS>(a);
        case 1: return launch_cfg<KW, KA, 4, 4, MODE_PL, FS>(a);
    }
    return EBS_ERR_UNSUPPORTED;
}

// One object file per (k_w, k_a, filter specialisation) instantiates this (conv_tiled_inst.hip, compiled
// once per triple): kind 0 = plain convolution, 1 = re-quantising, 2 = plane pairs.
template <int KW, int KA, int FS> int launch_tiled_pair(const ConvArgs &a, int v, int kind);

#define EBS_DEFINE_TILED_PAIR(KWV, KAV, FSV)                                              \
    template <> int launch_tiled_pair<KWV, KAV, FSV>(const ConvArgs &a, int v, int kind)   \
    {                                                                                      \
        switch (kind) {                                                                    \
            case 0: return launch_bits<KWV, KAV, FSV>(a, v);                               \
            case 1: return launch_bits_req<KWV, KAV, FSV>(a, v);                           \
            case 2: return launch_bits_planes<KWV, KAV, FSV>(a, v);                        \
        }                                                                                  \
        return EBS_ERR_UNSUPPORTED;                                                        \
    }

}  // namespace ebs
