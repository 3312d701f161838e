// AND + bitcount convolution, "channel per lane" arrangement, for 3x3 and 1x1 filters (paper Sec. 3
// Eq. 2; Sec. 4.3 Eq. 13-14 fused into one kernel as in the tiled kernel: the bit-plane partial
// products stay in registers, one accumulator per shift class i+j).
//
// Mapping (CDNA4, 64-wide waves).  The waves of a work-group are independent: no LDS, no barrier.
//  * a lane owns ONE output channel; a wave owns 64 consecutive channels x a run of P consecutive
//    output positions of one output row (a "tile").
//  * activation words are wave-uniform.  The packed input is [word][position][plane] over the
//    zero-bordered grid, so the (P-1)*stride + filter-size input positions that one filter row of the run
//    touches are, for one reduction word, ONE contiguous piece of memory: it is fetched with
//    scalar loads and its words are the scalar operands of v_and_b32.  Weight words are per-lane
//    vector loads (one load brings the k_w planes of the lane's channel) and are reused for the P
//    positions.  Inner body per (word, plane pair, position): v_and_b32 v, s, v + accumulating
//    v_bcnt_u32_b32, as in the tiled kernel.
//  * everything about positions is wave-uniform and runs on the scalar unit; a wave stores 256
//    consecutive bytes of an NHWC output row per position straight from its accumulators.
//  * a reduction step is (filter row r, word w); the operands of the next step are requested
//    before the current step is multiplied.  The loop body is one block of instructions (offsets
//    advance by selects, not branches), which keeps the requests where they are written.
//  * layers whose output is one position per image (a fully-connected layer as a 1x1 convolution) take runs of
//    P consecutive IMAGES instead (template stride 0): the input piece of a step is then P pieces of k_a words,
//    one per image, and the launcher describes the batch as one output row of N positions.
//  * SPLIT, for layers with few positions and a long reduction (always with image runs): the four waves of a
//    work-group share ONE tile and take a quarter of the reduction steps each; the partial sums meet in LDS
//    (the only use of LDS and of a barrier here) and each wave finishes and stores its share of the positions.
#pragma once
#include "ebs_internal.h"
#include "fastdiv.h"
#include "requant.h"

#include <type_traits>

namespace ebs {

struct LaneShape {
    int K, cw, OH, OW;
    int Wp;             // bordered row length (W + 2)
    int plane_pos;      // bordered positions per image (H + 2) * (W + 2)
    int total_pos;      // N * plane_pos: positions per word of the packed input
    int origin;         // border - pad
    int runs;           // runs of P positions per output row
    int runs_full;      // TAILED kernels: the first runs_full runs of a row hold P positions, the others P - 1
    int kgroups;        // ceil(K / 64)
    int ntiles;         // N*OH * runs * kgroups
    int xcd_chunk;      // ceil(work-groups / 8): work-groups of one die
    int touch_ahead;    // tiles between a tile and the one whose input it brings into the L2 (multiple of kgroups)
    int touch_ahead_pos;    // the same in position tiles (touch_ahead / kgroups)
    int per_channel;
    int wtop;           // SGN kernels: 2^k_w - 1 (signed weights 2q - wtop, Eq. 1a)
    unsigned act_bytes, wgt_bytes;      // sizes of the packed operands
    FastDiv div_kgroups, div_runs, div_oh;
    // fused re-quantisation (REQ kernels): the next layer's quantiser and packed layout
    float alpha, qs;
    int k_next, OHn, OWn, cwn, total_next;
    int ring_total, ring_per_image;     // dwords of the zero ring of the next layer's packed tensor (all images / one)
};

__device__ __forceinline__ uint32_t lane_bcnt_acc(uint32_t x, uint32_t acc)
{
    uint32_t d;
    asm("v_bcnt_u32_b32 %0, %1, %2" : "=v"(d) : "v"(x), "v"(acc));
    return d;
}

// bitcount(x) alone: what the first product of an accumulator uses, so that accumulators need no clearing
__device__ __forceinline__ uint32_t lane_bcnt_first(uint32_t x)
{
    uint32_t d;
    asm("v_bcnt_u32_b32 %0, %1, 0" : "=v"(d) : "v"(x));
    return d;
}

__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }

// Per-lane memory accesses go through buffer instructions: address = descriptor base + per-lane byte offset
// (a register that never changes) + wave-uniform byte offset (a scalar register).  Nothing of the address
// arithmetic then runs on the vector unit, which this kernel keeps for AND + bitcount.
constexpr unsigned kRawBufferFlags = 0x00020000u;      // untyped 32-bit data (gfx9 family)

__device__ __forceinline__ __amdgpu_buffer_rsrc_t raw_buffer(const void *base, unsigned bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, (int)bytes, (int)kRawBufferFlags);
}

template <int NW> struct BufferLoad;
template <> struct BufferLoad<1> {
    static __device__ __forceinline__ void run(uint32_t (&q)[1], __amdgpu_buffer_rsrc_t r, unsigned lane_bytes, unsigned uni_bytes)
    {
        q[0] = __builtin_amdgcn_raw_buffer_load_b32(r, (int)lane_bytes, (int)uni_bytes, 0);
    }
};
template <> struct BufferLoad<2> {
    static __device__ __forceinline__ void run(uint32_t (&q)[2], __amdgpu_buffer_rsrc_t r, unsigned lane_bytes, unsigned uni_bytes)
    {
        typedef uint32_t v2 __attribute__((ext_vector_type(2)));
        const v2 v = __builtin_amdgcn_raw_buffer_load_b64(r, (int)lane_bytes, (int)uni_bytes, 0);
        q[0] = v.x; q[1] = v.y;
    }
};
template <> struct BufferLoad<3> {
    static __device__ __forceinline__ void run(uint32_t (&q)[3], __amdgpu_buffer_rsrc_t r, unsigned lane_bytes, unsigned uni_bytes)
    {
        typedef uint32_t v3 __attribute__((ext_vector_type(3)));
        const v3 v = __builtin_amdgcn_raw_buffer_load_b96(r, (int)lane_bytes, (int)uni_bytes, 0);
        q[0] = v.x; q[1] = v.y; q[2] = v.z;
    }
};
template <> struct BufferLoad<4> {
    static __device__ __forceinline__ void run(uint32_t (&q)[4], __amdgpu_buffer_rsrc_t r, unsigned lane_bytes, unsigned uni_bytes)
    {
        typedef uint32_t v4 __attribute__((ext_vector_type(4)));
        const v4 v = __builtin_amdgcn_raw_buffer_load_b128(r, (int)lane_bytes, (int)uni_bytes, 0);
        q[0] = v.x; q[1] = v.y; q[2] = v.z; q[3] = v.w;
    }
};

template <int I, int N, class F> __device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

// REQ: instead of the int32 / fp32 outputs the kernel applies the next layer's activation quantiser (Eq. 1b-1c) and
// writes the next layer's packed bit planes: a wave's 64 lanes are 64 consecutive channels, so the ballot of level
// bit j over the wave IS the pair of 32-channel words of plane j; the work-groups also clear the zero ring.
// TAILED: rows whose length is no multiple of P are covered without overlap by runs of P and of P - 1 positions
// (14 = 4 + 4 + 3 + 3).  A short run is a run of P that starts one position early and leaves its first position
// out: all its loads stay inside the row, and the arithmetic and the store of that position are skipped (one
// wave-uniform branch per step).
// SGN: signed weights 2q - (2^k_w - 1) (Eq. 1a): the result is 2 * sum(q*a) - (2^k_w - 1) * sum(a) over the window.
// The window sums of the activation levels do not depend on the channel: each step's share is counted on the scalar
// unit from the input piece the wave holds anyway.
template <int KW, int KA, int P, int ST, int FS, bool REQ, bool SPLIT = false, bool TAILED = false, bool SGN = false>
__global__ void __launch_bounds__(256)
bd_conv_lane(const uint32_t *__restrict__ act, const uint32_t *__restrict__ wgt,
             const float *__restrict__ scale, const float *__restrict__ offset,
             int32_t *__restrict__ acc_out, float *__restrict__ out_f32, uint32_t *__restrict__ packed_next,
             const LaneShape sh)
{
    constexpr int NCLS = KW + KA - 1;
    constexpr bool IMG = ST == 0;                 // runs over images (1x1 filter, one output position per image)
    static_assert(!IMG || (FS == 1 && SPLIT), "image runs: 1x1 filters, split reduction");
    static_assert(!IMG || (!REQ && !SGN), "image runs: plain outputs, unsigned weights");
    constexpr int XST = IMG ? 1 : ST;             // distance of consecutive positions in a step's registers
    constexpr int NSEG = (P - 1) * XST + FS;      // input positions one filter row of the run touches
    constexpr int XN = NSEG * KA;                 // dwords of one step's input piece
    constexpr int QSTEP = kWgtGroup * KW;         // weights [k/16][tap][word][k%16][plane]: dwords per (tap, word)

    // ---- this wave's tile: dies take contiguous runs of work-groups (work-groups are dealt to the dies
    //      round-robin), a work-group four consecutive tiles; everything here is wave-uniform
    const unsigned lane = threadIdx.x & 63;
    const unsigned lane4 = lane * 4u;
    const int wave = uni(threadIdx.x >> 6);
    if constexpr (REQ) {
        // zero ring of the next layer's tensor, dealt evenly to all work-groups of the grid (also those beyond the
        // last tile): top row, bottom row, then the left/right columns of every image
        const int kmax = sh.k_next;
        const int wpp = sh.cwn * kmax;
        for (int idx = (int)(blockIdx.x * 256 + threadIdx.x); idx < sh.ring_total; idx += (int)(gridDim.x * 256)) {
            const int ni = idx / sh.ring_per_image;
            const int rem = idx - ni * sh.ring_per_image;
            const int b = rem / wpp;
            const int word = rem - b * wpp;
            int hp, wp;
            if (b < sh.OWn) { hp = 0; wp = b; }
            else if (b < 2 * sh.OWn) { hp = sh.OHn - 1; wp = b - sh.OWn; }
            else { const int cc = b - 2 * sh.OWn; hp = 1 + (cc >> 1); wp = (cc & 1) ? sh.OWn - 1 : 0; }
            const int wd = word / kmax, j = word - wd * kmax;
            packed_next[((size_t)wd * sh.total_next + ((size_t)ni * sh.OHn + hp) * sh.OWn + wp) * kmax + j] = 0u;
        }
    }
    const int wgi = (int)(blockIdx.x & 7) * sh.xcd_chunk + (int)(blockIdx.x >> 3);
    const int tile = SPLIT ? wgi : wgi * 4 + wave;
    if ((int)(blockIdx.x >> 3) >= sh.xcd_chunk || tile >= sh.ntiles) return;
    const int ptile = (int)fd_div((uint32_t)tile, sh.div_kgroups);
    const int kg = tile - ptile * sh.kgroups;
    const int grow = (int)fd_div((uint32_t)ptile, sh.div_runs);       // n*OH + oh
    const int run = ptile - grow * sh.runs;
    const int n = (int)fd_div((uint32_t)grow, sh.div_oh);
    const int oh = grow - n * sh.OH;
    // first position of a run, and whether the run leaves its first position out (TAILED).  Otherwise the last run
    // of a row is moved left and the overlap is computed twice.
    auto run_start = [&](int r, bool &short_run) {
        int o = r * P;
        short_run = false;
        if constexpr (TAILED) {
            short_run = r >= sh.runs_full;
            if (short_run) o -= r - sh.runs_full + 1;
        }
        if (o > sh.OW - P) o = sh.OW - P;
        return o;
    };
    bool skip0;
    const int ow0 = run_start(run, skip0);

    const int k = kg * 64 + (int)lane;
    const int kc = k < sh.K ? k : sh.K - 1;
    // byte offset of the lane's channel in the packed weights
    const unsigned qlane = (unsigned)(((kc / kWgtGroup) * (FS * FS) * sh.cw * kWgtGroup + (kc % kWgtGroup)) * KW) * 4u;
    const __amdgpu_buffer_rsrc_t wbuf = raw_buffer(wgt, sh.wgt_bytes);
    const int ci = sh.per_channel ? kc : 0;
    const float sc = scale[ci];
    const float of = offset ? offset[ci] : 0.0f;

    // ---- the reduction: steps (filter row r, word w), w fastest.  Offsets of a step's operands (dwords):
    // (image runs: "ow0" is the first image of the run, its one input position is the piece)
    auto piece_of = [&](int n_, int oh_, int ow_) {
        if constexpr (IMG) return (unsigned)uni((ow_ * sh.plane_pos + sh.origin * sh.Wp + sh.origin) * KA);
        else return (unsigned)uni((n_ * sh.plane_pos + (oh_ * ST + sh.origin) * sh.Wp + ow_ * ST + sh.origin) * KA);
    };
    const unsigned img_step = (unsigned)sh.plane_pos * KA;      // image runs: dwords from one image's piece to the next
    const unsigned x_wstep = (unsigned)sh.total_pos * KA;                       // next word
    // reduction steps of this wave, and the (filter row, word) of its first one
    const int my_steps = SPLIT ? (FS * sh.cw) >> 2 : FS * sh.cw;
    const int step0 = SPLIT ? wave * my_steps : 0;
    const int r0 = FS == 1 ? 0 : (step0 >= sh.cw) + (step0 >= 2 * sh.cw);
    const int w0 = step0 - r0 * sh.cw;
    const unsigned piece0 = piece_of(n, oh, ow0);
    unsigned x_off = piece0 + (unsigned)w0 * x_wstep + (unsigned)(r0 * sh.Wp * KA);
    unsigned q_off = (unsigned)((r0 * FS * sh.cw + w0) * QSTEP);
    const unsigned x_rwrap = (unsigned)sh.Wp * KA - (unsigned)(sh.cw - 1) * x_wstep;   // first word of the next filter row
    const unsigned q_rwrap = (unsigned)((FS - 1) * sh.cw * QSTEP + QSTEP);
    const unsigned q_tap = (unsigned)(sh.cw * QSTEP);
    // Every step's input piece lies in another part of memory (steps go over words and filter rows), a step's
    // scalar loads are only requested one step ahead, and the input is read straight from device memory: taken
    // alone, each step would wait for it in turn.  Vector loads whose values are not used bring the pieces into
    // the L2 beforehand, one lane per step and 128-byte line:
    //  * the first tiles of a die (nothing ran before them) touch their own pieces,
    //  * every tile touches the pieces of the tile that the die starts `touch_ahead` tiles later - about one
    //    generation of resident waves - so that tile finds them in the L2 when it starts.
    constexpr int PF_LINES = IMG ? P : (XN - 1 + 31) / 32 + 1;
    const __amdgpu_buffer_rsrc_t abuf = raw_buffer(act, sh.act_bytes);
    auto touch = [&](unsigned tile_piece, uint32_t (&pf)[PF_LINES]) {
        const int steps = my_steps;               // <= 64 (launcher)
        const int sl = step0 + ((int)lane < steps ? (int)lane : steps - 1);
        const int r = FS == 1 ? 0 : (sl >= sh.cw) + (sl >= 2 * sh.cw);
        const unsigned piece = tile_piece + (unsigned)(sl - r * sh.cw) * x_wstep + (unsigned)(r * sh.Wp * KA);
#pragma unroll
        for (int ln = 0; ln < PF_LINES; ++ln) {
            const unsigned e = IMG ? (unsigned)ln * img_step : (unsigned)(ln * 32 < XN - 1 ? ln * 32 : XN - 1);
            pf[ln] = __builtin_amdgcn_raw_buffer_load_b32(abuf, (int)((piece + e) * 4u), 0, 0);
        }
    };
    uint32_t pf_own[PF_LINES], pf_ahead[PF_LINES];
    const int die_tile = SPLIT ? (int)(blockIdx.x >> 3) : (int)(blockIdx.x >> 3) * 4 + wave;   // index among the die's tiles
    const int die_tiles = SPLIT ? sh.xcd_chunk : sh.xcd_chunk * 4;
    const bool touch_own = die_tile < sh.touch_ahead && my_steps > 2;     // (two steps are requested at once anyway)
    if (touch_own) touch(piece0, pf_own);
    const bool touch_next = kg == 0 && die_tile + sh.touch_ahead < die_tiles && tile + sh.touch_ahead < sh.ntiles;
    if (touch_next) {
        // touch_ahead is a multiple of the channel groups: the tile ahead is channel group 0 of its positions
        const int ptile_a = ptile + sh.touch_ahead_pos;
        const int grow_a = (int)fd_div((uint32_t)ptile_a, sh.div_runs);
        const int run_a = ptile_a - grow_a * sh.runs;
        const int n_a = (int)fd_div((uint32_t)grow_a, sh.div_oh);
        const int oh_a = grow_a - n_a * sh.OH;
        bool short_a;
        const int ow_a = run_start(run_a, short_a);
        touch(piece_of(n_a, oh_a, ow_a), pf_ahead);
    }
    // REQ: what the epilogue needs of the next layer's tensor is worked out here and parked in vector registers
    // (the scalar registers are what the two input buffers of the reduction need): the address of the wave's
    // first output word, the distance to the second word of a plane for lanes 32-63, the writer lanes, the quantiser
    uint32_t rq_base_lo = 0, rq_base_hi = 0, rq_span = 0, rq_voff = 0, rq_k = 0, rq_flags = 0;
    float rq_alpha = 0.0f, rq_qs = 0.0f;
    if constexpr (REQ) {
        const size_t posn = ((size_t)n * sh.OHn + oh + kActBorder) * sh.OWn + ow0 + kActBorder;
        const size_t word_dwords = (size_t)sh.total_next * sh.k_next;       // from a word's planes to the next word's
        const uint64_t base = (uint64_t)(packed_next + (size_t)(kg * 2) * word_dwords + posn * sh.k_next);
        rq_base_lo = (uint32_t)base;
        rq_base_hi = (uint32_t)(base >> 32);
        rq_span = (uint32_t)((word_dwords + (size_t)P * sh.k_next) * 4);    // (launcher: below 2^31)
        rq_voff = (lane >> 5) ? (uint32_t)(word_dwords * 4) : 0u;
        rq_k = (uint32_t)sh.k_next;
        rq_flags = (((lane & 31u) == 0u && kg * 2 + (int)(lane >> 5) < sh.cwn) ? 1u : 0u) | (k < sh.K ? 2u : 0u);
        rq_alpha = sh.alpha;
        rq_qs = sh.qs;
        asm volatile("" : "+v"(rq_base_lo), "+v"(rq_base_hi), "+v"(rq_span), "+v"(rq_voff), "+v"(rq_k), "+v"(rq_flags),
                          "+v"(rq_alpha), "+v"(rq_qs));
    }
    // the affine map and the next layer's quantiser on position p of the run; the ballot of level bit j over the
    // 64 channel lanes is the pair of 32-channel words of plane j, stored by lanes 0 and 32
    auto requant_store = [&](int p, uint32_t v, __amdgpu_buffer_rsrc_t nbuf, int k_next) {
        const uint32_t lv = (rq_flags & 2u) ? requant_level((int32_t)v, sc, of, rq_alpha, rq_qs) : 0u;
#pragma unroll
        for (int j = 0; j < kMaxBits; ++j) {
            if (j < k_next) {
                const unsigned long long m = __ballot((lv >> j) & 1u);
                const uint32_t word = (lane >> 5) ? (uint32_t)(m >> 32) : (uint32_t)m;
                if (rq_flags & 1u)
                    __builtin_amdgcn_raw_buffer_store_b32(word, nbuf, (int)rq_voff, (int)((unsigned)(p * k_next + j) * 4u), 0);
            }
        }
    };
    auto requant_buffer = [&]() {
        const uint64_t base = ((uint64_t)(uint32_t)uni((int)rq_base_hi) << 32) | (uint32_t)uni((int)rq_base_lo);
        return raw_buffer(reinterpret_cast<const void *>(base), (unsigned)uni((int)rq_span));
    };
    // SGN: lane e (< XN) also reads word e of every step's input piece (see the window sums below)
    static_assert(!SGN || XN <= 64, "one lane per word of the input piece");
    const unsigned xv_lane = lane < (unsigned)XN ? lane4 : 0x80000000u;      // beyond any descriptor: reads 0
    const unsigned xv_shift = lane % KA;                                     // the lane's plane
    int w_next = w0;                              // word index of the step the offsets point at
    int left = my_steps;                          // steps not yet requested
    // request the operands of the step the offsets point at (one scalar piece of input, one per-lane load per
    // tap that brings the k_w planes), then move the offsets one step on - without a branch, so that the loop
    // body stays one block of instructions; past the last step the offsets stay where they are
    auto issue = [&](uint32_t (&x)[XN], uint32_t (&q)[FS][KW], uint32_t &xv) {
        const uint32_t *xs = act + x_off;         // wave-uniform address: scalar loads
        if constexpr (SGN) xv = __builtin_amdgcn_raw_buffer_load_b32(abuf, (int)xv_lane, (int)(x_off * 4u), 0);
        if constexpr (IMG) {
#pragma unroll
            for (int p = 0; p < P; ++p)
#pragma unroll
                for (int j = 0; j < KA; ++j) x[p * KA + j] = xs[(unsigned)p * img_step + (unsigned)j];
        } else {
#pragma unroll
            for (int e = 0; e < XN; ++e) x[e] = xs[e];
        }
#pragma unroll
        for (int s = 0; s < FS; ++s) BufferLoad<KW>::run(q[s], wbuf, qlane, (q_off + (unsigned)s * q_tap) * 4u);
        const bool more = --left > 0;
        const bool wrap = w_next + 1 == sh.cw;
        w_next = wrap ? 0 : w_next + 1;
        x_off += more ? (wrap ? x_rwrap : x_wstep) : 0u;
        q_off += more ? (wrap ? q_rwrap : (unsigned)QSTEP) : 0u;
    };

    // SGN: the window sums of the activation levels.  Besides the scalar loads, lane e (< XN) reads word e of every
    // step's input piece with a vector load and keeps a running sum of its bitcounts, weighted by its plane; what
    // a position's window holds is put together from those lanes once, after the reduction.  (Counting on the
    // scalar unit from the piece in scalar registers was tried first: the temporaries did not fit beside the two
    // input buffers.)
    uint32_t level_sum = 0u;
    auto window_sums = [&](uint32_t xv) {
        if constexpr (SGN) level_sum += (uint32_t)__builtin_popcount(xv) << xv_shift;
    };
    // (2^k_w - 1) * sum of the levels in the window of each position (wave-uniform; after the reduction)
    uint32_t wterm[P];
    auto window_terms = [&]() {
        if constexpr (SGN) {
            uint32_t column = level_sum;             // lane c * k_a: sum over the planes of input column c
#pragma unroll
            for (int j = 1; j < KA; ++j) column += __shfl_down(level_sum, j);
            uint32_t window = column;                // lane c * k_a: sum over the FS columns from c on
#pragma unroll
            for (int f = 1; f < FS; ++f) window += __shfl_down(column, f * KA);
#pragma unroll
            for (int p = 0; p < P; ++p)
                wterm[p] = (uint32_t)__builtin_amdgcn_readlane((int)window, p * XST * KA) * (uint32_t)sh.wtop;
        }
    };
    auto window_term = [&](int p) { return SGN ? wterm[p] : 0u; };
    uint32_t cls[P][NCLS];
    if constexpr (TAILED) {
        // (a position that is left out is never accumulated: give its registers a value)
#pragma unroll
        for (int c = 0; c < NCLS; ++c) cls[0][c] = 0u;
    }
    // Eq. 2 / Eq. 13 on one (filter row, word): the taps of the row for the P positions.  The very first step
    // writes every accumulator before it adds to it (shift class c first occurs at tap 0 with the smallest i).
    auto mac = [&](const uint32_t (&x)[XN], const uint32_t (&q)[FS][KW], uint32_t xv, auto first_step) {
        constexpr bool FIRST = decltype(first_step)::value;
        window_sums(xv);
        auto position = [&](auto pc) {
            constexpr int p = decltype(pc)::value;
#pragma unroll
            for (int s = 0; s < FS; ++s)
#pragma unroll
                for (int i = 0; i < KW; ++i)
#pragma unroll
                    for (int j = 0; j < KA; ++j) {
                        const uint32_t v = q[s][i] & x[(p * XST + s) * KA + j];
                        if (FIRST && s == 0 && (i == 0 || j == KA - 1))
                            cls[p][i + j] = lane_bcnt_first(v);
                        else
                            cls[p][i + j] = lane_bcnt_acc(v, cls[p][i + j]);
                    }
        };
        if constexpr (TAILED) {
            if (!skip0) position(std::integral_constant<int, 0>{});
            static_for<1, P>(position);
        } else {
#pragma unroll
            for (int s = 0; s < FS; ++s)
#pragma unroll
                for (int p = 0; p < P; ++p)
#pragma unroll
                    for (int i = 0; i < KW; ++i)
#pragma unroll
                        for (int j = 0; j < KA; ++j) {
                            const uint32_t v = q[s][i] & x[(p * XST + s) * KA + j];
                            if (FIRST && s == 0 && (i == 0 || j == KA - 1))
                                cls[p][i + j] = lane_bcnt_first(v);
                            else
                                cls[p][i + j] = lane_bcnt_acc(v, cls[p][i + j]);
                        }
        }
    };
    using first_t = std::integral_constant<bool, true>;
    using later_t = std::integral_constant<bool, false>;

    // Each step's operands are requested one step ahead; the loop takes two steps per trip (the launcher admits
    // only shapes whose number of steps, filter rows * words, is even).
    // Scalar loads can only be waited for all at once.  A step therefore first waits for its own input piece
    // (requested one step ago), then requests the next step's, then multiplies: the wait the multiplication needs
    // would otherwise also cover the request just made.
    uint32_t xa[XN], xb[XN], qa[FS][KW], qb[FS][KW];
    uint32_t va = 0u, vb = 0u;                    // SGN: the lanes' words of the two pieces
    const int trips = my_steps >> 1;
    issue(xa, qa, va);
    __builtin_amdgcn_s_waitcnt(0xC07F);           // lgkmcnt(0)
    __builtin_amdgcn_sched_barrier(0);
    issue(xb, qb, vb);
    __builtin_amdgcn_sched_barrier(0);
    mac(xa, qa, va, first_t{});
    __builtin_amdgcn_sched_barrier(0);
    for (int t = 1; t < trips; ++t) {
        __builtin_amdgcn_s_waitcnt(0xC07F);
        __builtin_amdgcn_sched_barrier(0);
        issue(xa, qa, va);
        __builtin_amdgcn_sched_barrier(0);
        mac(xb, qb, vb, later_t{});
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_waitcnt(0xC07F);
        __builtin_amdgcn_sched_barrier(0);
        issue(xb, qb, vb);
        __builtin_amdgcn_sched_barrier(0);
        mac(xa, qa, va, later_t{});
        __builtin_amdgcn_sched_barrier(0);
    }
    __builtin_amdgcn_s_waitcnt(0xC07F);
    __builtin_amdgcn_sched_barrier(0);
    mac(xb, qb, vb, later_t{});

    window_terms();
    // (keeps the touching loads)
    if (touch_own) {
#pragma unroll
        for (int ln = 0; ln < PF_LINES; ++ln) asm volatile("" ::"v"(pf_own[ln]));
    }
    if (touch_next) {
#pragma unroll
        for (int ln = 0; ln < PF_LINES; ++ln) asm volatile("" ::"v"(pf_ahead[ln]));
    }

    if constexpr (REQ && !SPLIT) {
        // ---- Eq. 14, then the next layer's levels and bit planes
        const __amdgpu_buffer_rsrc_t nbuf = requant_buffer();
        const int k_next = uni((int)rq_k);
#pragma unroll
        for (int p = 0; p < P; ++p) {
            if (TAILED && p == 0 && skip0) continue;       // (wave-uniform)
            uint32_t v = cls[p][0];
#pragma unroll
            for (int c = 1; c < NCLS; ++c) v += cls[p][c] << c;
            if constexpr (SGN) v = 2u * v - window_term(p);
            requant_store(p, v, nbuf, k_next);
        }
        return;
    }
    if constexpr (SPLIT) {
        // ---- Eq. 14 over the wave's quarter of the reduction; the quarters meet in LDS, and wave w finishes
        //      positions w, w + 4, ... (sum of the four quarters, affine epilogue, 64 consecutive values each)
        __shared__ uint32_t part[4][P][64];
#pragma unroll
        for (int p = 0; p < P; ++p) {
            uint32_t v = 0;
#pragma unroll
            for (int c = 0; c < NCLS; ++c) v += cls[p][c] << c;
            if constexpr (SGN) v = 2u * v - window_term(p);    // linear: holds for the quarters' partial sums
            part[wave][p][lane] = v;
        }
        __syncthreads();
        if constexpr (REQ) {
            // the next layer's levels and bit planes of the wave's positions
            const __amdgpu_buffer_rsrc_t nbuf = requant_buffer();
            const int k_next = uni((int)rq_k);
#pragma unroll
            for (int pp = 0; pp < (P + 3) / 4; ++pp) {
                const int p = wave + 4 * pp;
                if (p >= P) break;
                if (TAILED && p == 0 && skip0) continue;
                requant_store(p, part[0][p][lane] + part[1][p][lane] + part[2][p][lane] + part[3][p][lane], nbuf, k_next);
            }
            return;
        }
        const size_t o0 = ((size_t)grow * sh.OW + ow0) * sh.K + (size_t)(kg * 64);
        const unsigned prow = (unsigned)sh.K * 4u;
        const unsigned span = (unsigned)(P - 1) * prow + (unsigned)(sh.K - kg * 64 < 64 ? sh.K - kg * 64 : 64) * 4u;
        const __amdgpu_buffer_rsrc_t ibuf = raw_buffer(acc_out + o0, span);
        const __amdgpu_buffer_rsrc_t fbuf = raw_buffer(out_f32 ? out_f32 + o0 : nullptr, out_f32 ? span : 0u);
        if (k < sh.K) {
#pragma unroll
            for (int pp = 0; pp < (P + 3) / 4; ++pp) {
                const int p = wave + 4 * pp;
                if (p >= P) break;
                if (TAILED && p == 0 && skip0) continue;
                const uint32_t v = part[0][p][lane] + part[1][p][lane] + part[2][p][lane] + part[3][p][lane];
                __builtin_amdgcn_raw_buffer_store_b32(v, ibuf, (int)lane4, (int)((unsigned)p * prow), 0);
                if (out_f32)
                    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, fmaf((float)(int32_t)v, sc, of)),
                                                          fbuf, (int)lane4, (int)((unsigned)p * prow), 0);
            }
        }
        return;
    }
    // ---- Eq. 14 and the affine epilogue; per position a wave writes 64 consecutive values
    if (k < sh.K) {
        int32_t acc[P];
#pragma unroll
        for (int p = 0; p < P; ++p) {
            uint32_t v = 0;
#pragma unroll
            for (int c = 0; c < NCLS; ++c) v += cls[p][c] << c;
            if constexpr (SGN) v = 2u * v - window_term(p);
            acc[p] = (int32_t)v;
        }
        // descriptors that start at the wave's first output value and end after its last one (the range check
        // counts the scalar offset too); the lane offset selects the channel, the scalar offset the position
        const size_t o0 = ((size_t)grow * sh.OW + ow0) * sh.K + (size_t)(kg * 64);
        const unsigned prow = (unsigned)sh.K * 4u;
        const unsigned span = (unsigned)(P - 1) * prow + (unsigned)(sh.K - kg * 64 < 64 ? sh.K - kg * 64 : 64) * 4u;
        const __amdgpu_buffer_rsrc_t ibuf = raw_buffer(acc_out + o0, span);
#pragma unroll
        for (int p = 0; p < P; ++p) {
            if (TAILED && p == 0 && skip0) continue;
            __builtin_amdgcn_raw_buffer_store_b32((uint32_t)acc[p], ibuf, (int)lane4, (int)((unsigned)p * prow), 0);
        }
        if (out_f32) {
            const __amdgpu_buffer_rsrc_t fbuf = raw_buffer(out_f32 + o0, span);
#pragma unroll
            for (int p = 0; p < P; ++p) {
                if (TAILED && p == 0 && skip0) continue;
                __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, fmaf((float)acc[p], sc, of)), fbuf,
                                                      (int)lane4, (int)((unsigned)p * prow), 0);
            }
        }
    }
}

// Positions per run: the large choice where accumulators (P * shift classes) and the scalar registers of the
// input pieces (two buffers of ((P-1)*stride + filter size) * k_a) allow it, and a small one for narrow rows.
template <int KW, int KA, int ST, int FS = 3> struct LaneRun {
    static constexpr int NCLS = KW + KA - 1;
    static constexpr int BIG = ST == 1 ? ((KA <= 2 && NCLS <= 4) ? 14 : 7) : (KA <= 2 ? 7 : 4);
    static constexpr int SMALL = ST == 1 ? 7 : 4;
    // stride 2 with three or four activation bits has only the runs of four (scalar registers): rows of 14 or 7
    // outputs are covered as 4 + 4 + 3 + 3 and 4 + 3
    static constexpr bool TAILED = ST == 2 && KA >= 3;
};

template <int KW, int KA, int P, int ST, int FS, bool REQ, bool SPLIT = false, bool TAILED = false, bool SGN = false>
static int launch_lane_cfg(const ConvArgs &a)
{
    constexpr bool IMG = ST == 0;       // runs over images: one output position per image
    if ((a.wtop != 0) != SGN || (a.next != nullptr) != REQ) return EBS_ERR_UNSUPPORTED;
    if (a.R != FS || a.S != FS || a.pad > kActBorder) return EBS_ERR_UNSUPPORTED;
    if (IMG ? (a.OH != 1 || a.OW != 1 || a.N < P) : (a.stride != ST || a.OW < P)) return EBS_ERR_UNSUPPORTED;
    // image runs: the batch is described to the kernel as one output row of N positions
    const int rows = IMG ? 1 : a.N * a.OH;
    const int row_len = IMG ? a.N : a.OW;
    // the loop takes two steps (filter row, word) per trip; one lane per step touches the step's input piece
    // (split reduction: per wave, a quarter of the steps)
    if (SPLIT ? (((FS * a.cw) & 7) || FS * a.cw > 256) : (((FS * a.cw) & 1) || FS * a.cw > 64)) return EBS_ERR_UNSUPPORTED;
    constexpr int FSZ = FS * FS;
    LaneShape sh{};
    sh.K = a.K; sh.cw = a.cw; sh.OH = IMG ? 1 : a.OH; sh.OW = row_len;
    sh.Wp = a.W + 2 * kActBorder;
    sh.plane_pos = (a.H + 2 * kActBorder) * sh.Wp;
    sh.total_pos = a.N * sh.plane_pos;
    sh.origin = kActBorder - a.pad;
    sh.runs = (row_len + P - 1) / P;
    sh.runs_full = sh.runs;
    if (TAILED) {
        // exact cover by runs of P and P - 1 where the row is long enough for it
        const int shorter = sh.runs * P - row_len;
        if (shorter < sh.runs) sh.runs_full = sh.runs - shorter;
    }
    sh.kgroups = (a.K + 63) / 64;
    long long ntiles = (long long)rows * sh.runs * sh.kgroups;
    if (ntiles > (1LL << 30)) return EBS_ERR_UNSUPPORTED;
    sh.ntiles = (int)ntiles;
    sh.per_channel = a.per_channel;
    sh.wtop = a.wtop;
    const size_t act_bytes = (size_t)sh.total_pos * a.cw * KA * sizeof(uint32_t);
    const size_t wgt_bytes = (size_t)((a.K + kWgtGroup - 1) / kWgtGroup) * kWgtGroup * FSZ * a.cw * KW * sizeof(uint32_t);
    if (act_bytes >= (1ull << 31) || wgt_bytes >= (1ull << 31)) return EBS_ERR_UNSUPPORTED;   // 32-bit byte offsets
    sh.act_bytes = (unsigned)act_bytes;
    sh.wgt_bytes = (unsigned)wgt_bytes;
    sh.div_kgroups = make_fastdiv((uint32_t)sh.kgroups);
    sh.div_runs = make_fastdiv((uint32_t)sh.runs);
    sh.div_oh = make_fastdiv((uint32_t)sh.OH);

    if (REQ) {
        sh.alpha = a.alpha;
        sh.k_next = a.k_next;
        sh.qs = requant_qs(a.alpha, a.k_next);
        sh.OHn = a.OH + 2 * kActBorder;
        sh.OWn = a.OW + 2 * kActBorder;
        sh.cwn = words_per_pixel(a.K);
        sh.total_next = a.N * sh.OHn * sh.OWn;
        // (the epilogue addresses the second word of a plane by a 32-bit byte offset from the first)
        if (((long long)sh.total_next + P) * a.k_next * 4 >= (1LL << 31)) return EBS_ERR_UNSUPPORTED;
        const long long per_image = (2LL * sh.OWn + 2LL * a.OH) * sh.cwn * a.k_next;
        if (per_image * a.N > (1LL << 30)) return EBS_ERR_UNSUPPORTED;
        sh.ring_per_image = (int)per_image;
        sh.ring_total = (int)(per_image * a.N);
    }
    const DeviceShape *dev = device_shape();
    if (!dev) return EBS_ERR_HIP;
    if (!dev->gfx950) return EBS_ERR_UNSUPPORTED;       // run lengths and die numbering are gfx950's
    const long long wgs = SPLIT ? ntiles : (ntiles + 3) / 4;
    sh.xcd_chunk = (int)((wgs + 7) / 8);
    // one generation of resident waves of a die: 32 compute units x 4 SIMDs x 8 waves
    sh.touch_ahead_pos = (dev->cus / 8 * 32 / (SPLIT ? 4 : 1) + sh.kgroups - 1) / sh.kgroups;
    sh.touch_ahead = sh.touch_ahead_pos * sh.kgroups;
    hipLaunchKernelGGL((bd_conv_lane<KW, KA, P, ST, FS, REQ, SPLIT, TAILED, SGN>), dim3((unsigned)(sh.xcd_chunk * 8)), dim3(256), 0, a.stream,
                       a.act, a.wgt, a.scale, a.offset, a.acc, a.out, a.next, sh);
    return hip_ok(hipGetLastError());
}

// sel: 0 = large runs, 1 = small runs, 2 = small runs with the reduction split among a work-group's waves
template <int KW, int KA, int FS, bool REQ, bool SGN = false>
static int launch_lane_fs(const ConvArgs &a, int sel)
{
    using R1 = LaneRun<KW, KA, 1, FS>;
    using R2 = LaneRun<KW, KA, 2, FS>;
    if (sel == 2) {
        if (a.stride == 1) return launch_lane_cfg<KW, KA, R1::SMALL, 1, FS, REQ, true, false, SGN>(a);
        if constexpr (FS == 3) {
            if (a.stride == 2) return launch_lane_cfg<KW, KA, R2::BIG, 2, FS, REQ, true, R2::TAILED, SGN>(a);
        }
        return EBS_ERR_UNSUPPORTED;
    }
    if (a.stride == 1) {
        if (sel == 0) return launch_lane_cfg<KW, KA, R1::BIG, 1, FS, REQ, false, false, SGN>(a);
        return launch_lane_cfg<KW, KA, R1::SMALL, 1, FS, REQ, false, false, SGN>(a);
    }
    if (a.stride == 2) {
        if (sel == 0) return launch_lane_cfg<KW, KA, R2::BIG, 2, FS, REQ, false, R2::TAILED, SGN>(a);
        return launch_lane_cfg<KW, KA, R2::SMALL, 2, FS, REQ, false, R2::TAILED, SGN>(a);
    }
    return EBS_ERR_UNSUPPORTED;
}

// Runs of images for layers with one output position per image (1x1 filters): 8 images, or 4 for small batches
template <int KW, int KA>
static int launch_lane_images(const ConvArgs &a, int sel)
{
    if (sel == 0) return launch_lane_cfg<KW, KA, 8, 0, 1, false, true>(a);
    return launch_lane_cfg<KW, KA, 4, 0, 1, false, true>(a);
}

template <int KW, int KA>
static int launch_lane_pair_impl(const ConvArgs &a, int sel)
{
    if (!a.next && a.R == 1 && a.S == 1 && a.OH == 1 && a.OW == 1) return launch_lane_images<KW, KA>(a, sel);
    // signed weights: the 3x3 kernels only
    if (a.wtop) {
        if (a.R != 3 || a.S != 3) return EBS_ERR_UNSUPPORTED;
        return a.next ? launch_lane_fs<KW, KA, 3, true, true>(a, sel) : launch_lane_fs<KW, KA, 3, false, true>(a, sel);
    }
    if (a.next) {
        if (a.R == 3 && a.S == 3) return launch_lane_fs<KW, KA, 3, true>(a, sel);
        if (a.R == 1 && a.S == 1) return launch_lane_fs<KW, KA, 1, true>(a, sel);
        return EBS_ERR_UNSUPPORTED;
    }
    if (a.R == 3 && a.S == 3) return launch_lane_fs<KW, KA, 3, false>(a, sel);
    if (a.R == 1 && a.S == 1) return launch_lane_fs<KW, KA, 1, false>(a, sel);
    return EBS_ERR_UNSUPPORTED;
}

template <int KW, int KA> int launch_lane_pair(const ConvArgs &a, int sel);

#define EBS_DEFINE_LANE_PAIR(KWV, KAV)                                                     \
    template <> int launch_lane_pair<KWV, KAV>(const ConvArgs &a, int sel)                 \
    {                                                                                      \
        return launch_lane_pair_impl<KWV, KAV>(a, sel);                                    \
    }

}  // namespace ebs
