// Variant table and shape heuristics of the tiled convolution; the kernels are instantiated per
// (k_w, k_a, filter specialisation) from conv_tiled_inst.hip.
#include "ebs_internal.h"

namespace ebs {

template <int KW, int KA, int FS> int launch_tiled_pair(const ConvArgs &a, int v, int kind);
#define EBS_PAIRS(X)                                            \
    X(1, 1) X(1, 2) X(1, 3) X(1, 4) X(1, 5) X(2, 1) X(2, 2) X(2, 3) X(2, 4) X(2, 5) \
    X(3, 1) X(3, 2) X(3, 3) X(3, 4) X(3, 5) X(4, 1) X(4, 2) X(4, 3) X(4, 4) X(4, 5) \
    X(5, 1) X(5, 2) X(5, 3) X(5, 4) X(5, 5)
#define EBS_DECL(kw, ka) \
    template <> int launch_tiled_pair<kw, ka, 0>(const ConvArgs &a, int v, int kind); \
    template <> int launch_tiled_pair<kw, ka, 3>(const ConvArgs &a, int v, int kind);
EBS_PAIRS(EBS_DECL)
#undef EBS_DECL

// Order must match EBS_TILED_VARIANTS in conv_tiled_kernel.h.
static const char *const kNames[] = {
    "p4.tile64.ch2", "p4.tile64.ch1", "p4.tile64.ch4",
    "p4.tile32.ch2", "p4.tile32.ch1", "p4.tile32.ch4",
    "k4.tile64.ch2", "k4.tile64.ch1", "k4.tile64.ch4",
    "k4.tile32.ch2", "k4.tile32.ch1", "k4.tile32.ch4",
    "k4.tile16.ch2", "k4.tile16.ch1", "k4.tile16.ch4",
    "r4.tile64.ch4", "r4.tile32.ch4", "r4.tile16.ch4",
    "k4.wide.ch2", "k4.wide.ch1", "k4.wide.ch4",
    "lane.big", "lane.small",
    "pair",
    "lane.split",
};
static constexpr int kNumVariants = sizeof(kNames) / sizeof(kNames[0]);
enum { V_P4_64 = 0, V_P4_32 = 3, V_K4_64 = 6, V_K4_32 = 9, V_K4_16 = 12, V_R4_64 = 15, V_R4_32 = 16, V_R4_16 = 17, V_K4_WIDE = 18, V_LANE = 21, V_PAIR = 23, V_LANE_SPLIT = 24 };

int conv_tiled_variant_count() { return kNumVariants; }
const char *conv_tiled_variant_name(int v) { return (v >= 0 && v < kNumVariants) ? kNames[v] : "invalid"; }

// kind 0 = plain convolution, 1 = re-quantising, 2 = plane pairs
template <int FS>
static int run_pair(const ConvArgs &a, int v, int kind)
{
#define EBS_CASE(kw, ka) case (kw) * 8 + (ka): return launch_tiled_pair<kw, ka, FS>(a, v, kind);
    switch (a.kw * 8 + a.ka) { EBS_PAIRS(EBS_CASE) }
#undef EBS_CASE
    return EBS_ERR_BITWIDTH;
}

template <int FS>
static int run_fs(const ConvArgs &a, int v)
{
    return run_pair<FS>(a, v, 0);
}

int launch_conv_lane(const ConvArgs &a, int sel);
int lane_run_length(int kw, int ka, int stride, int fs, int sel);

static int run_variant(const ConvArgs &a, int v)
{
    if (v < 0 || v >= kNumVariants) return EBS_ERR_UNSUPPORTED;
    if (v == V_PAIR) return launch_conv_pair(a);
    if (v == V_LANE_SPLIT) return launch_conv_lane(a, 2);
    if (v >= V_LANE) return launch_conv_lane(a, v - V_LANE);
    if (a.R == 3 && a.S == 3) return run_fs<3>(a, v);     // unrolled 3x3 taps
    return run_fs<0>(a, v);
}

template <int FS>
static int run_req_fs(const ConvArgs &a, int v)
{
    return run_pair<FS>(a, v, 1);
}

template <int FS>
static int run_planes_fs(const ConvArgs &a, int v)
{
    return run_pair<FS>(a, v, 2);
}

// Stage 1 of the two-stage form: four-word chunks when the words per position allow, else single words.
int launch_planes_tiled(const ConvArgs &a)
{
    const int order[2] = {a.cw % 4 == 0 ? 1 : 0, 0};
    for (int i = 0; i < 2; ++i) {
        int rc = (a.R == 3 && a.S == 3) ? run_planes_fs<3>(a, order[i]) : run_planes_fs<0>(a, order[i]);
        if (rc != EBS_ERR_UNSUPPORTED) return rc;
    }
    return EBS_ERR_UNSUPPORTED;
}

// Slot of the chunk size inside a family of three: order ch2, ch1, ch4.
static int ch_slot(int cw) { return cw % 4 == 0 ? 2 : (cw % 2 == 0 ? 0 : 1); }

// Channels per wave of the (budget, bitwidths) tiles; mirrors TileOf / TileSel in the kernel header.
static int kt_of(int budget, int kw, int ka)
{
    static const int k64[9] = {16, 8, 8, 8, 4, 4, 4, 4, 4}, k32[9] = {16, 8, 8, 8, 4, 4, 4, 4, 4}, k16[9] = {16, 8, 4, 4, 4, 4, 4, 4, 4};
    if (ka == 5 && budget != 64) return kw <= 3 ? 8 : 4;
    const int *t = budget == 64 ? k64 : budget == 32 ? k32 : k16;
    return t[kw + ka - 2];
}

// Whether (and with which run length first) the channel-per-lane kernel should take the layer: -1 = no, else the
// preferred run selection (0 = large, 1 = small); the other one is the second choice.
static int lane_choice(const ConvArgs &a)
{
    const long long positions = (long long)a.N * a.OH * a.OW;
    const int rs = a.R * a.S;
    // Channel-per-lane kernel (3x3 filters): no LDS, scalar position arithmetic, direct 256-byte stores.  It wins
    // where the per-work-group costs of the tiled kernel weigh most - few plane pairs (short kernels), short
    // reductions - and loses on the deepest stride-1 layer (few positions: too few tiles), at the highest
    // bitwidths of the layers with many positions, and when many of a wave's 64 channel lanes would idle.
    // Measured on the ResNet-18 shapes, all 16 pairs, both kernels forced in turn.
    if (rs == 9 && a.R == 3 && a.kw <= 4 && a.ka <= 4 && (a.cw & 1) == 0 && (a.K % 64 == 0 || a.K >= 256)) {
        const int pairs = a.kw * a.ka;
        bool use = false;
        if (positions >= 8192) {
            if (a.stride == 1)
                use = pairs <= 4 || (pairs <= 9 && !(a.ka == 4 && a.kw >= 3)) || positions < 16384;
            else
                use = pairs <= 8;
        } else if (positions >= 3072 && a.stride == 2) {
            use = pairs <= 6;
        }
        // re-quantising: the tiled kernels own 8 instead of 4 channels per lane there, which costs them 8-14 % at
        // the highest bitwidths; the lane kernel pays 2-3 % for its epilogue (measured: (4,4) -4..-6 % on 128 @28x28,
        // 64->128 @56x56 s2, 256->512 @14x14 s2; stride 2 at (3,3)/(4,3) -2..-5 %; (3,4) +-3 %, left alone)
        if (a.next && positions >= 3072 && (pairs == 16 || (a.stride == 2 && a.ka == 3 && a.kw >= 3))) use = true;
        // (signed weights cost the tiled kernels another 8 % there: (3,4) on 128 @28x28 156 vs 167 us; stride 2: equal)
        if (a.next && a.wtop && positions >= 3072 && a.stride == 1) use = true;
        if (use) {
            // small runs where the large ones leave fewer than six tiles per SIMD and divide the row
            const int big = lane_run_length(a.kw, a.ka, a.stride, a.R, 0), small = lane_run_length(a.kw, a.ka, a.stride, a.R, 1);
            int sel = 0;
            if (big > 0 && small > 0 && a.OW >= big) {
                const long long tiles_big = (long long)a.N * a.OH * ((a.OW + big - 1) / big) * ((a.K + 63) / 64);
                if (tiles_big < 6 * 1024 && small < big && a.OW % small == 0) sel = 1;
            } else {
                sel = 1;
            }
            // the last run of a row is moved left and recomputes the overlap: not where that is over 15 % of the work
            const int run = sel ? small : big;
            if (run > 0 && (long long)((a.OW + run - 1) / run) * run * 100 <= (long long)a.OW * 115) {
                return sel;
            }
        }
    }
    // 1x1 filters: the same kernel with the short runs (the long ones were slower on every shape tried) wherever
    // the reduction has at least eight words, and at nine plane pairs on shorter ones; layers with a short
    // reduction and fewer pairs are bound by their output writes and do as well or better with the wide tiles.
    // Measured on the ResNet-50 bottleneck shapes at (2,4), (3,3), (4,2): -3..-10 % (256->64 @56x56), -10 %
    // (1024->256 @14x14), -7..-10 % (256->1024 @14x14), -17 % (64->256 @56x56 at (3,3)).
    // Layers with fewer positions as long as the rows hold a run: 512->2048 @7x7 16.3 / 54.6 / 92.0 us at (1,1) /
    // (3,3) / (4,4) against 23.6 / 63.8 / 102.2 us of the best tiling.
    if (rs == 1 && a.kw <= 4 && a.ka <= 4 && !a.wtop && (a.cw & 1) == 0 && a.K % 64 == 0 && (a.cw >= 8 || a.kw * a.ka >= 8)) {
        const int run = lane_run_length(a.kw, a.ka, a.stride, 1, 1);
        if (positions >= 8192 ||
            (positions >= 2048 && run > 0 && a.OW >= run && (long long)((a.OW + run - 1) / run) * run * 100 <= (long long)a.OW * 115))
            return 1;
    }
    // One output position per image (a fully-connected layer): runs of images, the reduction split among the
    // four waves of a work-group.  Measured on 2048 -> 1000 at batch 1024 against the best tiling: 61.7 vs 75 us
    // at (4,4), 39.7 vs 51 at (3,3), 22 vs 33 at (2,2), 24 vs 33 at (1,4), 20.9 vs 31 at (4,1), 14.4 vs 18.5 at (1,1);
    // 4096 -> 4096 at batch 128: 21.4 vs 41.3 us at (2,2), 62.7 vs 91.2 at (4,4).
    if (rs == 1 && a.OH == 1 && a.OW == 1 && !a.next && a.kw <= 4 && a.ka <= 4 && !a.wtop && (a.cw & 7) == 0 &&
        a.cw <= 256 && a.N >= 64 && (long long)((a.K + 63) / 64) * 64 * 100 <= (long long)a.K * 115) {
        // runs of 8 images for one-bit activations (little arithmetic per step), else 4 (8 were 7-33 % slower)
        return a.ka == 1 ? 0 : 1;
    }
    return -1;
}

// Channel-per-lane kernel with the reduction split among the four waves of a work-group: 3x3 layers with few
// positions and at least 256 input channels, where a wave of the unsplit kernel is one long chain of dependent
// steps.  Measured on the ResNet-18 shapes against the choice below it: 512 @7x7 -3..-9 % up to six plane pairs
// and at (3,3), +-1 % at eight and sixteen; 256->512 @14x14 stride 2 -7..-9 % with one- or two-bit activations
// (runs of seven positions; equal at (1,1)).
static bool split_choice(const ConvArgs &a)
{
    const long long positions = (long long)a.N * a.OH * a.OW;
    const int pairs = a.kw * a.ka;
    if ((a.wtop && a.R != 3) || a.R != a.S || (a.R != 3 && a.R != 1) || a.kw > 4 || a.ka > 4 || (a.cw & 7) || a.R * a.cw > 256)
        return false;
    if (positions < 2048 || (a.K % 64 != 0 && a.K < 256)) return false;
    const int run = lane_run_length(a.kw, a.ka, a.stride, a.R, a.stride == 1 ? 1 : 0);
    if (run <= 0 || a.OW < run || (long long)((a.OW + run - 1) / run) * run * 100 > (long long)a.OW * 115) return false;
    // only where the unsplit kernel would have at most four waves per SIMD (3584 on the layers above; with 7168
    // or 14336 - 256 @14x14, 1x1 1024->256 @14x14, 1x1 512->2048 @7x7 - the unsplit kernel is faster)
    if ((long long)a.N * a.OH * ((a.OW + run - 1) / run) * ((a.K + 63) / 64) > 4096) return false;
    // 1x1 filters (stride 1): 2048->512 @7x7 15.7 / 28.3 / 54.4 / 91.2 us at (1,1) / (2,2) / (3,3) / (4,4) against
    // 30.1 / 40.9 / 71.4 / 114.7 us of the best tiling (unsplit channel-per-lane kernel: 16.8 / 33.6 / 64.1 / 105.8)
    if (a.R == 1) return a.stride == 1;
    // (re-quantising: the tiled kernels that split the reduction are slower than their plain forms, 230 vs 199 us
    // on 512 @7x7 at (4,4), so there all pairs)
    if (a.stride == 1) return a.next || pairs <= 6 || pairs == 9;
    // (three- and four-bit activations: runs of four and three positions that cover the row exactly; 256->512 @14x14
    // stride 2: -4 % at (1,4) and (2,4), -9 % at (2,3), -7 % at (3,3) against the next best kernel, +1 % at (4,4);
    // at (1,3) the unsplit kernel is 2 % faster)
    if (a.stride == 2) return a.ka <= 2 ? pairs >= 2 : (pairs >= 4 && pairs < 16);
    return false;
}

// Fused re-quantisation: the K4 kernels whose work-groups own whole 32-channel words; layers with few
// positions and a long reduction split the reduction among the waves instead (work-groups of 8 channels).
int launch_requant_tiled(const ConvArgs &a)
{
    const long long positions = (long long)a.N * a.OH * a.OW;
    const int rs = a.R * a.S;
    // 3x3 layers with at most 16 input channels: two taps per word
    {
        const int rc = launch_conv_pair(a);
        if (rc != EBS_ERR_UNSUPPORTED) return rc;
    }
    // the channel-per-lane kernel where the plain convolution would use it
    if (split_choice(a)) {
        const int rc = launch_conv_lane(a, 2);
        if (rc != EBS_ERR_UNSUPPORTED) return rc;
    }
    {
        const int sel = lane_choice(a);
        if (sel >= 0) {
            int rc = launch_conv_lane(a, sel);
            if (rc == EBS_ERR_UNSUPPORTED) rc = launch_conv_lane(a, 1 - sel);
            if (rc != EBS_ERR_UNSUPPORTED) return rc;
        }
    }
    int order[4];
    int n = 0;
    if ((rs > 1 || a.kw * a.ka <= 2) && rs * a.cw >= 64 && positions <= 16384 && a.cw % 4 == 0) order[n++] = 3;
    if (a.K < 32) order[n++] = a.cw % 2 == 0 ? 4 : 5;  // 32-channel work-groups would be mostly idle
    order[n++] = ch_slot(a.cw);       // preferred chunk size
    order[n++] = 1;                   // single-word chunks: the smallest footprint
    for (int i = 0; i < n; ++i) {
        int rc = (a.R == 3 && a.S == 3) ? run_req_fs<3>(a, order[i]) : run_req_fs<0>(a, order[i]);
        if (rc != EBS_ERR_UNSUPPORTED) return rc;
    }
    return EBS_ERR_UNSUPPORTED;
}

int launch_conv_tiled(const ConvArgs &a, int variant)
{
    if (variant >= 0) return run_variant(a, variant);
    // Shape heuristic, from sweeps over ResNet-shaped layers on MI355X: small register tiles
    // win (more, shorter work-groups balance the 1024 SIMDs and hide latency); the four waves
    // of a work-group share one staged position tile and take four channel tiles (K4) when the
    // layer has that many channels, and split the reduction (R4) when there are few output
    // positions and a long reduction.
    const long long positions = (long long)a.N * a.OH * a.OW;
    const int slot = ch_slot(a.cw);
    const int rs = a.R * a.S;
    int order[14];
    int n = 0;
    // 3x3 layers with at most 16 input channels: two taps per word (half the AND + bitcount work of the
    // one-tap-per-word kernels, whose words are half zeros there)
    if (a.C <= 16 && rs == 9 && a.R == 3 && a.K <= 32) order[n++] = V_PAIR;
    if (split_choice(a)) order[n++] = V_LANE_SPLIT;
    {
        const int sel = lane_choice(a);
        if (sel >= 0) {
            order[n++] = V_LANE + sel;
            order[n++] = V_LANE + 1 - sel;
        }
    }
    // reduction split: 8 channels per wave for one-bit weights with 3-4 bit activations (4 would leave too
    // little arithmetic per step), else the 16-register tiles
    // (1x1 filters: only at one or two plane pairs; with more, the channel split is faster)
    if ((rs > 1 || a.kw * a.ka <= 2) && rs * a.cw >= 64 && positions <= 16384 && a.cw % 4 == 0)
        order[n++] = (a.kw == 1 && (a.ka == 3 || a.ka == 4)) ? V_R4_32 : V_R4_16;
    // 1x1 layers with at most 8 reduction words per output are bound by their output writes: wide tiles
    // (32-channel pieces of each output row) up to 8 plane pairs; measured -15 % on 64->256 @56x56, -2..4 % on 256->64
    if (rs == 1 && a.cw <= 8 && a.kw * a.ka <= 8 && a.K >= 32) order[n++] = V_K4_WIDE + slot;
    // channel split: the 16-register tiles (interleaved sweeps: never slower than the 32-register ones)
    // (one-bit weights with 3-4 bit activations: little arithmetic per staged byte, so half-size chunks - twice
    // the resident work-groups - are faster: 26 vs 45 us on 128->256 @28x28 stride 2 at (1,3))
    const int kslot = (a.kw == 1 && a.ka >= 3 && a.cw % 4 == 0) ? 0 : slot;
    if (a.K >= 4 * kt_of(16, a.kw, a.ka)) order[n++] = V_K4_16 + kslot;
    order[n++] = V_P4_32 + slot;
    order[n++] = V_P4_32 + 1;       // ch1: smallest staging footprint
    for (int i = 0; i < n; ++i) {
        int rc = run_variant(a, order[i]);
        if (rc != EBS_ERR_UNSUPPORTED) return rc;
    }
    return EBS_ERR_UNSUPPORTED;
}

}  // namespace ebs
