// Variant table and shape heuristic of the tiled convolution; the kernels are
// instantiated per weight bitwidth in conv_tiled_kw*.hip.
#include "ebs_internal.h"

namespace ebs {

template <int KW> int launch_tiled_kw(const ConvArgs &a, int v);
template <> int launch_tiled_kw<1>(const ConvArgs &a, int v);
template <> int launch_tiled_kw<2>(const ConvArgs &a, int v);
template <> int launch_tiled_kw<3>(const ConvArgs &a, int v);
template <> int launch_tiled_kw<4>(const ConvArgs &a, int v);

static const char *const kNames[] = {
    "p4.tile128.ch2", "p4.tile128.ch1", "p4.tile128.ch4",
    "p4.tile64.ch2", "p4.tile64.ch1", "p4.tile64.ch4",
    "p4.tile32.ch2", "p4.tile32.ch1", "p4.tile32.ch4",
    "k4.tile128.ch2", "k4.tile128.ch1", "k4.tile128.ch4",
    "k4.tile64.ch2", "k4.tile64.ch1", "k4.tile64.ch4",
    "k4.tile32.ch2", "k4.tile32.ch1", "k4.tile32.ch4",
    "r4.tile128.ch4", "r4.tile64.ch4", "r4.tile32.ch4",
};
static constexpr int kNumVariants = sizeof(kNames) / sizeof(kNames[0]);

int conv_tiled_variant_count() { return kNumVariants; }
const char *conv_tiled_variant_name(int v) { return (v >= 0 && v < kNumVariants) ? kNames[v] : "invalid"; }

static int run_variant(const ConvArgs &a, int v)
{
    if (v < 0 || v >= kNumVariants) return EBS_ERR_UNSUPPORTED;
    switch (a.kw) {
        case 1: return launch_tiled_kw<1>(a, v);
        case 2: return launch_tiled_kw<2>(a, v);
        case 3: return launch_tiled_kw<3>(a, v);
        case 4: return launch_tiled_kw<4>(a, v);
    }
    return EBS_ERR_BITWIDTH;
}

// Index of the variant with this chunk size inside a budget family (order ch2, ch1, ch4).
static int ch_index(int cw) { return cw >= 4 ? 2 : (cw >= 2 ? 0 : 1); }

int launch_conv_tiled(const ConvArgs &a, int variant)
{
    if (variant >= 0) return run_variant(a, variant);
    // Heuristic: few outputs with a long reduction -> split the reduction among the waves;
    // otherwise the 64-register tile, falling back to smaller staging footprints.
    long long outputs = (long long)a.N * a.OH * a.OW * a.K;
    int order[5];
    int n = 0;
    if (outputs < (1 << 22) && a.cw >= 4) order[n++] = 19;
    order[n++] = 3 + ch_index(a.cw);
    order[n++] = 6 + ch_index(a.cw);
    order[n++] = 7;
    for (int i = 0; i < n; ++i) {
        int rc = run_variant(a, order[i]);
        if (rc != EBS_ERR_UNSUPPORTED) return rc;
    }
    return EBS_ERR_UNSUPPORTED;
}

}  // namespace ebs
