// Dispatch of the channel-per-lane convolution (kernels: conv_lane_kernel.h, instantiated per (k_w, k_a)
// pair from conv_lane_inst.hip).
#include "ebs_internal.h"

namespace ebs {

template <int KW, int KA> int launch_lane_pair(const ConvArgs &a, int sel);
#define EBS_LANE_PAIRS(X) \
    X(1, 1) X(1, 2) X(1, 3) X(1, 4) X(2, 1) X(2, 2) X(2, 3) X(2, 4) \
    X(3, 1) X(3, 2) X(3, 3) X(3, 4) X(4, 1) X(4, 2) X(4, 3) X(4, 4)
#define EBS_DECL(kw, ka) template <> int launch_lane_pair<kw, ka>(const ConvArgs &a, int sel);
EBS_LANE_PAIRS(EBS_DECL)
#undef EBS_DECL

// sel: 0 = large runs of positions, 1 = small runs.
// EBS_ERR_UNSUPPORTED for anything but 3x3 (pad <= 1) and 1x1 filters, stride 1 or 2, bitwidths up to 4, an even
// number of (filter row, 32-channel word) steps up to 64, unsigned weights, and output rows at least one run long.
// 1x1 layers with one output position per image (fully-connected layers) run over 8 (sel 0) or 4 images instead.
int launch_conv_lane(const ConvArgs &a, int sel)
{
#define EBS_CASE(kw, ka) case (kw) * 8 + (ka): return launch_lane_pair<kw, ka>(a, sel);
    switch (a.kw * 8 + a.ka) { EBS_LANE_PAIRS(EBS_CASE) }
#undef EBS_CASE
    return EBS_ERR_UNSUPPORTED;
}

// Positions per run of the (k_w, k_a, stride, filter size) kernels; mirrors LaneRun in conv_lane_kernel.h.
// 0 = no kernel.
int lane_run_length(int kw, int ka, int stride, int fs, int sel)
{
    if (kw < 1 || kw > 4 || ka < 1 || ka > 4 || (fs != 1 && fs != 3)) return 0;
    const int ncls = kw + ka - 1;
    if (stride == 1) return sel == 0 ? ((ka <= 2 && ncls <= 4) ? 14 : 7) : 7;
    if (stride == 2) return sel == 0 ? (ka <= 2 ? 7 : 4) : 4;
    return 0;
}

}  // namespace ebs
