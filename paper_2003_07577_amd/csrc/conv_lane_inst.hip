// Channel-per-lane convolution kernels of ONE (k_w, k_a) pair (both strides, both run lengths).  The build
// compiles this file once per pair with -DEBS_KW=<1..4> -DEBS_KA=<1..4>.
#include "conv_lane_kernel.h"
#if !defined(EBS_KW) || !defined(EBS_KA)
#error "compile with -DEBS_KW=.. -DEBS_KA=.. (paper_2003_07577_amd/build.py does)"
#endif
namespace ebs {
EBS_DEFINE_LANE_PAIR(EBS_KW, EBS_KA)
}
