// Two-taps-per-word convolution kernels of ONE (k_w, k_a) pair (16 and 32 channel lanes, plain and
// re-quantising).  The build compiles this file once per pair with -DEBS_KW=<1..5> -DEBS_KA=<1..5>.
#include "conv_pair_kernel.h"
#if !defined(EBS_KW) || !defined(EBS_KA)
#error "compile with -DEBS_KW=.. -DEBS_KA=.. (paper_2003_07577_amd/build.py does)"
#endif
namespace ebs {
EBS_DEFINE_PAIR_PAIR(EBS_KW, EBS_KA)
}
