// Tiled convolution kernels of ONE (k_w, k_a, filter specialisation) triple: every variant of the plain,
// re-quantising and plane-pair kernels.  The build compiles this file once per triple with
// -DEBS_KW=<1..5> -DEBS_KA=<1..5> -DEBS_FS=<0|3>, so that the instantiations spread over many parallel jobs.
#include "conv_tiled_kernel.h"
#if !defined(EBS_KW) || !defined(EBS_KA) || !defined(EBS_FS)
#error "compile with -DEBS_KW=.. -DEBS_KA=.. -DEBS_FS=.. (paper_2003_07577_amd/build.py does)"
#endif
namespace ebs {
EBS_DEFINE_TILED_PAIR(EBS_KW, EBS_KA, EBS_FS)
}
