// Dispatch of the two-taps-per-word convolution for 3x3 layers with at most 16 input channels
// (kernels: conv_pair_kernel.h, instantiated per (k_w, k_a) pair from conv_pair_inst.hip).
#include "ebs_internal.h"

namespace ebs {

template <int KW, int KA> int launch_pair_pair(const ConvArgs &a);
#define EBS_PAIR_PAIRS(X)                                            \
    X(1, 1) X(1, 2) X(1, 3) X(1, 4) X(1, 5) X(2, 1) X(2, 2) X(2, 3) X(2, 4) X(2, 5) \
    X(3, 1) X(3, 2) X(3, 3) X(3, 4) X(3, 5) X(4, 1) X(4, 2) X(4, 3) X(4, 4) X(4, 5) \
    X(5, 1) X(5, 2) X(5, 3) X(5, 4) X(5, 5)
#define EBS_DECL(kw, ka) template <> int launch_pair_pair<kw, ka>(const ConvArgs &a);
EBS_PAIR_PAIRS(EBS_DECL)
#undef EBS_DECL

// Plain convolution (a.next == null) or the fused re-quantising form.  EBS_ERR_UNSUPPORTED for anything but
// 3x3 filters with pad <= 1 and stride 1 or 2 on at most 16 input and 32 output channels.
int launch_conv_pair(const ConvArgs &a)
{
#define EBS_CASE(kw, ka) case (kw) * 8 + (ka): return launch_pair_pair<kw, ka>(a);
    switch (a.kw * 8 + a.ka) { EBS_PAIR_PAIRS(EBS_CASE) }
#undef EBS_CASE
    return EBS_ERR_UNSUPPORTED;
}

}  // namespace ebs
