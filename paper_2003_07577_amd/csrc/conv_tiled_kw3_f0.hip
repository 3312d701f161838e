// Tiled convolution kernels: 3-bit weights, generic filter (all activation bitwidths, all variants).
#include "conv_tiled_kernel.h"
namespace ebs {
EBS_DEFINE_TILED_KW(3, 0)
}
