// Tiled convolution kernels: 4-bit weights, 3x3 filter specialisation (all activation bitwidths, all variants).
#include "conv_tiled_kernel.h"
namespace ebs {
EBS_DEFINE_TILED_KW(4, 3)
}
