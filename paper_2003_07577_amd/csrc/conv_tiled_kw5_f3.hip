// Tiled convolution kernels: 5-bit weights, 3x3 filter specialisation (all activation bitwidths, the heuristic's variants).
#include "conv_tiled_kernel.h"
namespace ebs {
EBS_DEFINE_TILED_KW(5, 3)
}
