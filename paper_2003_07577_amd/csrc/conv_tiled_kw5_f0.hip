// Tiled convolution kernels: 5-bit weights, generic filter (all activation bitwidths, the heuristic's variants).
#include "conv_tiled_kernel.h"
namespace ebs {
EBS_DEFINE_TILED_KW(5, 0)
}
