// Tiled convolution kernels for 1-bit weights (all activation bitwidths, all variants).
#include "conv_tiled_kernel.h"
namespace ebs {
EBS_DEFINE_TILED_KW(1)
}
