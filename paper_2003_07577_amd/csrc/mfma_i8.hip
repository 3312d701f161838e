#include "ebs_internal.h"
namespace ebs {
int launch_conv_mfma_i8(const uint8_t *, const uint8_t *, const ConvArgs &) { return EBS_ERR_UNSUPPORTED; }
}
