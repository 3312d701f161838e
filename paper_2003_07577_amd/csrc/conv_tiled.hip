#include "ebs_internal.h"
namespace ebs {
int launch_conv_tiled(const ConvArgs &, int) { return EBS_ERR_UNSUPPORTED; }
int conv_tiled_variant_count() { return 0; }
const char *conv_tiled_variant_name(int) { return "invalid"; }
}
