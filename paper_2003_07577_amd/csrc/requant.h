// Activation quantiser of the next layer (paper Eq. 1b-1c: clip to [0, alpha] - the clip at 0 is the
// ReLU -, normalise, round half up to b bits) applied to an affine output x = scale*acc + offset.
// A rounding decides an integer level, so the order of the single-precision operations is fixed:
//   x = fmaf((float)acc, scale, offset); z = min(max(x, 0), alpha); level = floor(fmaf(z, qs, 0.5))
// with qs = (float)(2^b - 1) / alpha evaluated once on the host (one IEEE division).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ebs {

inline float requant_qs(float alpha, int bits) { return (float)((1 << bits) - 1) / alpha; }

__device__ __forceinline__ uint32_t requant_level(int32_t acc, float scale, float offset, float alpha, float qs)
{
    const float x = fmaf((float)acc, scale, offset);
    const float z = fminf(fmaxf(x, 0.0f), alpha);
    return (uint32_t)(int)floorf(fmaf(z, qs, 0.5f));
}

}  // namespace ebs
