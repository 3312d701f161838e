// Internal declarations shared by the translation units of libebs (host side).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "ebs.h"

namespace ebs {

// Weight words are grouped by 16 output channels so that one reduction step of
// a channel tile is one contiguous run of words (see pack.hip).
constexpr int kWgtGroup = 16;

// Largest bitwidth of weights and activations: the search space of the paper is {1, ..., 5}
// (Sec. 5, implementation details).
constexpr int kMaxBits = 5;
// Candidate bitwidths of one aggregated quantisation function (Sec. 4.1); the paper searches five.
constexpr int kMaxCandidates = EBS_MAX_CANDIDATES;

struct ConvArgs {
    const uint32_t *act;   // packed activations  [cw][N][H+2][W+2][k_a], zero border of one position
    const uint32_t *wgt;   // packed weights      [ceil(K/16)][R*S][cw][16][k_w]
    int N, C, H, W, K, R, S, stride, pad, OH, OW, cw, kw, ka;
    const float *scale;
    const float *offset;   // may be null
    int per_channel;
    int32_t *acc;          // [N*OH*OW][K]
    float *out;            // may be null
    hipStream_t stream;
    // fused re-quantisation (next != null): instead of acc/out the kernel writes the NEXT layer's
    // packed activations [ceil(K/32)][N][OH+2][OW+2][k_next]; the zero ring is written first
    uint32_t *next;
    float alpha;           // clip of the next layer's activation quantiser
    int k_next;            // its bitwidth
    // signed weights (Eq. 1a): 0 = unsigned levels; otherwise 2^k_w - 1, and the kernels return
    // 2*sum(q*a) - wtop*sum(a), the product with the integer weights 2q - (2^k_w - 1)
    int wtop;
};

inline int words_per_pixel(int C) { return (C + 31) / 32; }

// Packed activations carry a zero border of this many positions on every side
// of each image, so that a 3x3 / pad-1 filter tap never leaves the buffer and
// needs no bounds check.
constexpr int kActBorder = 1;
// Slack dwords after the last position so that vector loads of a few words may
// run past the end of the last position.
constexpr int kActTailDwords = 4;

// 3x3 layers with at most 16 input channels: the packed weights end with a section that holds two taps per
// word, ceil16(K) * 5 * k_w dwords (conv_pair_kernel.h)
inline bool has_pair_section(int C, int R, int S) { return C <= 16 && R == 3 && S == 3; }
int launch_conv_pair(const ConvArgs &a);         // EBS_ERR_UNSUPPORTED when the shape is not the pair kernel's

int launch_conv_naive(const ConvArgs &a);
int launch_requant_naive(const ConvArgs &a);
int launch_zero_border(uint32_t *packed, int N, int H, int W, int words, int planes, hipStream_t st);
// Returns EBS_ERR_UNSUPPORTED when the tiling cannot run this shape.
int launch_conv_tiled(const ConvArgs &a, int variant);
int launch_requant_tiled(const ConvArgs &a);
// Two-stage form (Sec. 4.3): stage 1 writes the k_w*k_a partial-product planes where a.acc
// points ([m*k_a + k][N*OH*OW][K], int32); stage 2 recombines them (Eq. 14) and applies scale/offset.
int launch_planes_tiled(const ConvArgs &a);      // EBS_ERR_UNSUPPORTED when the tiling cannot run the shape
int launch_planes_naive(const ConvArgs &a);
int launch_pow2_depthwise(const int32_t *planes, long long plane_elems, int K, int kw, int ka, const float *scale,
                          const float *offset, int per_channel, int32_t *acc, float *out, hipStream_t st);
// Quantisers and aggregated quantisation functions (quantize.hip); workspace: 256 device bytes.
int quantize_weights(const float *w, size_t count, int bits, uint8_t *levels, void *workspace, hipStream_t st);
int quantize_weights_static(const float *w, size_t count, int bits, uint8_t *levels, hipStream_t st);
int quantize_activations(const float *x, size_t count, float alpha, int bits, uint8_t *levels, hipStream_t st);
int aggregate_weights(const float *w, size_t count, const int *bits, int n, const float *strengths, const float *gumbel,
                      float tau, float *out, void *workspace, hipStream_t st);
int aggregate_activations(const float *x, size_t count, float alpha, const int *bits, int n, const float *strengths,
                          const float *gumbel, float tau, float *out, void *workspace, hipStream_t st);
int conv_tiled_variant_count();
const char *conv_tiled_variant_name(int variant);

// What the launch heuristics assume of the current device, read from the runtime once per device.
// nullptr: the runtime gave no device (the error is in last_hip_error()).
struct DeviceShape {
    int cus;            // compute units
    bool gfx950;        // the architecture these kernels are written and tuned for
};
const DeviceShape *device_shape();

// Last HIP error this thread's library calls have seen (hipSuccess if none).
hipError_t &last_hip_error();
inline int hip_ok(hipError_t e)
{
    if (e == hipSuccess) return EBS_OK;
    last_hip_error() = e;
    return EBS_ERR_HIP;
}

}  // namespace ebs
