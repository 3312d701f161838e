// C-ABI entry points of libebs: argument validation and kernel dispatch.
// Everything behind these calls runs in the library's own HIP kernels.
#include "ebs_internal.h"

#include <cstring>
#include <mutex>

namespace ebs {
int pack_activations(const uint8_t *levels, uint32_t *packed, int N, int H, int W, int C, int bits, hipStream_t st);
int pack_weights(const uint8_t *levels, uint32_t *packed, int K, int C, int R, int S, int bits, hipStream_t st);
int check_levels(const uint8_t *levels, size_t count, int bits, int32_t *flag, hipStream_t st);
int launch_conv_mfma_i8(const uint8_t *act, const uint8_t *wgt, const ConvArgs &a);

hipError_t &last_hip_error()
{
    static thread_local hipError_t e = hipSuccess;
    return e;
}

const DeviceShape *device_shape()
{
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static DeviceShape shapes[kMaxDevices];
    static bool known[kMaxDevices];
    int dev = 0;
    if (hip_ok(hipGetDevice(&dev))) return nullptr;
    if (dev < 0 || dev >= kMaxDevices) {
        last_hip_error() = hipErrorInvalidDevice;
        return nullptr;
    }
    std::lock_guard<std::mutex> lock(mu);
    if (!known[dev]) {
        hipDeviceProp_t prop;
        if (hip_ok(hipGetDeviceProperties(&prop, dev))) return nullptr;
        shapes[dev].cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 1;
        shapes[dev].gfx950 = std::strncmp(prop.gcnArchName, "gfx950", 6) == 0;
        known[dev] = true;
    }
    return &shapes[dev];
}

static const long long kMaxElems = (1LL << 31) - 1;

static bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
static bool bits_ok(int b) { return b >= 1 && b <= kMaxBits; }

static int check_act_shape(int N, int H, int W, int C)
{
    if (N <= 0 || H <= 0 || W <= 0 || C <= 0) return EBS_ERR_SHAPE;
    long long pixels = (long long)N * H * W;
    if (pixels > kMaxElems || pixels * C > kMaxElems) return EBS_ERR_SHAPE;
    long long padded = (long long)N * (H + 2 * kActBorder) * (W + 2 * kActBorder);
    if (padded * words_per_pixel(C) * 4 + kActTailDwords > kMaxElems) return EBS_ERR_SHAPE;
    return EBS_OK;
}

static int check_wgt_shape(int K, int C, int R, int S)
{
    if (K <= 0 || C <= 0 || R <= 0 || S <= 0) return EBS_ERR_SHAPE;
    long long kpad = ((long long)K + kWgtGroup - 1) / kWgtGroup * kWgtGroup;
    if ((long long)K * R * S * C > kMaxElems) return EBS_ERR_SHAPE;
    if (kpad * R * S * words_per_pixel(C) * 4 > kMaxElems) return EBS_ERR_SHAPE;
    return EBS_OK;
}

// Validates a convolution request and fills the geometry fields.
static int check_conv(ConvArgs &a, const void *p0, const void *p1, bool need_scale = true)
{
    if (!p0 || !p1 || (need_scale && !a.scale) || (!a.acc && !a.next)) return EBS_ERR_NULL;
    if (!bits_ok(a.kw) || !bits_ok(a.ka)) return EBS_ERR_BITWIDTH;
    int rc = check_act_shape(a.N, a.H, a.W, a.C);
    if (rc) return rc;
    rc = check_wgt_shape(a.K, a.C, a.R, a.S);
    if (rc) return rc;
    if (a.stride <= 0 || a.pad < 0 || a.pad >= a.R || a.pad >= a.S) return EBS_ERR_SHAPE;
    if (a.H + 2 * a.pad < a.R || a.W + 2 * a.pad < a.S) return EBS_ERR_SHAPE;
    a.OH = (a.H + 2 * a.pad - a.R) / a.stride + 1;
    a.OW = (a.W + 2 * a.pad - a.S) / a.stride + 1;
    a.cw = words_per_pixel(a.C);
    if ((long long)a.N * a.OH * a.OW * a.K > kMaxElems) return EBS_ERR_SHAPE;
    // kernels number output positions in 32 bits and round the last tile up (tiles of at most 1024 positions);
    // check_act_shape already keeps N*(H+2)*(W+2) below 2^29, so this is a second fence, not the first
    if ((long long)a.N * a.OH * a.OW > kMaxElems - 1024) return EBS_ERR_SHAPE;
    // the largest accumulator, C*R*S*(2^k_w - 1)*(2^k_a - 1), must fit an int32
    if ((long long)a.C * a.R * a.S * ((1 << a.kw) - 1) * ((1 << a.ka) - 1) > kMaxElems) return EBS_ERR_SHAPE;
    if (!aligned16(p0) || !aligned16(p1) || !aligned16(a.acc) || (a.out && !aligned16(a.out)) || !aligned16(a.next))
        return EBS_ERR_ALIGN;
    if ((reinterpret_cast<uintptr_t>(a.scale) & 3u) || (a.offset && (reinterpret_cast<uintptr_t>(a.offset) & 3u)))
        return EBS_ERR_ALIGN;
    return EBS_OK;
}

static int run_conv(int variant, ConvArgs &a)
{
    int nt = conv_tiled_variant_count();
    if (variant < 0 || variant > 1 + nt) return EBS_ERR_UNSUPPORTED;
    if (variant == 1) return launch_conv_naive(a);
    if (variant >= 2) return launch_conv_tiled(a, variant - 2);
    int rc = launch_conv_tiled(a, -1);  // heuristic choice among the tiled variants
    if (rc == EBS_ERR_UNSUPPORTED) rc = launch_conv_naive(a);
    return rc;
}

}  // namespace ebs

using namespace ebs;

extern "C" {

int ebs_version(void) { return 211; }

const char *ebs_last_hip_error(void) { return hipGetErrorName(ebs::last_hip_error()); }

const char *ebs_status_string(int s)
{
    switch (s) {
        case EBS_OK: return "EBS_OK";
        case EBS_ERR_NULL: return "EBS_ERR_NULL: required pointer is null";
        case EBS_ERR_BITWIDTH: return "EBS_ERR_BITWIDTH: bitwidth outside [1,5]";
        case EBS_ERR_SHAPE: return "EBS_ERR_SHAPE: invalid or too large shape";
        case EBS_ERR_ALIGN: return "EBS_ERR_ALIGN: buffer not 16-byte aligned";
        case EBS_ERR_UNSUPPORTED: return "EBS_ERR_UNSUPPORTED: no kernel for this request";
        case EBS_ERR_HIP: return "EBS_ERR_HIP: HIP runtime error at launch";
        case EBS_ERR_LEVEL_RANGE: return "EBS_ERR_LEVEL_RANGE: level exceeds bitwidth";
    }
    return "unknown ebs status";
}

size_t ebs_packed_weights_bytes(int K, int C, int R, int S, int k_w)
{
    if (!bits_ok(k_w) || check_wgt_shape(K, C, R, S)) return 0;
    size_t kpad = ((size_t)K + kWgtGroup - 1) / kWgtGroup * kWgtGroup;
    size_t dwords = kpad * R * S * words_per_pixel(C) * k_w;
    if (has_pair_section(C, R, S)) dwords += kpad * 5 * k_w;
    return dwords * sizeof(uint32_t);
}

size_t ebs_packed_activations_bytes(int N, int H, int W, int C, int k_a)
{
    if (!bits_ok(k_a) || check_act_shape(N, H, W, C)) return 0;
    size_t padded = (size_t)N * (H + 2 * kActBorder) * (W + 2 * kActBorder);
    return (padded * words_per_pixel(C) * k_a + kActTailDwords) * sizeof(uint32_t);
}

int ebs_pack_weights(const uint8_t *levels, int K, int C, int R, int S, int k_w, void *packed, void *stream)
{
    if (!levels || !packed) return EBS_ERR_NULL;
    if (!bits_ok(k_w)) return EBS_ERR_BITWIDTH;
    int rc = check_wgt_shape(K, C, R, S);
    if (rc) return rc;
    if (!aligned16(levels) || !aligned16(packed)) return EBS_ERR_ALIGN;
    return pack_weights(levels, (uint32_t *)packed, K, C, R, S, k_w, (hipStream_t)stream);
}

int ebs_pack_activations(const uint8_t *levels, int N, int H, int W, int C, int k_a, void *packed, void *stream)
{
    if (!levels || !packed) return EBS_ERR_NULL;
    if (!bits_ok(k_a)) return EBS_ERR_BITWIDTH;
    int rc = check_act_shape(N, H, W, C);
    if (rc) return rc;
    if (!aligned16(levels) || !aligned16(packed)) return EBS_ERR_ALIGN;
    return pack_activations(levels, (uint32_t *)packed, N, H, W, C, k_a, (hipStream_t)stream);
}

int ebs_conv_variant_count(void) { return 1 + conv_tiled_variant_count(); }

const char *ebs_conv_variant_name(int v)
{
    if (v == 0) return "heuristic";
    if (v == 1) return "naive";
    if (v >= 2 && v < 2 + conv_tiled_variant_count()) return conv_tiled_variant_name(v - 2);
    return "invalid";
}

int ebs_mixed_conv2d_variant(int variant, const void *packed_act, const void *packed_wgt,
                             int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                             int k_w, int k_a, const float *scale, const float *offset, int per_channel,
                             int32_t *acc_out, float *out_f32, void *stream)
{
    ConvArgs a{};
    a.act = (const uint32_t *)packed_act;
    a.wgt = (const uint32_t *)packed_wgt;
    a.N = N; a.C = C; a.H = H; a.W = W; a.K = K; a.R = R; a.S = S;
    a.stride = stride; a.pad = pad; a.kw = k_w; a.ka = k_a;
    a.scale = scale; a.offset = offset; a.per_channel = per_channel ? 1 : 0;
    a.acc = acc_out; a.out = out_f32; a.stream = (hipStream_t)stream;
    int rc = check_conv(a, packed_act, packed_wgt);
    if (rc) return rc;
    return run_conv(variant, a);
}

int ebs_mixed_conv2d(const void *packed_act, const void *packed_wgt,
                     int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                     int k_w, int k_a, const float *scale, const float *offset, int per_channel,
                     int32_t *acc_out, float *out_f32, void *stream)
{
    return ebs_mixed_conv2d_variant(0, packed_act, packed_wgt, N, C, H, W, K, R, S, stride, pad, k_w, k_a,
                                    scale, offset, per_channel, acc_out, out_f32, stream);
}

size_t ebs_partial_products_bytes(int N, int H, int W, int K, int R, int S, int stride, int pad, int k_w, int k_a)
{
    if (!bits_ok(k_w) || !bits_ok(k_a)) return 0;
    if (N <= 0 || H <= 0 || W <= 0 || K <= 0 || R <= 0 || S <= 0 || stride <= 0 || pad < 0) return 0;
    if (pad >= R || pad >= S || H + 2 * pad < R || W + 2 * pad < S) return 0;
    long long OH = (H + 2 * pad - R) / stride + 1, OW = (W + 2 * pad - S) / stride + 1;
    long long elems = (long long)N * OH * OW;
    if (elems > kMaxElems || elems * K > kMaxElems) return 0;
    return (size_t)elems * K * k_w * k_a * sizeof(int32_t);
}

int ebs_binary_conv_planes(const void *packed_act, const void *packed_wgt,
                           int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                           int k_w, int k_a, int32_t *planes, void *stream)
{
    ConvArgs a{};
    a.act = (const uint32_t *)packed_act;
    a.wgt = (const uint32_t *)packed_wgt;
    a.N = N; a.C = C; a.H = H; a.W = W; a.K = K; a.R = R; a.S = S;
    a.stride = stride; a.pad = pad; a.kw = k_w; a.ka = k_a;
    a.acc = planes; a.stream = (hipStream_t)stream;
    int rc = check_conv(a, packed_act, packed_wgt, false);
    if (rc) return rc;
    rc = launch_planes_tiled(a);
    if (rc == EBS_ERR_UNSUPPORTED) rc = launch_planes_naive(a);
    return rc;
}

int ebs_pow2_depthwise(const int32_t *planes, long long positions, int K, int k_w, int k_a,
                       const float *scale, const float *offset, int per_channel,
                       int32_t *acc_out, float *out_f32, void *stream)
{
    if (!planes || !scale || !acc_out) return EBS_ERR_NULL;
    if (!bits_ok(k_w) || !bits_ok(k_a)) return EBS_ERR_BITWIDTH;
    if (positions <= 0 || K <= 0 || positions > kMaxElems || positions * K > kMaxElems) return EBS_ERR_SHAPE;
    if (!aligned16(planes) || !aligned16(acc_out) || (out_f32 && !aligned16(out_f32))) return EBS_ERR_ALIGN;
    if ((reinterpret_cast<uintptr_t>(scale) & 3u) || (offset && (reinterpret_cast<uintptr_t>(offset) & 3u)))
        return EBS_ERR_ALIGN;
    return launch_pow2_depthwise(planes, positions * K, K, k_w, k_a, scale, offset, per_channel ? 1 : 0,
                                 acc_out, out_f32, (hipStream_t)stream);
}

int ebs_mixed_conv2d_mfma_i8(const uint8_t *act_levels, const uint8_t *wgt_levels,
                             int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                             const float *scale, const float *offset, int per_channel,
                             int32_t *acc_out, float *out_f32, void *stream)
{
    ConvArgs a{};
    a.N = N; a.C = C; a.H = H; a.W = W; a.K = K; a.R = R; a.S = S;
    a.stride = stride; a.pad = pad; a.kw = 4; a.ka = 4;
    a.scale = scale; a.offset = offset; a.per_channel = per_channel ? 1 : 0;
    a.acc = acc_out; a.out = out_f32; a.stream = (hipStream_t)stream;
    int rc = check_conv(a, act_levels, wgt_levels);
    if (rc) return rc;
    return launch_conv_mfma_i8(act_levels, wgt_levels, a);
}

int ebs_mixed_conv2d_signed(const void *packed_act, const void *packed_wgt,
                            int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                            int k_w, int k_a, const float *scale, const float *offset, int per_channel,
                            int32_t *acc_out, float *out_f32, void *stream)
{
    ConvArgs a{};
    a.act = (const uint32_t *)packed_act;
    a.wgt = (const uint32_t *)packed_wgt;
    a.N = N; a.C = C; a.H = H; a.W = W; a.K = K; a.R = R; a.S = S;
    a.stride = stride; a.pad = pad; a.kw = k_w; a.ka = k_a;
    a.scale = scale; a.offset = offset; a.per_channel = per_channel ? 1 : 0;
    a.acc = acc_out; a.out = out_f32; a.stream = (hipStream_t)stream;
    int rc = check_conv(a, packed_act, packed_wgt);
    if (rc) return rc;
    a.wtop = (1 << k_w) - 1;
    return run_conv(0, a);
}

int ebs_mixed_conv2d_requant(const void *packed_act, const void *packed_wgt,
                             int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                             int k_w, int k_a, int signed_weights,
                             const float *scale, const float *offset, int per_channel,
                             float alpha_next, int k_next, void *packed_next, void *stream)
{
    if (!packed_next) return EBS_ERR_NULL;
    if (!bits_ok(k_next)) return EBS_ERR_BITWIDTH;
    if (!(alpha_next > 0.0f) || !(alpha_next < 3.0e38f)) return EBS_ERR_SHAPE;
    ConvArgs a{};
    a.act = (const uint32_t *)packed_act;
    a.wgt = (const uint32_t *)packed_wgt;
    a.N = N; a.C = C; a.H = H; a.W = W; a.K = K; a.R = R; a.S = S;
    a.stride = stride; a.pad = pad; a.kw = k_w; a.ka = k_a;
    a.scale = scale; a.offset = offset; a.per_channel = per_channel ? 1 : 0;
    a.next = (uint32_t *)packed_next; a.alpha = alpha_next; a.k_next = k_next;
    a.stream = (hipStream_t)stream;
    int rc = check_conv(a, packed_act, packed_wgt);
    if (rc) return rc;
    rc = check_act_shape(N, a.OH, a.OW, K);          // the next layer's packed tensor must be addressable
    if (rc) return rc;
    a.wtop = signed_weights ? (1 << k_w) - 1 : 0;
    rc = launch_requant_tiled(a);                     // writes the zero ring itself
    if (rc != EBS_ERR_UNSUPPORTED) return rc;
    rc = launch_zero_border(a.next, N, a.OH, a.OW, words_per_pixel(K), k_next, a.stream);
    if (rc) return rc;
    return launch_requant_naive(a);
}

static bool finite_pos(float v) { return v > 0.0f && v < 3.0e38f; }
static int check_elementwise(const void *in, const void *out, size_t count)
{
    if (!in || !out) return EBS_ERR_NULL;
    if (count == 0 || count >= ((size_t)1 << 40)) return EBS_ERR_SHAPE;
    if (!aligned16(in) || !aligned16(out)) return EBS_ERR_ALIGN;
    return EBS_OK;
}
static int check_candidates(const int *bits, int n_bits, const float *strengths, const float *gumbel, float tau)
{
    if (!bits || !strengths) return EBS_ERR_NULL;
    if (n_bits < 1 || n_bits > kMaxCandidates) return EBS_ERR_BITWIDTH;
    for (int i = 0; i < n_bits; ++i)
        if (bits[i] < 1 || bits[i] > 8) return EBS_ERR_BITWIDTH;
    if (gumbel && !finite_pos(tau)) return EBS_ERR_SHAPE;
    return EBS_OK;
}

int ebs_quantize_weights(const float *w, size_t count, int k_w, uint8_t *levels, void *workspace, void *stream)
{
    if (!workspace) return EBS_ERR_NULL;
    int rc = check_elementwise(w, levels, count);
    if (rc) return rc;
    if (k_w < 1 || k_w > 8) return EBS_ERR_BITWIDTH;
    if (!aligned16(workspace)) return EBS_ERR_ALIGN;
    return quantize_weights(w, count, k_w, levels, workspace, (hipStream_t)stream);
}

int ebs_quantize_weights_static(const float *w, size_t count, int k_w, uint8_t *levels, void *stream)
{
    int rc = check_elementwise(w, levels, count);
    if (rc) return rc;
    if (count > (size_t)EBS_STATIC_MAX_COUNT) return EBS_ERR_SHAPE;
    if (k_w < 1 || k_w > 8) return EBS_ERR_BITWIDTH;
    return quantize_weights_static(w, count, k_w, levels, (hipStream_t)stream);
}

int ebs_quantize_activations(const float *x, size_t count, float alpha, int k_a, uint8_t *levels, void *stream)
{
    int rc = check_elementwise(x, levels, count);
    if (rc) return rc;
    if (k_a < 1 || k_a > 8) return EBS_ERR_BITWIDTH;
    if (!finite_pos(alpha)) return EBS_ERR_SHAPE;
    return quantize_activations(x, count, alpha, k_a, levels, (hipStream_t)stream);
}

int ebs_aggregate_weights(const float *w, size_t count, const int *bits, int n_bits, const float *strengths,
                          const float *gumbel, float tau, float *w_hat, void *workspace, void *stream)
{
    if (!workspace) return EBS_ERR_NULL;
    int rc = check_elementwise(w, w_hat, count);
    if (rc) return rc;
    rc = check_candidates(bits, n_bits, strengths, gumbel, tau);
    if (rc) return rc;
    if (!aligned16(workspace)) return EBS_ERR_ALIGN;
    return aggregate_weights(w, count, bits, n_bits, strengths, gumbel, tau, w_hat, workspace, (hipStream_t)stream);
}

int ebs_aggregate_activations(const float *x, size_t count, float alpha, const int *bits, int n_bits,
                              const float *strengths, const float *gumbel, float tau, float *x_hat,
                              void *workspace, void *stream)
{
    if (!workspace) return EBS_ERR_NULL;
    int rc = check_elementwise(x, x_hat, count);
    if (rc) return rc;
    rc = check_candidates(bits, n_bits, strengths, gumbel, tau);
    if (rc) return rc;
    if (!finite_pos(alpha)) return EBS_ERR_SHAPE;
    if (!aligned16(workspace)) return EBS_ERR_ALIGN;
    return aggregate_activations(x, count, alpha, bits, n_bits, strengths, gumbel, tau, x_hat, workspace, (hipStream_t)stream);
}

int ebs_check_levels(const uint8_t *levels, size_t count, int bits, int32_t *device_flag, void *stream)
{
    if (!levels || !device_flag) return EBS_ERR_NULL;
    if (bits < 1 || bits > 7) return EBS_ERR_BITWIDTH;
    if (count == 0) return EBS_ERR_SHAPE;
    return check_levels(levels, count, bits, device_flag, (hipStream_t)stream);
}

}  // extern "C"
