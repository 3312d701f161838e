// Quantisers (paper Preliminaries, Eq. 1a-1c) and the aggregated quantisation functions of
// the bitwidth search (Sec. 4.1: Eq. 6 weights, Eq. 7 activations, Eq. 8 stochastic
// coefficients).  All element-wise and HBM-bound, apart from one max reduction.
//
// Weights (Eq. 1a) are evaluated in double precision: a rounding decides an integer level, a
// weight tensor is small and quantised once per step, and a correctly ordered double
// evaluation agrees with any other double evaluation except within ~1e-16 of a tie.
//   max|tanh W| = tanh(max|W|) (tanh is odd and increasing), so the reduction runs on the
//   single-precision inputs themselves and is exact.
// Activations (Eq. 1b-1c) are evaluated in single precision in the fixed order of requant.h.
//
// Workspace (device memory of the caller, 256 bytes): dword 0 = bits of max|w|; byte 64 =
// eight doubles, the coefficients of the candidates; byte 128 = eight floats,
// coefficient_i * alpha / (2^b_i - 1).
#include "ebs_internal.h"
#include "requant.h"
#include <mutex>

namespace ebs {

// Workspace of ebs_quantize_weights_static: the same 256 bytes the caller of ebs_quantize_weights
// brings in, here a device array of the library itself (one copy per GPU, at an address of its
// own on each; held until the process ends).  Host code never uses the array's name as a
// pointer: the address on the current device comes from hipGetSymbolAddress, once per device.
static __device__ __align__(256) unsigned char scratch[EBS_QUANT_WORKSPACE_BYTES];

constexpr int kMaxDevices = 64;

// Address of `scratch` on the current device (looked up on the first call per device, kept after).
static int static_workspace(void **out)
{
    static std::mutex mu;
    static void *ptrs[kMaxDevices] = {};
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_ok(e);
    if (dev < 0 || dev >= kMaxDevices) return EBS_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(mu);
    if (!ptrs[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return hip_ok(e);
        if (!p) return EBS_ERR_HIP;
        ptrs[dev] = p;
    }
    *out = ptrs[dev];
    return EBS_OK;
}

struct Candidates {
    int n;
    int bits[kMaxCandidates];
    float qs[kMaxCandidates];      // (2^b - 1) / alpha (activations only)
};

__global__ void quant_ws_clear(uint32_t *ws) { ws[0] = 0u; }

__global__ void __launch_bounds__(256)
absmax_kernel(const float *__restrict__ w, size_t count, uint32_t *__restrict__ ws)
{
    __shared__ uint32_t part[4];
    const size_t step = (size_t)gridDim.x * 256;
    uint32_t m = 0u;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < count; i += step) {
        uint32_t b = __float_as_uint(w[i]) & 0x7FFFFFFFu;     // |w|: non-negative floats order like integers
        if (b > 0x7F800000u) b = 0u;                           // NaN takes no part
        m = b > m ? b : m;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const uint32_t o = (uint32_t)__shfl_xor((int)m, off);
        m = o > m ? o : m;
    }
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int i = 1; i < 4; ++i) m = part[i] > m ? part[i] : m;
        atomicMax(ws, m);
    }
}

// Normalised weight of Eq. 1a before rounding: tanh(w) / (2 max|tanh W|) + 1/2; 1/2 for an all-zero tensor.
__device__ __forceinline__ double normalised_weight(float w, double m)
{
    if (m == 0.0) return 0.5;
    return __dadd_rn(__ddiv_rn(tanh((double)w), __dmul_rn(2.0, m)), 0.5);
}

__device__ __forceinline__ double level_of(double x, int n)     // round half up
{
    return floor(__dadd_rn(__dmul_rn((double)n, x), 0.5));
}

__global__ void __launch_bounds__(256)
quantize_weights_kernel(const float *__restrict__ w, size_t count, int n_levels,
                        const uint32_t *__restrict__ ws, uint8_t *__restrict__ levels)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= count) return;
    const double m = tanh((double)__uint_as_float(ws[0]));
    levels[i] = (uint8_t)(int)level_of(normalised_weight(w[i], m), n_levels);
}

// Four activations per thread: one 16-byte load, one 4-byte store.
__global__ void __launch_bounds__(256)
quantize_activations_kernel(const float *__restrict__ x, size_t count, float alpha, float qs,
                            uint8_t *__restrict__ levels)
{
    const size_t i4 = ((size_t)blockIdx.x * 256 + threadIdx.x) * 4;
    if (i4 >= count) return;
    if (i4 + 3 < count) {
        const float4 v = *reinterpret_cast<const float4 *>(x + i4);
        const float e[4] = {v.x, v.y, v.z, v.w};
        uint32_t packed = 0u;
#pragma unroll
        for (int k = 0; k < 4; ++k)
            packed |= (uint32_t)(int)floorf(fmaf(fminf(fmaxf(e[k], 0.0f), alpha), qs, 0.5f)) << (8 * k);
        *reinterpret_cast<uint32_t *>(levels + i4) = packed;
    } else {
        for (size_t i = i4; i < count; ++i)
            levels[i] = (uint8_t)(int)floorf(fmaf(fminf(fmaxf(x[i], 0.0f), alpha), qs, 0.5f));
    }
}

// Coefficients of the candidates: softmax of the strengths (Eq. 6-7), or with Gumbel noise g and
// temperature tau the softmax of (log p + g) / tau (Eq. 8).  One thread; at most eight candidates.
__global__ void coefficients_kernel(const float *__restrict__ strengths, const float *__restrict__ gumbel, double tau,
                                    const Candidates cand, double alpha, uint8_t *__restrict__ ws)
{
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    double p[kMaxCandidates];
    double top = (double)strengths[0];
    for (int i = 1; i < cand.n; ++i) top = fmax(top, (double)strengths[i]);
    double sum = 0.0;
    for (int i = 0; i < cand.n; ++i) { p[i] = exp((double)strengths[i] - top); sum += p[i]; }
    for (int i = 0; i < cand.n; ++i) p[i] /= sum;
    if (gumbel) {
        double y[kMaxCandidates];
        for (int i = 0; i < cand.n; ++i) y[i] = (log(p[i]) + (double)gumbel[i]) / tau;
        top = y[0];
        for (int i = 1; i < cand.n; ++i) top = fmax(top, y[i]);
        sum = 0.0;
        for (int i = 0; i < cand.n; ++i) { p[i] = exp(y[i] - top); sum += p[i]; }
        for (int i = 0; i < cand.n; ++i) p[i] /= sum;
    }
    double *cd = reinterpret_cast<double *>(ws + 64);
    float *cf = reinterpret_cast<float *>(ws + 128);
    for (int i = 0; i < kMaxCandidates; ++i) {
        const bool on = i < cand.n;
        cd[i] = on ? p[i] : 0.0;
        cf[i] = on ? (float)(p[i] * alpha / (double)((1 << cand.bits[i]) - 1)) : 0.0f;
    }
}

__global__ void __launch_bounds__(256)
aggregate_weights_kernel(const float *__restrict__ w, size_t count, const Candidates cand,
                         const uint8_t *__restrict__ ws, float *__restrict__ out)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= count) return;
    const double m = tanh((double)__uint_as_float(*reinterpret_cast<const uint32_t *>(ws)));
    const double *coef = reinterpret_cast<const double *>(ws + 64);
    const double x = normalised_weight(w[i], m);
    double acc = 0.0;
    for (int c = 0; c < cand.n; ++c) {
        const int n = (1 << cand.bits[c]) - 1;
        const double what = __dadd_rn(__ddiv_rn(__dmul_rn(2.0, level_of(x, n)), (double)n), -1.0);   // Eq. 1a
        acc = __dadd_rn(acc, __dmul_rn(coef[c], what));
    }
    out[i] = (float)acc;
}

// NC: number of candidates, a compile-time constant so that the coefficients sit in registers and the
// candidate loop is unrolled (the kernel is then bound by HBM, not by instruction issue).
template <int NC>
__global__ void __launch_bounds__(256)
aggregate_activations_kernel(const float *__restrict__ x, size_t count, float alpha, const Candidates cand,
                             const uint8_t *__restrict__ ws, float *__restrict__ out)
{
    const size_t i4 = ((size_t)blockIdx.x * 256 + threadIdx.x) * 4;
    if (i4 >= count) return;
    const float *cfp = reinterpret_cast<const float *>(ws + 128);
    float cf[NC], qs[NC];
#pragma unroll
    for (int c = 0; c < NC; ++c) { cf[c] = cfp[c]; qs[c] = cand.qs[c]; }
    auto one = [&](float v) {
        const float z = fminf(fmaxf(v, 0.0f), alpha);
        float acc = 0.0f;
#pragma unroll
        for (int c = 0; c < NC; ++c) acc = fmaf(floorf(fmaf(z, qs[c], 0.5f)), cf[c], acc);
        return acc;
    };
    if (i4 + 3 < count) {
        const float4 v = *reinterpret_cast<const float4 *>(x + i4);
        *reinterpret_cast<float4 *>(out + i4) = make_float4(one(v.x), one(v.y), one(v.z), one(v.w));
    } else {
        for (size_t i = i4; i < count; ++i) out[i] = one(x[i]);
    }
}

static unsigned blocks_for(size_t items) { return (unsigned)((items + 255) / 256); }

static int reduce_absmax(const float *w, size_t count, uint32_t *ws, hipStream_t st)
{
    hipLaunchKernelGGL(quant_ws_clear, dim3(1), dim3(1), 0, st, ws);
    size_t want = (count + 255) / 256;
    unsigned blocks = (unsigned)(want < 256 ? want : 256);       // one atomic per block on a single address: keep them few
    hipLaunchKernelGGL(absmax_kernel, dim3(blocks), dim3(256), 0, st, w, count, ws);
    return hip_ok(hipGetLastError());
}

int quantize_weights(const float *w, size_t count, int bits, uint8_t *levels, void *workspace, hipStream_t st)
{
    uint32_t *ws = (uint32_t *)workspace;
    int rc = reduce_absmax(w, count, ws, st);
    if (rc) return rc;
    hipLaunchKernelGGL(quantize_weights_kernel, dim3(blocks_for(count)), dim3(256), 0, st, w, count, (1 << bits) - 1, ws, levels);
    return hip_ok(hipGetLastError());
}

// Same kernels as quantize_weights, the workspace being the library's own device array: no allocation
// anywhere (the first kernel clears the one word that must start at zero).
int quantize_weights_static(const float *w, size_t count, int bits, uint8_t *levels, hipStream_t st)
{
    void *ws = nullptr;
    int rc = static_workspace(&ws);
    if (rc) return rc;
    return quantize_weights(w, count, bits, levels, ws, st);
}

int quantize_activations(const float *x, size_t count, float alpha, int bits, uint8_t *levels, hipStream_t st)
{
    hipLaunchKernelGGL(quantize_activations_kernel, dim3(blocks_for((count + 3) / 4)), dim3(256), 0, st,
                       x, count, alpha, requant_qs(alpha, bits), levels);
    return hip_ok(hipGetLastError());
}

static Candidates make_candidates(const int *bits, int n, float alpha)
{
    Candidates c{};
    c.n = n;
    for (int i = 0; i < n; ++i) {
        c.bits[i] = bits[i];
        c.qs[i] = alpha > 0.0f ? requant_qs(alpha, bits[i]) : 0.0f;
    }
    return c;
}

int aggregate_weights(const float *w, size_t count, const int *bits, int n, const float *strengths, const float *gumbel,
                      float tau, float *out, void *workspace, hipStream_t st)
{
    const Candidates cand = make_candidates(bits, n, 0.0f);
    int rc = reduce_absmax(w, count, (uint32_t *)workspace, st);
    if (rc) return rc;
    hipLaunchKernelGGL(coefficients_kernel, dim3(1), dim3(1), 0, st, strengths, gumbel, (double)tau, cand, 1.0, (uint8_t *)workspace);
    hipLaunchKernelGGL(aggregate_weights_kernel, dim3(blocks_for(count)), dim3(256), 0, st, w, count, cand,
                       (const uint8_t *)workspace, out);
    return hip_ok(hipGetLastError());
}

int aggregate_activations(const float *x, size_t count, float alpha, const int *bits, int n, const float *strengths,
                          const float *gumbel, float tau, float *out, void *workspace, hipStream_t st)
{
    const Candidates cand = make_candidates(bits, n, alpha);
    hipLaunchKernelGGL(coefficients_kernel, dim3(1), dim3(1), 0, st, strengths, gumbel, (double)tau, cand, (double)alpha,
                       (uint8_t *)workspace);
    const dim3 grid(blocks_for((count + 3) / 4));
#define EBS_NC(nc) case nc: hipLaunchKernelGGL(aggregate_activations_kernel<nc>, grid, dim3(256), 0, st, x, count, alpha, \
                                               cand, (const uint8_t *)workspace, out); break;
    switch (n) { EBS_NC(1) EBS_NC(2) EBS_NC(3) EBS_NC(4) EBS_NC(5) EBS_NC(6) EBS_NC(7) EBS_NC(8) }
#undef EBS_NC
    return hip_ok(hipGetLastError());
}

}  // namespace ebs
