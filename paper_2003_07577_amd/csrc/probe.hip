// Micro-benchmarks that measure the achievable denominators of the rooflines:
// the sustained issue rate of the AND + accumulating-bitcount pair (the inner
// body of Eq. 2 on this hardware) and the device copy bandwidth.
#include "ebs_internal.h"
#include "ebs_probe.h"

namespace ebs {

// acc + bitcount(x) in one instruction (v_bcnt_u32_b32 adds its second operand), written out as in the
// convolution kernels: left to itself the optimiser regroups sums of bitcounts into count + three-operand add,
// 2.5 issue slots per pair instead of 2, and the probe would under-measure the peak it is there to establish.
__device__ __forceinline__ uint32_t probe_bcnt_acc(uint32_t x, uint32_t acc)
{
    uint32_t d;
    asm("v_bcnt_u32_b32 %0, %1, %2" : "=v"(d) : "v"(x), "v"(acc));
    return d;
}

// Each lane keeps 32 accumulators and applies, per loop trip, 8 scalar operands
// to 4 vector operands: 32 (v_and_b32, v_bcnt_u32_b32) pairs, no memory traffic.
__global__ void __launch_bounds__(256)
probe_and_bcnt_kernel(const uint32_t *__restrict__ seed, uint32_t *__restrict__ sink, int trips)
{
    uint32_t x[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) x[p] = seed[(threadIdx.x + p * 64) & 255];
    uint32_t q[8];
#pragma unroll
    for (int c = 0; c < 8; ++c) q[c] = seed[256 + c];       // uniform address -> scalar registers
    uint32_t acc[4][8];
#pragma unroll
    for (int p = 0; p < 4; ++p)
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[p][c] = 0u;
    for (int t = 0; t < trips; ++t) {
#pragma unroll
        for (int rep = 0; rep < 4; ++rep) {
#pragma unroll
            for (int p = 0; p < 4; ++p)
#pragma unroll
                for (int c = 0; c < 8; ++c) acc[p][c] = probe_bcnt_acc(q[c] & x[p], acc[p][c]);
#pragma unroll
            for (int p = 0; p < 4; ++p) x[p] = __builtin_amdgcn_mov_dpp(x[p], 0x130 /* wave_shl:1 */, 0xf, 0xf, false);
        }
    }
    uint32_t s = 0;
#pragma unroll
    for (int p = 0; p < 4; ++p)
#pragma unroll
        for (int c = 0; c < 8; ++c) s += acc[p][c];
    sink[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

__global__ void __launch_bounds__(256)
probe_copy_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst, size_t n16)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t step = (size_t)gridDim.x * blockDim.x;
    for (; i < n16; i += step) dst[i] = src[i];
}

__global__ void __launch_bounds__(256)
probe_fill_kernel(uint4 *__restrict__ dst, size_t n16)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t step = (size_t)gridDim.x * blockDim.x;
    uint4 v = {1u, 2u, 3u, 4u};
    for (; i < n16; i += step) dst[i] = v;
}

}  // namespace ebs

using namespace ebs;

extern "C" {

int ebs_probe_and_bcnt(const uint32_t *seed, uint32_t *sink, int blocks, int trips, void *stream)
{
    if (!seed || !sink) return EBS_ERR_NULL;
    if (blocks <= 0 || trips <= 0) return EBS_ERR_SHAPE;
    hipLaunchKernelGGL(probe_and_bcnt_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, seed, sink, trips);
    return hip_ok(hipGetLastError());
}

long long ebs_probe_and_bcnt_pairs(int blocks, int trips)
{
    return (long long)blocks * 256 * trips * 4 * 32;
}

int ebs_probe_copy(const void *src, void *dst, size_t bytes, int blocks, void *stream)
{
    if (!dst) return EBS_ERR_NULL;
    if (bytes == 0 || (bytes & 15) || blocks <= 0) return EBS_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(dst) & 15) || (reinterpret_cast<uintptr_t>(src) & 15)) return EBS_ERR_ALIGN;
    if (src)
        hipLaunchKernelGGL(probe_copy_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream,
                           (const uint4 *)src, (uint4 *)dst, bytes / 16);
    else
        hipLaunchKernelGGL(probe_fill_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, (uint4 *)dst, bytes / 16);
    return hip_ok(hipGetLastError());
}

}  // extern "C"
