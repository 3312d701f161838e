// Division of a 31-bit unsigned integer by a runtime-constant divisor with one
// high multiply: the host prepares (m, a, s) once, kernels evaluate
// q = (mulhi(x, m) + (a ? x : 0)) >> s.  Valid for 0 <= x < 2^31, 1 <= d < 2^31.
#pragma once
#include <stdint.h>

namespace ebs {

struct FastDiv {
    uint32_t d, m, a, s;
};

inline FastDiv make_fastdiv(uint32_t d)
{
    FastDiv f{};
    f.d = d;
    if (d <= 1) {            // x / 1
        f.d = 1; f.m = 0; f.a = 1; f.s = 0;
        return f;
    }
    uint32_t l = 0;
    while ((1ull << l) < d) ++l;                       // l = ceil(log2 d) >= 1
    f.m = (uint32_t)(((1ull << (31 + l)) / d) + 1);    // < 2^32 because d > 2^(l-1)
    f.a = 0;
    f.s = l - 1;                                       // mulhi already shifts by 32
    return f;
}

#if defined(__HIPCC__)
__device__ __forceinline__ uint32_t fd_div(uint32_t x, const FastDiv &f)
{
    return (__umulhi(x, f.m) + (f.a ? x : 0u)) >> f.s;
}
#endif

inline uint32_t fd_div_host(uint32_t x, const FastDiv &f)
{
    return (uint32_t)((((uint64_t)x * f.m) >> 32) + (f.a ? x : 0u)) >> f.s;
}

}  // namespace ebs
