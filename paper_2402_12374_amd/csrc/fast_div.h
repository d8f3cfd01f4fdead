// Division of a 31-bit unsigned number by a divisor that is fixed for a whole kernel launch, as a
// multiplication: the host works out the multiplier once, the kernel spends a multiply-high, a
// shift and a select-by-mask (three scalar instructions for a uniform dividend) instead of the
// 25-instruction vector sequence of a hardware-less integer division.
//
// For d >= 2 let l = ceil(log2 d), m = ceil(2^(31 + l) / d) (it fits 32 bits because d > 2^(l-1)).
// Then m d = 2^(31 + l) + e with 0 <= e < d <= 2^l, and for n < 2^31
//     floor(n m / 2^(31 + l)) = floor(n / d + n e / (d 2^(31 + l)))  with  n e / 2^(31 + l) < 1,
// which is floor(n / d): the second term cannot carry n / d over the next integer, since the
// fractional part of n / d is at most (d - 1) / d.  d = 1 has no such m; it is handled by a mask
// that lets the dividend through.
#pragma once
#include <cstdint>
#include <hip/hip_runtime.h>

namespace seqtree {

struct FastDiv {
    uint32_t mul;     // m
    uint32_t shift;   // l - 1: the multiply-high already shifts by 32
    uint32_t one;     // all ones iff d == 1
};

inline FastDiv make_fast_div(uint32_t d) {
    FastDiv f{0u, 0u, 0u};
    if (d <= 1) { f.one = 0xFFFFFFFFu; return f; }
    uint32_t l = 0;
    while ((1ull << l) < d) ++l;
    const unsigned long long top = 1ull << (31 + l);
    f.mul = (uint32_t)((top + d - 1) / d);
    f.shift = l - 1;
    return f;
}

// n < 2^31
__host__ __device__ __forceinline__ uint32_t fast_div(uint32_t n, const FastDiv& f) {
#if defined(__HIP_DEVICE_COMPILE__)
    const uint32_t hi = __umulhi(n, f.mul);
#else
    const uint32_t hi = (uint32_t)(((unsigned long long)n * f.mul) >> 32);
#endif
    return (hi >> f.shift) | (n & f.one);
}

}  // namespace seqtree
