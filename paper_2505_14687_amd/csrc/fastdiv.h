// Division of a non-negative 31-bit integer by a divisor known on the host, as one multiply-high and
// two shifts.  The kernels decompose tile, group and token indices by grid extents that are launch
// parameters; the compiler's general 32-bit division costs about thirty instructions each.
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#define GRAT_HD __host__ __device__ __forceinline__
#else
#define GRAT_HD inline
#endif

namespace grat {

struct FastDiv {
    uint32_t d;    // the divisor, >= 1
    uint32_t m;    // ceil(2^(31 + sh) / d), below 2^32
    uint32_t sh;   // ceil(log2 d)
};

// For 0 <= n < 2^31:  n / d == (2n * m) >> (32 + sh).  Proof: m * d = 2^(31+sh) + e with 0 <= e < d, so
// n * m / 2^(31+sh) = n / d + n * e / (d * 2^(31+sh)), and the excess is below 1 / d because
// n < 2^31 and e < d <= 2^sh; an excess below 1 / d cannot carry n / d over the next integer.
inline FastDiv make_fastdiv(uint32_t d) {
    FastDiv f;
    f.d = d < 1 ? 1 : d;
    f.sh = 0;
    while ((1ull << f.sh) < f.d) ++f.sh;
    const uint64_t num = 1ull << (31 + f.sh);
    f.m = (uint32_t)((num + f.d - 1) / f.d);
    return f;
}

GRAT_HD uint32_t mulhi_u32(uint32_t a, uint32_t b) {
#if defined(__HIP_DEVICE_COMPILE__)
    return __umulhi(a, b);
#else
    return (uint32_t)(((uint64_t)a * b) >> 32);
#endif
}

GRAT_HD uint32_t fdiv(uint32_t n, const FastDiv& f) { return mulhi_u32(n << 1, f.m) >> f.sh; }

// quotient and remainder
GRAT_HD void fdivmod(uint32_t n, const FastDiv& f, uint32_t& q, uint32_t& r) {
    q = fdiv(n, f);
    r = n - q * f.d;
}

}  // namespace grat
