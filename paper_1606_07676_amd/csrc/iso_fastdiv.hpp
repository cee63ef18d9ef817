// Division of a 32-bit unsigned integer by a run-time invariant divisor with one
// multiply-high, used to turn a flat work index into (rank, entry, chunk) and a
// rank into its torus coordinate without hardware integer division.
// (Round-up multiplier method of Granlund & Montgomery; exact for every 32-bit
// numerator and every divisor in [1, 2^31].)
#pragma once

#include <cstdint>

#if defined(__HIPCC__)
#define ISO_HD __host__ __device__ __forceinline__
#else
#define ISO_HD inline
#endif

namespace iso {

struct FastDiv {
    uint32_t mul;
    uint32_t sh1;
    uint32_t sh2;
    uint32_t div;
};

inline FastDiv make_fastdiv(uint32_t d) {
    FastDiv f;
    uint32_t l = 0;
    while ((uint64_t(1) << l) < d) ++l;             // l = ceil(log2 d)
    f.mul = (uint32_t)(((uint64_t(1) << 32) * ((uint64_t(1) << l) - d)) / d + 1);
    f.sh1 = l < 1 ? l : 1;
    f.sh2 = l > 0 ? l - 1 : 0;
    f.div = d;
    return f;
}

ISO_HD uint32_t mulhi_u32(uint32_t a, uint32_t b) {
#if defined(__HIP_DEVICE_COMPILE__)
    return __umulhi(a, b);
#else
    return (uint32_t)(((uint64_t)a * b) >> 32);
#endif
}

ISO_HD uint32_t fast_div(uint32_t n, const FastDiv &f) {
    const uint32_t t = mulhi_u32(f.mul, n);
    return (t + ((n - t) >> f.sh1)) >> f.sh2;
}

// q = n / d, r = n % d
ISO_HD void fast_divmod(uint32_t n, const FastDiv &f, uint32_t &q, uint32_t &r) {
    q = fast_div(n, f);
    r = n - q * f.div;
}

}  // namespace iso
