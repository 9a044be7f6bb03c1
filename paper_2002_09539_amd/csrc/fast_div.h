// Division of a 31-bit dividend by a divisor known on the host, as a multiplication (Granlund and Montgomery's round-up
// method): m = floor(2^32 (2^s - d) / d) + 1 with s = ceil(log2 d), and q / d = (t + ((q - t) >> 1)) >> (s - 1) with
// t = mulhi(q, m).  The streaming kernels use it to turn a linear index into (sample, row, column).
#pragma once
#include <hip/hip_runtime.h>

namespace ols {

struct FastDiv {
    unsigned magic, shift;
};

inline FastDiv make_div(unsigned d) {
    FastDiv f = {0u, 0u};
    unsigned s = 0;
    while ((1ull << s) < d) ++s;
    f.shift = s;
    if (s > 0) f.magic = (unsigned)((((1ull << s) - d) << 32) / d + 1);
    return f;
}

// q / d for 0 <= q < 2^31
__host__ __device__ __forceinline__ unsigned fast_div(unsigned q, const FastDiv& d) {
    if (d.shift == 0) return q;   // d = 1
    const unsigned t = (unsigned)(((unsigned long long)q * d.magic) >> 32);   // one v_mul_hi_u32 on the device
    return (t + ((q - t) >> 1)) >> (d.shift - 1);
}

}  // namespace ols
