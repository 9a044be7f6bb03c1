// Host check of the reciprocal division the streaming kernels use for index arithmetic: against the machine's own
// division for every divisor up to 8192 and a set of large ones, at the dividends around every multiple the sampling
// reaches, at random dividends and at the largest dividend allowed (2^31 - 1).  Built with the host compiler by
// tests/test_fast_div_cpu.py; prints the number of mismatches.
#include "fast_div.h"

#include <cstdint>
#include <cstdio>
#include <vector>

int main() {
    long bad = 0, n = 0;
    auto check = [&](unsigned q, unsigned d, const ols::FastDiv& f) {
        ++n;
        if (ols::fast_div(q, f) != q / d) {
            if (bad < 5) std::printf("q=%u d=%u got %u want %u\n", q, d, ols::fast_div(q, f), q / d);
            ++bad;
        }
    };
    std::vector<unsigned> ds;
    for (unsigned d = 1; d <= 8192; ++d) ds.push_back(d);
    for (unsigned d : {65535u, 65536u, 65537u, 1000003u, 16777215u, 16777216u, 16777217u, (1u << 30) - 1, 1u << 30, (1u << 30) + 1,
                       (1u << 31) - 2, (1u << 31) - 1})
        ds.push_back(d);
    uint64_t rng = 0x9E3779B97F4A7C15ull;
    for (unsigned d : ds) {
        const ols::FastDiv f = ols::make_div(d);
        for (uint64_t k = 0; k * d < (1ull << 31); k += (k < 64 ? 1 : k / 3 + 1))
            for (int o = -2; o <= 2; ++o) {
                const int64_t q = (int64_t)(k * d) + o;
                if (q >= 0 && q < (1ll << 31)) check((unsigned)q, d, f);
            }
        for (int t = 0; t < 256; ++t) {
            rng = rng * 6364136223846793005ull + 1442695040888963407ull;
            check((unsigned)(rng >> 33), d, f);
        }
        check((1u << 31) - 1, d, f);
    }
    std::printf("%ld checks, %ld mismatches\n", n, bad);
    return bad != 0;
}
