// Host check of csrc/fd_fastdiv.hpp: exhaustive over small divisors and numerators, then edge
// numerators (multiples of d and their neighbours, the top of the 31-bit range) for many divisors.
#include <cstdio>
#include <cstdlib>

#include "../paper_2511_02168_amd/csrc/fd_fastdiv.hpp"

static unsigned long long checked = 0;

static int check(uint32_t n, uint32_t d, fd::FastDiv f)
{
    ++checked;
    if (fd::fast_div(n, f) != n / d) {
        std::printf("MISMATCH n=%u d=%u got %u want %u\n", n, d, fd::fast_div(n, f), n / d);
        return 1;
    }
    return 0;
}

int main()
{
    const uint32_t top = 0x7fffffffu;
    int bad = 0;
    for (uint32_t d = 1; d <= 4096 && !bad; ++d) {
        const fd::FastDiv f = fd::make_fastdiv(d);
        for (uint32_t n = 0; n < 70000 && !bad; ++n) bad |= check(n, d, f);
    }
    uint64_t x = 88172645463325252ull;
    for (int it = 0; it < 200000 && !bad; ++it) {
        x ^= x << 13; x ^= x >> 7; x ^= x << 17;                     // xorshift: seeded, no library RNG
        uint32_t d = (uint32_t)(x >> 33) & top;
        if (it % 3 == 0) d >>= (x & 31);                              // all magnitudes
        if (d == 0) d = 1;
        const fd::FastDiv f = fd::make_fastdiv(d);
        const uint32_t qmax = top / d;
        const uint32_t qs[6] = {0u, 1u, qmax / 2, qmax > 0 ? qmax - 1 : 0u, qmax, (uint32_t)(x % (qmax + 1ull))};
        for (uint32_t q : qs) {
            const uint64_t m = (uint64_t)q * d;
            for (long long delta = -2; delta <= 2 && !bad; ++delta) {
                const long long n = (long long)m + delta;
                if (n >= 0 && n <= (long long)top) bad |= check((uint32_t)n, d, f);
            }
            if (m + d - 1 <= top) bad |= check((uint32_t)(m + d - 1), d, f);
        }
        bad |= check(top, d, f);
        bad |= check((uint32_t)(x & top), d, f);
    }
    std::printf("%s %llu\n", bad ? "FAIL" : "OK", checked);
    return bad;
}
