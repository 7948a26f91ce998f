// Host check of the multiply-high division that the tile kernel uses to decompose a
// workgroup index (harris_launch.h): every quotient must equal the hardware division.
// Built and run by tests/test_abi_host.py; prints "ok <pairs checked>" or the first mismatch.
#include <cstdint>
#include <cstdio>

#include "harris_launch.h"

static uint64_t state = 0x9e3779b97f4a7c15ull;
static uint32_t next_u32() {
    state ^= state << 13; state ^= state >> 7; state ^= state << 17;
    return (uint32_t)(state >> 16);
}

static bool check(uint32_t x, uint32_t d, unsigned long long& count) {
    const harris_launch::FastDiv f = harris_launch::make_fastdiv(d);
    ++count;
    if (harris_launch::fastdiv(x, f) == x / d) return true;
    std::printf("mismatch: %u / %u gives %u, expected %u\n", x, d, harris_launch::fastdiv(x, f), x / d);
    return false;
}

int main() {
    unsigned long long count = 0;
    const uint32_t edge[] = {0u, 1u, 2u, 3u, 0x7ffffffeu, 0x7fffffffu, 0x80000000u, 0x80000001u, 0xfffffffeu, 0xffffffffu};
    // Every small divisor against every small dividend, multiples of the divisor and their neighbours.
    for (uint32_t d = 1; d <= 2048; ++d) {
        for (uint32_t x = 0; x <= 4096; ++x) if (!check(x, d, count)) return 1;
        for (uint32_t e : edge) if (!check(e, d, count)) return 1;
        for (uint32_t q = 0xffffffffu / d; q > 0xffffffffu / d - 3 && q > 0; --q)
            for (int o = -1; o <= 1; ++o) if (!check(q * d + (uint32_t)o, d, count)) return 1;
    }
    // Divisors around every power of two, and random ones, against edge and random dividends.
    for (int l = 1; l < 32; ++l)
        for (int o = -2; o <= 2; ++o) {
            const uint32_t d = (1u << l) + (uint32_t)o;
            if (d == 0) continue;
            for (uint32_t e : edge) if (!check(e, d, count)) return 1;
            for (int i = 0; i < 2000; ++i) if (!check(next_u32(), d, count)) return 1;
            for (uint32_t q = 0; q < 4 && q <= 0xffffffffu / d; ++q)
                for (int oo = -1; oo <= 1; ++oo) if (!check(q * d + (uint32_t)oo, d, count)) return 1;
        }
    for (int i = 0; i < 200000; ++i) {
        uint32_t d = next_u32() >> (next_u32() % 32);
        if (d == 0) d = 1;
        if (!check(next_u32(), d, count)) return 1;
        if (!check(next_u32() % d, d, count)) return 1;
        const uint32_t q = (uint32_t)(next_u32() % (0xffffffffull / d + 1ull));
        if (!check(q * d, d, count)) return 1;
        if (q > 0 && !check(q * d - 1u, d, count)) return 1;
    }
    std::printf("ok %llu\n", count);
    return 0;
}
