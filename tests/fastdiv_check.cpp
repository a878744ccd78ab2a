// Host check of csrc/fastdiv.h: the multiply-high division equals n / d for every divisor up to 70 000 (edge
// values, multiples and their predecessors, random n) and for 20 million random (n, d) pairs below 2^31.
#include "fastdiv.h"
#include <cstdio>
#include <cstdlib>
int main() {
    using namespace grat;
    unsigned long long bad = 0, cnt = 0;
    auto check = [&](uint32_t d, uint32_t n) { FastDiv f = make_fastdiv(d); ++cnt; if (fdiv(n, f) != n / d) { if (bad < 10) printf("BAD n=%u d=%u got %u want %u\n", n, d, fdiv(n, f), n / d); ++bad; } };
    const uint32_t edge[] = {0u, 1u, 2u, 3u, 63u, 64u, 65u, 255u, 256u, 65535u, 65536u, 0x7ffffffeu, 0x7fffffffu, 0x40000000u, 0x3fffffffu};
    uint32_t x = 12345u;
    auto rnd = [&]() { x ^= x << 13; x ^= x >> 17; x ^= x << 5; return x; };
    for (uint32_t d = 1; d <= 70000; ++d) {
        for (uint32_t n : edge) check(d, n);
        for (uint32_t k = 0; k < 8; ++k) { check(d, d * k); if (d * k) check(d, d * k - 1); }
        for (int i = 0; i < 20; ++i) check(d, rnd() & 0x7fffffffu);
        const uint32_t top = 0x7fffffffu / d * d; check(d, top); if (top) check(d, top - 1);
    }
    for (int i = 0; i < 20000000; ++i) { uint32_t d = rnd() & 0x7fffffffu; if (!d) d = 1; if (i & 1) d >>= (rnd() & 31); if (!d) d = 1; check(d, rnd() & 0x7fffffffu); }
    for (int s = 0; s < 31; ++s) for (int o = -2; o <= 2; ++o) { long long d = (1ll << s) + o; if (d >= 1 && d < (1ll << 31)) for (uint32_t n : edge) check((uint32_t)d, n); }
    printf("%llu checks, %llu bad\n", cnt, bad);
    return bad != 0;
}
