// Host-side check of the launch-constant division used by every kernel's work-item decode
// (swaa::make_fastdiv / swaa::fastdiv): exact for every numerator below 2^31.
// Built and run by tests/test_host_fastdiv.py; needs no GPU.
#include <cstdint>
#include <cstdio>

#include "swaa_common.h"

static unsigned long long state = 0x9E3779B97F4A7C15ull;
static unsigned long long next() {  // xorshift64*
    state ^= state >> 12;
    state ^= state << 25;
    state ^= state >> 27;
    return state * 0x2545F4914F6CDD1Dull;
}

int main() {
    long bad = 0, checked = 0;
    auto check = [&](unsigned n, unsigned d) {
        ++checked;
        if (swaa::fastdiv(n, swaa::make_fastdiv(d)) != n / d) {
            if (bad < 10) std::printf("mismatch: %u / %u\n", n, d);
            ++bad;
        }
    };
    // every divisor up to 2^16 against the numerators where a wrong multiplier shows first
    for (unsigned d = 1; d <= 65536; ++d) {
        const unsigned top = 0x7fffffffu / d * d;
        const unsigned ns[] = {0u, 1u, d - 1, d, d + 1, 2 * d - 1, 2 * d, top - 1, top, 0x7ffffffeu, 0x7fffffffu};
        for (unsigned n : ns)
            if (n <= 0x7fffffffu) check(n, d);
        for (int i = 0; i < 16; ++i) check((unsigned)next() & 0x7fffffffu, d);
    }
    // random divisors of every magnitude
    for (int i = 0; i < 4000000; ++i) {
        unsigned d = ((unsigned)next() & 0x7fffffffu) >> (next() % 31);
        if (d == 0) d = 1;
        check((unsigned)next() & 0x7fffffffu, d);
        check(0x7fffffffu / d * d, d);
    }
    std::printf("checked %ld divisions, %ld wrong\n", checked, bad);
    return bad != 0;
}
