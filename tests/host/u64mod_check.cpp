// Host check of the exact 64-bit remainder used by the hashing kernels: the
// same header the device code includes, compiled for the CPU and compared with
// the C `%` operator on adversarial and random operands.
#include <cstdint>
#include <cstdio>

#include "u64mod.h"

static uint64_t rng_state = 0x853C49E6748FEA9Bull;
static uint64_t next()
{
    rng_state ^= rng_state << 13;
    rng_state ^= rng_state >> 7;
    rng_state ^= rng_state << 17;
    return rng_state;
}

int main()
{
    const uint64_t edge_r[] = {1, 2, 3, 7, 10, 63, 64, 65, 1000003, 10000000, 1000000000, 250000000,
                               (1ull << 31) - 1, 1ull << 31, (1ull << 32) - 1, 1ull << 32, (1ull << 32) + 1,
                               (1ull << 40) + 17, (1ull << 62), (1ull << 62) + 1, (1ull << 63) - 25, (1ull << 63) - 1};
    const uint64_t edge_x[] = {0, 1, 2, ~0ull, ~0ull - 1, 1ull << 63, (1ull << 63) - 1, (1ull << 63) + 1,
                               1ull << 32, (1ull << 32) - 1, 0xFFFFFFFF00000000ull, 0x00000000FFFFFFFFull};
    long checked = 0;
    for (uint64_t R : edge_r) {
        const uint64_t m = emb_mod_magic(R);
        for (uint64_t x : edge_x) {
            if (emb_fast_mod(x, R, m) != x % R) { std::printf("FAIL x=%llu R=%llu\n", (unsigned long long)x, (unsigned long long)R); return 1; }
            ++checked;
        }
        // multiples of R and their neighbours are where an off-by-one quotient shows
        for (int k = 0; k < 2000; ++k) {
            uint64_t q = next() % (~0ull / R);
            for (int d = -2; d <= 2; ++d) {
                uint64_t x = q * R + (uint64_t)d;
                if (emb_fast_mod(x, R, m) != x % R) { std::printf("FAIL x=%llu R=%llu\n", (unsigned long long)x, (unsigned long long)R); return 1; }
                ++checked;
            }
        }
    }
    for (int i = 0; i < 2000000; ++i) {
        uint64_t R = next() >> (next() % 63 + 1);
        if (R == 0 || R >= (1ull << 63)) continue;
        uint64_t x = next() >> (next() % 64);
        if (emb_fast_mod(x, R, emb_mod_magic(R)) != x % R) { std::printf("FAIL x=%llu R=%llu\n", (unsigned long long)x, (unsigned long long)R); return 1; }
        ++checked;
    }
    std::printf("OK %ld\n", checked);
    return 0;
}
