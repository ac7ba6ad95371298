// Host check of the reciprocal multiplication the fused attention kernel decomposes its workgroup index with:
// floor(n / d) == (n * ceil(2^40 / d)) >> 40 for every n the launcher admits (n d < 2^40, n / d < 2^23).
// Exhaustive over small n, and around every multiple of d near the admitted maximum, for many divisors.
#include <cstdint>
#include <cstdio>
#include "../../paper_2507_05228_amd/csrc/attn_bf16.h"

static bool check(uint32_t n, uint32_t d, uint64_t magic) {
    if (div_by_magic(n, magic) == n / d) return true;
    std::printf("MISMATCH n=%u d=%u got=%u want=%u\n", n, d, div_by_magic(n, magic), n / d);
    return false;
}

int main() {
    const uint32_t divisors[] = {1, 2, 3, 5, 7, 8, 12, 31, 32, 33, 63, 64, 96, 127, 255, 256, 257, 1000, 1023, 1024,
                                 4095, 4096, 4097, 12345, 65535, 65536, 65537, 1000003};
    uint64_t checked = 0;
    for (uint32_t d : divisors) {
        const uint64_t magic = div_magic(d);
        // the largest n the launcher's test admits for this divisor (capped at 2^32 - 1)
        uint64_t n_max = ((1ull << 40) - 1) / d;
        if (n_max / d >= (1ull << 23)) n_max = ((1ull << 23) - 1) * (uint64_t)d + (d - 1);
        if (n_max > 0xffffffffull) n_max = 0xffffffffull;
        while (n_max > 0 && !div_magic_covers(n_max, d)) --n_max;
        if (!div_magic_covers(n_max, d)) { std::printf("no admitted range for d=%u\n", d); return 1; }
        const uint64_t lo_end = n_max < 300000 ? n_max : 300000;
        for (uint64_t n = 0; n <= lo_end; ++n, ++checked)
            if (!check((uint32_t)n, d, magic)) return 1;
        // around multiples of d, from the top of the range downwards
        const uint64_t q_top = n_max / d;
        for (uint64_t k = 0; k < 20000 && k <= q_top; ++k) {
            const uint64_t m = (q_top - k) * d;
            for (int64_t off = -2; off <= 2; ++off) {
                const int64_t n = (int64_t)m + off;
                if (n < 0 || (uint64_t)n > n_max) continue;
                ++checked;
                if (!check((uint32_t)n, d, magic)) return 1;
            }
        }
        if (!check((uint32_t)n_max, d, magic)) return 1;
    }
    std::printf("DIV_MAGIC_OK %llu cases\n", (unsigned long long)checked);
    return 0;
}
