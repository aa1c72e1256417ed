// Host-side check of csrc/code_fields.h: running the extraction plan on the CPU gives back every code.
// For each bit width: random and extreme code vectors are packed (code k at bit k * PB of the lane's stream), every
// step of the plan is applied as the kernel applies it (shifted source, and-or with the mask and the exponent
// constant), the two halves are read as fp16 numbers, and number - code_offset(k) must be the code, exactly, with
// every code produced once.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cmath>

#include "../../paper_2309_15531_amd/csrc/code_fields.h"

// value of a (normal, positive) fp16 bit pattern
static float half_value(uint32_t h) {
    const int e = (h >> 10) & 31, m = h & 1023;
    return std::ldexp(1.0f + m / 1024.0f, e - 15);
}

template <int PB>
static int check(uint64_t seed) {
    int bad = 0;
    for (int trial = 0; trial < 2000; ++trial) {
        int code[32];
        for (int k = 0; k < 32; ++k) {
            seed = seed * 6364136223846793005ull + 1442695040888963407ull;
            const int r = static_cast<int>(seed >> 40) & ((1 << PB) - 1);
            code[k] = trial == 0 ? 0 : (trial == 1 ? (1 << PB) - 1 : (trial == 2 ? (k & 1 ? (1 << PB) - 1 : 0) : r));
        }
        uint32_t w[PB + 1] = {};
        for (int k = 0; k < 32; ++k) {
            const int b = k * PB;
            w[b / 32] |= static_cast<uint32_t>(code[k]) << (b % 32);
            if (b % 32 + PB > 32) w[b / 32 + 1] |= static_cast<uint32_t>(code[k]) >> (32 - b % 32);
        }
        int seen[32] = {};
        for (int s = 0; s < field_steps<PB>(); ++s) {
            const FieldStep f = field_step<PB>(s);
            uint32_t src = w[f.word];
            if (f.shift) {
                // 3 bits: the stream shifted across words; 4 and 2 bits: the word alone
                const uint64_t two = PB == 3 ? (static_cast<uint64_t>(f.word + 1 < PB ? w[f.word + 1] : 0u) << 32) | w[f.word] : w[f.word];
                src = static_cast<uint32_t>(two >> f.shift);
            }
            const uint32_t v = (src & f.mask) | field_orc<PB>(f.orc_id);
            const int ks[2] = {f.k_lo, f.k_hi};
            for (int h = 0; h < 2; ++h) {
                if (ks[h] < 0) continue;
                if (ks[h] >= 32) { ++bad; continue; }
                ++seen[ks[h]];
                const float got = half_value((v >> (16 * h)) & 0xffffu) - code_offset<PB>(ks[h]);
                if (got != static_cast<float>(code[ks[h]])) ++bad;
            }
        }
        for (int k = 0; k < 32; ++k) bad += seen[k] != 1;
    }
    return bad;
}

int main() {
    const int b2 = check<2>(1), b3 = check<3>(2), b4 = check<4>(3);
    std::printf("2 bits: %d, 3 bits: %d, 4 bits: %d mismatches\n", b2, b3, b4);
    return (b2 | b3 | b4) ? 1 : 0;
}
