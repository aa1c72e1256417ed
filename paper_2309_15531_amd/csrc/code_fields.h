// How the de-quantizing matrix-vector product reads b-bit codes out of a packed stream without an
// integer-to-float conversion (Sec. 4.5 / App. D kernel; the scheme is this build's).
//
// A field of b bits that starts at bit s <= 10 - b of a 16-bit half, under the exponent bits of
// 2^(10-s), is the fp16 number 2^(10-s) + code: the field sits in the low fraction bits, whose unit
// at that exponent is 2^-s.  One and-or therefore turns a 32-bit word into two such numbers (one per
// half), which a mixed-precision fma takes as operands; the constants 2^(10-s) leave the sum later
// (code_offset).  Fields that do not start low enough in their half are read from a shifted copy of
// the word (4 and 2 bits) or of the whole 96-bit stream (3 bits, whose codes straddle every boundary).
//
// A lane's 32 codes are `PB` words, code k at bit k * PB of the stream.  field_step<PB>(s) is step s
// of the plan: which word, shifted by how much, which mask and exponent constant, and which two codes
// come out.  Plain constexpr C++: the kernel unrolls over it, the host-side check runs it on the CPU.
#pragma once

#include <cstdint>

#if defined(__HIPCC__)
#define CODE_FIELDS_FN __host__ __device__ constexpr
#else
#define CODE_FIELDS_FN constexpr
#endif

struct FieldStep {
    int word;         // source word of the lane's PB words
    int shift;        // read from the stream shifted right by this many bits (0, 8 or 10), starting at that word
    uint32_t mask;    // the two fields, one per half
    int orc_id;       // which exponent constant (field_orc) is or-ed in
    int k_lo, k_hi;   // codes that come out in the low and high half (-1: none)
};

// bit pattern of the fp16 value 2^e
CODE_FIELDS_FN uint32_t f16_exp2(int e) { return static_cast<uint32_t>(e + 15) << 10; }

// 3 bits: stream t (0: as stored, 1: shifted by 8), word w belong to class (w + t) % 3; step q of a class takes
// the field at bit f3_start(c, q, 0) of the low half and f3_start(c, q, 1) of the high half (-1: none)
CODE_FIELDS_FN int f3_start(int c, int q, int h) {
    constexpr int S[3][3][2] = {{{0, 2}, {3, 5}, {6, -1}}, {{1, 0}, {4, 3}, {7, 6}}, {{2, 1}, {5, 4}, {-1, 7}}};
    return S[c][q][h];
}

template <int PB>
CODE_FIELDS_FN int field_steps() { return PB == 3 ? 18 : 16; }
template <int PB>
CODE_FIELDS_FN int field_orcs() { return PB == 4 ? 2 : (PB == 2 ? 5 : 9); }

template <int PB>
CODE_FIELDS_FN uint32_t field_orc(int id) {
    if (PB == 4) return f16_exp2(id == 0 ? 10 : 6) * 0x10001u;       // fields at bit 0 and at bit 4
    if (PB == 2) return f16_exp2(10 - 2 * id) * 0x10001u;            // fields at bits 0, 2, 4, 6, 8
    const int c = id / 3, q = id % 3;                                // 3 bits: a different start in each half
    return (f3_start(c, q, 0) >= 0 ? f16_exp2(10 - f3_start(c, q, 0)) : 0u) |
           (f3_start(c, q, 1) >= 0 ? f16_exp2(10 - f3_start(c, q, 1)) << 16 : 0u);
}

template <int PB>
CODE_FIELDS_FN FieldStep field_step(int s) {
    if (PB == 4) {                                                   // word i, step n: nibbles n and n + 4
        const int i = s / 4, n = s % 4;
        return {i, 8 * (n >> 1), (n & 1) ? 0x00F000F0u : 0x000F000Fu, n & 1, 8 * i + n, 8 * i + n + 4};
    }
    if (PB == 2) {                                                   // word i, step q: fields q and q + 8
        const int i = s / 8, q = s % 8, p = q < 5 ? q : q - 5;       // fields 5..7 from the word shifted by 10
        return {i, q < 5 ? 0 : 10, 0x00030003u << (2 * p), p, 16 * i + q, 16 * i + 8 + q};
    }
    const int t = s / 9, w = (s % 9) / 3, q = s % 3, c = (w + t) % 3;
    const int s_lo = f3_start(c, q, 0), s_hi = f3_start(c, q, 1);
    return {w, 8 * t, (s_lo >= 0 ? 7u << s_lo : 0u) | (s_hi >= 0 ? 7u << (16 + s_hi) : 0u), 3 * c + q,
            s_lo >= 0 ? (32 * w + s_lo + 8 * t) / 3 : -1, s_hi >= 0 ? (32 * w + 16 + s_hi + 8 * t) / 3 : -1};
}

// what code k was read as, minus the code: 2^(10 - s), s the start of its field within its half
template <int PB>
CODE_FIELDS_FN float code_offset(int k) {
    if (PB == 4) return (k & 1) ? 64.0f : 1024.0f;
    if (PB == 2) {
        const int f = k & 7;                                         // field within its half: 0..4 direct, 5..7 shifted by 10
        return static_cast<float>(1024 >> (2 * (f < 5 ? f : f - 5)));
    }
    const int b = 3 * k, t = (b & 15) <= 7 ? 0 : 1;
    return static_cast<float>(1024 >> ((b - 8 * t) & 15));
}
