// The 16-bit group word of the b + 16/g storage format: helpers shared by the quantizer and the GPTQ sweep.
#pragma once

#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include <cstdint>

// 16-bit group word (mfmt = the code width b, 0 = fp32 scale and u8 zero kept apart): the scale
// is rounded to fp16 (nearest even) and that to the 16-b leading bits of its 15-bit pattern
// (nearest even on the pattern: an unsigned float with fp16's exponent and 11-b fraction bits);
// a pattern of 0 becomes 1, the format's smallest value.  Everything after it (zero-point,
// codes, dW) is computed from the rounded scale, so what is stored de-quantizes exactly as scored.
__device__ __forceinline__ uint32_t scale_pattern(float s, int b) {
    const uint32_t h = __half_as_ushort(__float2half_rn(s));
    const int d = b - 1;
    const uint32_t q = (h + ((1u << d) >> 1) - 1u + ((h >> d) & 1u)) >> d;
    return q ? q : 1u;
}
__device__ __forceinline__ float round_scale(float s, int b) {
    return __half2float(__ushort_as_half(static_cast<unsigned short>(scale_pattern(s, b) << (b - 1))));
}
// writes a group's parameters: fp32 scale and u8 zero-point, or the 16-bit word (pattern << b | zero)
// into `scales` taken as an array of u16
__device__ __forceinline__ void store_params(float* __restrict__ scales, uint8_t* __restrict__ zeros, int64_t i, float s,
                                             float z, int mfmt) {
    if (mfmt) {
        if (scales)
            reinterpret_cast<uint16_t*>(scales)[i] =
                static_cast<uint16_t>((scale_pattern(s, mfmt) << mfmt) | static_cast<uint32_t>(z));
    } else {
        if (scales) scales[i] = s;
        if (zeros) zeros[i] = static_cast<uint8_t>(z);
    }
}

// scale and zero-point of a group word (mfmt = b)
__device__ __forceinline__ float word_scale(uint32_t word, int mfmt) {
    return __half2float(__ushort_as_half(static_cast<unsigned short>((word >> mfmt) << (mfmt - 1))));
}
__device__ __forceinline__ float word_zero(uint32_t word, int mfmt) { return static_cast<float>(word & ((1u << mfmt) - 1u)); }
