// Correctly rounded fp32 quotient w/s from a precomputed reciprocal.
//
// The quantizer divides every weight of a group by the same scale.  With
// y = RN(1/s) computed once per group by a true IEEE division, the quotient of
// each weight costs three operations instead of a full division sequence:
//     t = RN(w*y);  r = fma(-s, t, w) (the exact residual);  q = fma(r, y, t).
// q equals the correctly rounded w/s for every w that is an fp16 value (at most
// 11 significant bits) and every normal fp32 s for which no intermediate leaves
// the normal range; tests/host/fastdiv_check.cpp verifies this exhaustively over
// all significand pairs (the operations are invariant under power-of-two
// scaling of w and s).  Callers take the plain division when fastdiv_ok(s)
// is false.
//
// Plain C++ (fmaf), so that the same text compiles for the host-side check and,
// through hipcc, for the device (v_fma_f32 is a single-rounding fused op).
#pragma once

#include <cmath>

#if defined(__HIPCC__)
#define FASTDIV_FN __host__ __device__ __forceinline__
#else
#define FASTDIV_FN inline
#endif

// s in [2^-40, 2^40]: with |w| in {0} U [2^-24, 65504] every intermediate stays normal.
FASTDIV_FN bool fastdiv_ok(float s) { return s >= 9.094947e-13f && s <= 1.0995116e12f; }

FASTDIV_FN float fastdiv(float w, float s, float y) {
    const float t = w * y;
    const float r = fmaf(-s, t, w);
    return fmaf(r, y, t);
}
