// Group-wise asymmetric round-to-nearest quantizer (paper Sec. 2.1, 3.2, 4.1)
// for both grouping dimensions, and the bit-packing of its codes.
//
// The arithmetic is IEEE fp32, one rounding per operation (the file is built
// with -ffp-contract=off): per group
//   mx = clip*max(max w,0), mn = clip*min(min w,0), scale = (mx-mn)/qmax or 1,
//   zero = clamp(rint(-mn/scale)), code = clamp(rint(w/scale)+zero),
//   dW = w - scale*(code-zero).
// The work is bandwidth bound: every kernel reads W once from HBM (the per-IC
// kernel re-reads its tile from cache) with 16-byte loads and writes each
// output once.
#include "common.h"
#include "fastdiv.h"
#include "scale_format.h"

#include <cstdlib>
#include <type_traits>

namespace {

struct GroupParams {
    float scale;
    float zero;
};

__device__ __forceinline__ GroupParams group_params(float mn, float mx, float clip, float qmax, int mfmt) {
    mx = fmaxf(mx, 0.0f);
    mn = fminf(mn, 0.0f);
    mx = clip * mx;
    mn = clip * mn;
    const float range = mx - mn;
    float scale = range / qmax;
    if (range == 0.0f) scale = 1.0f;
    if (mfmt) scale = round_scale(scale, mfmt);
    float z = rintf((-mn) / scale);
    z = fminf(fmaxf(z, 0.0f), qmax);
    return {scale, z};
}

__device__ __forceinline__ float quant_code(float w, float scale, float zero, float qmax) {
    const float q = rintf(w / scale) + zero;
    return fminf(fmaxf(q, 0.0f), qmax);
}

__device__ __forceinline__ float weight_error(float w, float q, float scale, float zero) {
    const float what = scale * (q - zero);
    return w - what;
}

__device__ __forceinline__ void unpack8(const uint4& v, float (&w)[8]) {
    const __half2* h = reinterpret_cast<const __half2*>(&v);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float2 f = __half22float2(h[i]);
        w[2 * i] = f.x;
        w[2 * i + 1] = f.y;
    }
}

// Stores 8 consecutive dW values of row `row` starting at column `col` (a multiple of 8);
// elem = row*in + col.  The scaled fp16 form goes to the scoring layout.
__device__ __forceinline__ void store_dw8(void* dW, int dW_dtype, const float* __restrict__ colscale,
                                          int64_t elem, int64_t row, int64_t col, int64_t out, int64_t in,
                                          const float (&d)[8]) {
    if (dW_dtype == ADADIM_DW_F32) {
        float4* p = reinterpret_cast<float4*>(static_cast<float*>(dW) + elem);
        p[0] = make_float4(d[0], d[1], d[2], d[3]);
        p[1] = make_float4(d[4], d[5], d[6], d[7]);
    } else {
        float s[8];
        if (dW_dtype == ADADIM_DW_F16_SCALED) {
            const float4 a = *reinterpret_cast<const float4*>(colscale + col);
            const float4 b = *reinterpret_cast<const float4*>(colscale + col + 4);
            s[0] = d[0] * a.x; s[1] = d[1] * a.y; s[2] = d[2] * a.z; s[3] = d[3] * a.w;
            s[4] = d[4] * b.x; s[5] = d[5] * b.y; s[6] = d[6] * b.z; s[7] = d[7] * b.w;
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) s[i] = d[i];
        }
        uint4 o;
        __half2* h = reinterpret_cast<__half2*>(&o);
#pragma unroll
        for (int i = 0; i < 4; ++i) h[i] = __floats2half2_rn(s[2 * i], s[2 * i + 1]);
        const int64_t at = dW_dtype == ADADIM_DW_F16_SCALED ? score_index(row, col, out, in) : elem;
        *reinterpret_cast<uint4*>(static_cast<__half*>(dW) + at) = o;
    }
}

__device__ __forceinline__ void store_dw1(void* dW, int dW_dtype, const float* __restrict__ colscale,
                                          int64_t elem, int64_t row, int64_t col, int64_t out, int64_t in, float d) {
    if (dW_dtype == ADADIM_DW_F32) {
        static_cast<float*>(dW)[elem] = d;
    } else if (dW_dtype == ADADIM_DW_F16_SCALED) {
        static_cast<__half*>(dW)[score_index(row, col, out, in)] = __float2half_rn(d * colscale[col]);
    } else {
        static_cast<__half*>(dW)[elem] = __float2half_rn(d);
    }
}

// per-OC, any group length: one wavefront per group, element-wise accesses.
__global__ __launch_bounds__(256) void quant_oc_generic(const __half* __restrict__ W, int64_t n_groups, int g,
                                                        int64_t out, int64_t in, float clip, float qmax, int mfmt,
                                                        uint8_t* __restrict__ codes, float* __restrict__ scales,
                                                        uint8_t* __restrict__ zeros, void* __restrict__ dW,
                                                        int dW_dtype, const float* __restrict__ colscale) {
    const int lane = threadIdx.x & 63;
    const int64_t grp = int64_t(blockIdx.x) * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (grp >= n_groups) return;  // whole wavefront leaves together
    const int64_t base = grp * g;
    float mn = 0.0f, mx = 0.0f;   // the range contains zero anyway
    for (int i = lane; i < g; i += 64) {
        const float w = __half2float(W[base + i]);
        mn = fminf(mn, w);
        mx = fmaxf(mx, w);
    }
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) {
        mn = fminf(mn, __shfl_xor(mn, m, 64));
        mx = fmaxf(mx, __shfl_xor(mx, m, 64));
    }
    const GroupParams gp = group_params(mn, mx, clip, qmax, mfmt);
    if (lane == 0) {
        store_params(scales, zeros, grp, gp.scale, gp.zero, mfmt);
    }
    for (int i = lane; i < g; i += 64) {
        const float w = __half2float(W[base + i]);
        const float q = quant_code(w, gp.scale, gp.zero, qmax);
        if (codes) codes[base + i] = static_cast<uint8_t>(q);
        if (dW)
            store_dw1(dW, dW_dtype, colscale, base + i, (base + i) / in, (base + i) % in, out, in,
                      weight_error(w, q, gp.scale, gp.zero));
    }
}

// ---------------------------------------------------------------------------
// Fast paths.  Same arithmetic, organised for bandwidth:
//  * the per-weight division uses the group's correctly rounded reciprocal
//    (fastdiv.h: three operations, bit-identical to the IEEE quotient);
//  * min/max across the lanes of a group go through DPP row operations
//    instead of LDS permutes;
//  * several 16-byte chunks per thread are in flight at once;
//  * the bit stream is assembled in registers (2, 3, 4 and 8 bits).

struct GroupParamsR {
    float scale, zero, rcp;
    bool fast;
};

// IEEE division that the optimiser may not hoist out of the (rarely taken, wave-uniform)
// branch it sits in: the empty volatile asm pins it there.
__device__ __forceinline__ float pinned_div(float a, float b) {
    asm volatile("" : "+v"(a));
    return a / b;
}

// Same results as group_params, with the divisions replaced by fastdiv where its
// preconditions hold: range/qmax through the reciprocal of qmax (exact for every
// range, see fastdiv_check.cpp), -mn/scale through the reciprocal of the scale when
// mn is an fp16 value (clip == 1).  The plain divisions sit behind wave-uniform
// branches so that they cost nothing when no lane needs them.
__device__ __forceinline__ GroupParamsR group_params_r(float mn, float mx, float clip, float qmax, float rqmax, int mfmt) {
    mx = fmaxf(mx, 0.0f);
    mn = fminf(mn, 0.0f);
    mx = clip * mx;
    mn = clip * mn;
    const float range = mx - mn;
    float scale = fastdiv(range, qmax, rqmax);
    if (__any(!(range >= 8.6736174e-19f) && range != 0.0f)) scale = pinned_div(range, qmax);   // below 2^-60: tiny clip
    if (range == 0.0f) scale = 1.0f;
    if (mfmt) scale = round_scale(scale, mfmt);
    const float rcp = 1.0f / scale;
    const bool fast = fastdiv_ok(scale);
    float zq = fastdiv(-mn, scale, rcp);
    if (__any(!fast || clip != 1.0f)) zq = pinned_div(-mn, scale);
    const float z = __builtin_amdgcn_fmed3f(rintf(zq), 0.0f, qmax);
    return {scale, z, rcp, fast};
}

template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) {
    return __builtin_bit_cast(
        float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u(uint32_t v) {
    return static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(v), CTRL, 0xf, 0xf, true));
}

// Bit stream of 8 codes held by one lane, for chunk c of a flat [out, in] weight.
// PB = bits per code (2, 3, 4 or 8).  Words are written straight to `packed`
// (rows are whole numbers of words because in % 32 == 0).
template <int PB>
__device__ __forceinline__ void pack8_store(const float (&q)[8], int64_t c, bool valid,
                                            uint32_t* __restrict__ packed) {
    uint32_t lo = 0, hi = 0;  // 8*PB bits, little end first
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const uint32_t code = static_cast<uint32_t>(q[i]);
        const int bit = i * PB;
        if (bit < 32) lo |= code << bit;
        if (bit + PB > 32) hi |= bit >= 32 ? code << (bit - 32) : code >> (32 - bit);
    }
    if constexpr (PB == 8) {
        if (valid) reinterpret_cast<uint2*>(packed)[c] = make_uint2(lo, hi);
    } else if constexpr (PB == 4) {
        if (valid) packed[c] = lo;
    } else if constexpr (PB == 2) {
        const uint32_t other = dpp_u<0xB1>(lo);       // partner lane's 16 bits
        if (valid && (c & 1) == 0) packed[c >> 1] = lo | (other << 16);
    } else {                                           // PB == 3: four lanes -> three words
        const uint32_t next = dpp_u<0xF9>(lo);        // quad_perm [1,2,3,3]: the next lane's 24 bits
        const int j = static_cast<int>(c & 3);
        if (valid && j < 3) packed[(c >> 2) * 3 + j] = (lo >> (8 * j)) | (next << (24 - 8 * j));
    }
}

// ---------------------------------------------------------------------------
// per-IC: a block owns the g rows of one row-group and COLS = 32*VEC adjacent
// columns.  Lane x of row-slice y scans rows y, y+8, ... of its VEC columns,
// the 8 slices are combined through LDS, the column parameters are computed
// once, and a second sweep (served by L2) quantizes.
template <int VEC>
__global__ __launch_bounds__(256) void quant_ic_tile(const __half* __restrict__ W, int64_t out, int64_t in, int g,
                                                     float clip, float qmax, int mfmt, uint8_t* __restrict__ codes,
                                                     float* __restrict__ scales, uint8_t* __restrict__ zeros,
                                                     void* __restrict__ dW, int dW_dtype,
                                                     const float* __restrict__ colscale) {
    constexpr int COLS = 32 * VEC;
    __shared__ float s_mn[8][COLS];
    __shared__ float s_mx[8][COLS];
    __shared__ float s_scale[COLS];
    __shared__ float s_zero[COLS];

    const int tx = threadIdx.x & 31;
    const int ty = threadIdx.x >> 5;
    const int64_t col0 = int64_t(blockIdx.x) * COLS + tx * VEC;
    const int64_t row0 = int64_t(blockIdx.y) * g;
    const bool col_ok = col0 < in;  // in % VEC == 0, so the whole vector is inside

    float mn[VEC], mx[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) mn[v] = mx[v] = 0.0f;
    if (col_ok) {
        for (int r = ty; r < g; r += 8) {
            const __half* p = W + (row0 + r) * in + col0;
            float w[VEC];
            if constexpr (VEC == 8) {
                float t[8];
                unpack8(*reinterpret_cast<const uint4*>(p), t);
#pragma unroll
                for (int v = 0; v < 8; ++v) w[v] = t[v];
            } else {
                w[0] = __half2float(p[0]);
            }
#pragma unroll
            for (int v = 0; v < VEC; ++v) {
                mn[v] = fminf(mn[v], w[v]);
                mx[v] = fmaxf(mx[v], w[v]);
            }
        }
    }
#pragma unroll
    for (int v = 0; v < VEC; ++v) {
        s_mn[ty][tx * VEC + v] = mn[v];
        s_mx[ty][tx * VEC + v] = mx[v];
    }
    __syncthreads();
    for (int cidx = threadIdx.x; cidx < COLS; cidx += 256) {
        float a = s_mn[0][cidx], b = s_mx[0][cidx];
#pragma unroll
        for (int y = 1; y < 8; ++y) {
            a = fminf(a, s_mn[y][cidx]);
            b = fmaxf(b, s_mx[y][cidx]);
        }
        const GroupParams gp = group_params(a, b, clip, qmax, mfmt);
        s_scale[cidx] = gp.scale;
        s_zero[cidx] = gp.zero;
        const int64_t col = int64_t(blockIdx.x) * COLS + cidx;
        if (col < in) {
            const int64_t gi = int64_t(blockIdx.y) * in + col;
            store_params(scales, zeros, gi, gp.scale, gp.zero, mfmt);
        }
    }
    __syncthreads();
    if (!col_ok || (!codes && !dW)) return;
    float sc[VEC], zp[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) {
        sc[v] = s_scale[tx * VEC + v];
        zp[v] = s_zero[tx * VEC + v];
    }
    for (int r = ty; r < g; r += 8) {
        const int64_t elem = (row0 + r) * in + col0;
        if constexpr (VEC == 8) {
            float w[8], q[8];
            unpack8(*reinterpret_cast<const uint4*>(W + elem), w);
#pragma unroll
            for (int v = 0; v < 8; ++v) q[v] = quant_code(w[v], sc[v], zp[v], qmax);
            if (codes) {
                uint32_t lo = 0, hi = 0;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    lo |= static_cast<uint32_t>(q[i]) << (8 * i);
                    hi |= static_cast<uint32_t>(q[4 + i]) << (8 * i);
                }
                *reinterpret_cast<uint2*>(codes + elem) = make_uint2(lo, hi);
            }
            if (dW) {
                float d[8];
#pragma unroll
                for (int v = 0; v < 8; ++v) d[v] = weight_error(w[v], q[v], sc[v], zp[v]);
                store_dw8(dW, dW_dtype, colscale, elem, row0 + r, col0, out, in, d);
            }
        } else {
            const float w = __half2float(W[elem]);
            const float q = quant_code(w, sc[0], zp[0], qmax);
            if (codes) codes[elem] = static_cast<uint8_t>(q);
            if (dW) store_dw1(dW, dW_dtype, colscale, elem, row0 + r, col0, out, in, weight_error(w, q, sc[0], zp[0]));
        }
    }
}

// ---------------------------------------------------------------------------
// Element arithmetic of the streaming kernels.  v_fma_mix_f32 reads an fp16 operand straight
// from one half of a packed register, so the weight is never converted on its own:
//     t   = fma(w, y, -0)            = RN(w*y)                  (y = RN(1/scale))
//     r   = fma(-scale, t, w)        the exact residual         (fastdiv.h)
//     quo = fma(r, y, t)             = RN(w/scale)
//     k   = med3(rint(quo), -zero, qmax-zero)   = code - zero   (all three are small integers,
//           so clamping before or after adding the zero point gives the same code)
//     dW*c = fma(w, c, -(scale*c)*k) = RN((w - RN(scale*k))*c)  for a power of two c:
//           scaling by c is exact, so RN(scale*c*k) = c*RN(scale*k) and the single rounding of
//           the fma is the rounding of w - RN(scale*k).  c = 1 gives the plain dW.
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
// -0.0f the optimiser cannot see through: fma(w, y, -0) must stay an fma for the compiler to
// pick the mixed-precision form (as a plain product it would convert the fp16 operand first).
__device__ __forceinline__ float opaque_negzero() {
    float z = -0.0f;
    asm("" : "+v"(z));
    return z;
}
template <int HI>
__device__ __forceinline__ float fma_hff(uint32_t hpair, float b, float c) {   // fma(half HI of hpair, b, c)
    return __builtin_fmaf(static_cast<float>(__builtin_bit_cast(f16x2, hpair)[HI]), b, c);
}
template <int HI>
__device__ __forceinline__ float fma_ffh(float a, float b, uint32_t hpair) {   // fma(a, b, half HI of hpair)
    return __builtin_fmaf(a, b, static_cast<float>(__builtin_bit_cast(f16x2, hpair)[HI]));
}

// Per-column (per-IC) or per-group (per-OC) constants of the element arithmetic.
struct QConst {
    float y;      // RN(1/scale)
    float ns;     // -scale
    float nz;     // -zero
    float pz;     // qmax - zero
    float n0;     // -0.0f, opaque
};

// RN(w/scale) for the weight in half HI of `pair` (valid when fastdiv_ok(scale))
template <int HI>
__device__ __forceinline__ float quant_quo(uint32_t pair, const QConst& c) {
    const float t = fma_hff<HI>(pair, c.y, c.n0);
    const float r = fma_ffh<HI>(c.ns, t, pair);
    return fmaf(r, c.y, t);
}

// k = code - zero for the 8 weights of one 16-byte chunk, column constants c[0..7].  `slow`
// (wave-uniform) takes the IEEE division for scales outside fastdiv's range.
__device__ __forceinline__ void quant_k8(const uint32_t (&v)[4], const QConst (&c)[8], bool slow, float (&k)[8]) {
    float quo[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        quo[2 * i] = quant_quo<0>(v[i], c[2 * i]);
        quo[2 * i + 1] = quant_quo<1>(v[i], c[2 * i + 1]);
    }
    if (slow) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const f16x2 w = __builtin_bit_cast(f16x2, v[i]);
            quo[2 * i] = pinned_div(static_cast<float>(w[0]), -c[2 * i].ns);
            quo[2 * i + 1] = pinned_div(static_cast<float>(w[1]), -c[2 * i + 1].ns);
        }
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) k[i] = __builtin_amdgcn_fmed3f(rintf(quo[i]), c[i].nz, c[i].pz);
}

// the same with one group's constants for all 8 weights (per-OC)
__device__ __forceinline__ void quant_k8(const uint32_t (&v)[4], const QConst& c, bool slow, float (&k)[8]) {
    float quo[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        quo[2 * i] = quant_quo<0>(v[i], c);
        quo[2 * i + 1] = quant_quo<1>(v[i], c);
    }
    if (slow) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const f16x2 w = __builtin_bit_cast(f16x2, v[i]);
            quo[2 * i] = pinned_div(static_cast<float>(w[0]), -c.ns);
            quo[2 * i + 1] = pinned_div(static_cast<float>(w[1]), -c.ns);
        }
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) k[i] = __builtin_amdgcn_fmed3f(rintf(quo[i]), c.nz, c.pz);
}

__device__ __forceinline__ uint32_t pack_h2(float lo, float hi) {
    return __builtin_bit_cast(uint32_t, __floats2half2_rn(lo, hi));
}

__device__ __forceinline__ uint32_t pk_min(uint32_t a, uint32_t b) {   // v_pk_min_f16
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_min(__builtin_bit_cast(f16x2, a), __builtin_bit_cast(f16x2, b)));
}
__device__ __forceinline__ uint32_t pk_max(uint32_t a, uint32_t b) {   // v_pk_max_f16
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(f16x2, a), __builtin_bit_cast(f16x2, b)));
}
__device__ __forceinline__ float half_of(uint32_t pair, int hi) {
    return __half2float(__ushort_as_half(static_cast<unsigned short>(hi ? pair >> 16 : pair & 0xffffu)));
}

// (min, -max) pairs over clusters of LPG adjacent lanes (LPG a power of two, aligned): one
// packed minimum per exchange serves both.  quad_perm [1,0,3,2] and [2,3,0,1] exchange inside
// a quad, row_half_mirror pairs the two quads of 8 lanes, row_mirror the two halves of a row.
template <int LPG>
__device__ __forceinline__ uint32_t cluster_min2(uint32_t m) {
    if constexpr (LPG >= 2) m = pk_min(m, dpp_u<0xB1>(m));
    if constexpr (LPG >= 4) m = pk_min(m, dpp_u<0x4E>(m));
    if constexpr (LPG >= 8) m = pk_min(m, dpp_u<0x141>(m));
    if constexpr (LPG >= 16) m = pk_min(m, dpp_u<0x140>(m));
    if constexpr (LPG >= 32) m = pk_min(m, static_cast<uint32_t>(__shfl_xor(static_cast<int>(m), 16, 64)));
    if constexpr (LPG >= 64) m = pk_min(m, static_cast<uint32_t>(__shfl_xor(static_cast<int>(m), 32, 64)));
    return m;
}

// per-OC fast path: LPG lanes per group.  A block owns a tile of 16 rows x 64 chunks (512
// columns); wavefront w takes rows 4w..4w+3, lane l chunk l, so every load is one contiguous
// kilobyte and the four loads of a lane are in flight together.  The (min, -max) of a lane's
// chunk are taken on the packed fp16 values and meet across the group's lanes through DPP.
// With four or more lanes per group the four lanes of a quad sit in the same group for each of
// the wave's four rows: lane l works out the parameters of row l & 3 and the quad trades them,
// one parameter computation per wave instead of four.  The column-scaled fp16 dW goes to the
// scoring layout, where the 64-byte pieces of 16 consecutive rows of one 32-column block are
// adjacent: the tile is turned through LDS so that each store instruction writes such a
// contiguous kilobyte instead of 16 scattered pieces.
// (bx, by): the block's tile, handed in so that one launch can serve both grouping dimensions.
template <int LPG, int PB, bool SCALED>
__device__ __forceinline__ void quant_oc_body(unsigned bx, unsigned by, const uint4* __restrict__ W, int64_t out,
                                              int chunks_per_row, float clip, float qmax, float rqmax, int mfmt,
                                              uint8_t* __restrict__ codes, float* __restrict__ scales,
                                              uint8_t* __restrict__ zeros, void* __restrict__ dW, int dW_dtype,
                                              const float* __restrict__ colscale, uint32_t* __restrict__ packed) {
    constexpr int U = 4, PITCH = 68;                        // LDS row pitch in 16-byte units (conflict-free)
    __shared__ uint4 s_t[SCALED ? 16 * PITCH : 1];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int cc = bx * 64 + lane;                  // chunk within the row
    const int64_t row0 = int64_t(by) * 16;
    const bool col_ok = cc < chunks_per_row;                // whole groups: chunks_per_row % LPG == 0
    const int64_t in = int64_t(chunks_per_row) * 8;
    const bool turn = SCALED && score_blocked(in);
    uint4 raw[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t row = row0 + 4 * wave + u;
        raw[u] = (col_ok && row < out) ? W[row * chunks_per_row + cc] : make_uint4(0, 0, 0, 0);
    }
    float cs[8] = {1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f};
    if constexpr (SCALED) {
        if (col_ok) {
            const float4 a = *reinterpret_cast<const float4*>(colscale + int64_t(cc) * 8);
            const float4 b = *reinterpret_cast<const float4*>(colscale + int64_t(cc) * 8 + 4);
            cs[0] = a.x; cs[1] = a.y; cs[2] = a.z; cs[3] = a.w;
            cs[4] = b.x; cs[5] = b.y; cs[6] = b.z; cs[7] = b.w;
        }
    }
    // per row: (min, -max) of the group, low and high half of one register
    uint32_t m2[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint32_t mnp = pk_min(pk_min(raw[u].x, raw[u].y), pk_min(raw[u].z, raw[u].w));
        const uint32_t nmx = pk_max(pk_max(raw[u].x, raw[u].y), pk_max(raw[u].z, raw[u].w)) ^ 0x80008000u;
        const uint32_t lo = __builtin_amdgcn_perm(nmx, mnp, 0x05040100u);   // (min of even, -max of even elements)
        const uint32_t hi = __builtin_amdgcn_perm(nmx, mnp, 0x07060302u);   // the same of the odd elements
        m2[u] = cluster_min2<LPG>(pk_min(lo, hi));
    }
    float sc_u[U], zp_u[U], rc_u[U];
    bool slow;
    if constexpr (LPG >= 4) {
        const int mine = lane & 3;
        const uint32_t msel = (mine & 2) ? ((mine & 1) ? m2[3] : m2[2]) : ((mine & 1) ? m2[1] : m2[0]);
        const GroupParamsR gp = group_params_r(half_of(msel, 0), -half_of(msel, 1), clip, qmax, rqmax, mfmt);
        slow = __any(!gp.fast);
        sc_u[0] = dpp_f<0x00>(gp.scale); zp_u[0] = dpp_f<0x00>(gp.zero); rc_u[0] = dpp_f<0x00>(gp.rcp);
        sc_u[1] = dpp_f<0x55>(gp.scale); zp_u[1] = dpp_f<0x55>(gp.zero); rc_u[1] = dpp_f<0x55>(gp.rcp);
        sc_u[2] = dpp_f<0xAA>(gp.scale); zp_u[2] = dpp_f<0xAA>(gp.zero); rc_u[2] = dpp_f<0xAA>(gp.rcp);
        sc_u[3] = dpp_f<0xFF>(gp.scale); zp_u[3] = dpp_f<0xFF>(gp.zero); rc_u[3] = dpp_f<0xFF>(gp.rcp);
    } else {
        bool fast = true;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const GroupParamsR gp = group_params_r(half_of(m2[u], 0), -half_of(m2[u], 1), clip, qmax, rqmax, mfmt);
            sc_u[u] = gp.scale; zp_u[u] = gp.zero; rc_u[u] = gp.rcp;
            fast = fast && gp.fast;
        }
        slow = __any(!fast);
    }
    const float n0 = opaque_negzero();
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t row = row0 + 4 * wave + u;
        const bool valid = col_ok && row < out;
        const int64_t c = row * chunks_per_row + cc;         // flat chunk index
        const QConst qc = {rc_u[u], -sc_u[u], -zp_u[u], qmax - zp_u[u], n0};
        const uint32_t v[4] = {raw[u].x, raw[u].y, raw[u].z, raw[u].w};
        float k[8];
        quant_k8(v, qc, slow, k);
        if constexpr (PB != 0) {
            if (packed) {                                    // all lanes take part in the DPP
                float q[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) q[i] = k[i] + zp_u[u];
                pack8_store<PB>(q, c, valid, packed);
            }
        }
        if (dW != nullptr && (turn || valid)) {
            float d[8];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float s0 = SCALED ? qc.ns * cs[2 * i] : qc.ns, s1 = SCALED ? qc.ns * cs[2 * i + 1] : qc.ns;
                d[2 * i] = fma_hff<0>(v[i], cs[2 * i], s0 * k[2 * i]);
                d[2 * i + 1] = fma_hff<1>(v[i], cs[2 * i + 1], s1 * k[2 * i + 1]);
            }
            if (!SCALED && dW_dtype == ADADIM_DW_F32) {
                float4* p = reinterpret_cast<float4*>(static_cast<float*>(dW) + c * 8);
                p[0] = make_float4(d[0], d[1], d[2], d[3]);
                p[1] = make_float4(d[4], d[5], d[6], d[7]);
            } else {
                const uint4 o = make_uint4(pack_h2(d[0], d[1]), pack_h2(d[2], d[3]), pack_h2(d[4], d[5]), pack_h2(d[6], d[7]));
                if (turn) s_t[(4 * wave + u) * PITCH + lane] = o;
                else *reinterpret_cast<uint4*>(static_cast<__half*>(dW) + (SCALED ? score_index(row, int64_t(cc) * 8, out, in) : c * 8)) = o;
            }
        }
        if (!valid) continue;
        if ((cc & (LPG - 1)) == 0) {
            const int64_t grp = c / LPG;
            store_params(scales, zeros, grp, sc_u[u], zp_u[u], mfmt);
        }
        if (codes) {
            uint32_t lo = 0, hi = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                lo |= static_cast<uint32_t>(k[i] + zp_u[u]) << (8 * i);
                hi |= static_cast<uint32_t>(k[4 + i] + zp_u[u]) << (8 * i);
            }
            reinterpret_cast<uint2*>(codes)[c] = make_uint2(lo, hi);
        }
    }
    if (!turn) return;                                       // uniform
    __syncthreads();
    // store phase: wavefront w writes the tile's 32-column blocks 4w..4w+3; lane l carries row l >> 2,
    // quarter l & 3 of the block, so the 64 lanes cover 16 rows x 64 bytes = 1 KB contiguous
    const int srow = lane >> 2, sq = lane & 3;
    const int64_t grow = row0 + srow;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int kb = 4 * wave + u;                         // block within the tile
        const int chunk = bx * 64 + 4 * kb + sq;     // chunk within the row
        if (grow < out && chunk < chunks_per_row) {
            const int64_t at = score_index(grow, int64_t(chunk) * 8, out, in);
            *reinterpret_cast<uint4*>(static_cast<__half*>(dW) + at) = s_t[srow * PITCH + 4 * kb + sq];
        }
    }
}

template <int LPG, int PB, bool SCALED>
__global__ __launch_bounds__(256) void quant_oc_fast(const uint4* __restrict__ W, int64_t out, int chunks_per_row,
                                                     float clip, float qmax, float rqmax, int mfmt,
                                                     uint8_t* __restrict__ codes, float* __restrict__ scales,
                                                     uint8_t* __restrict__ zeros, void* __restrict__ dW,
                                                     int dW_dtype, const float* __restrict__ colscale,
                                                     uint32_t* __restrict__ packed) {
    quant_oc_body<LPG, PB, SCALED>(blockIdx.x, blockIdx.y, W, out, chunks_per_row, clip, qmax, rqmax, mfmt, codes, scales,
                                   zeros, dW, dW_dtype, colscale, packed);
}

// per-IC streaming path.  A group of G = 8*U*RW rows x 64 columns is shared by RW wavefronts, each
// holding 8*U rows: lane l takes rows 8u + (l >> 3), u = 0..U-1, of the 8 columns of chunk l & 7,
// so every load instruction fetches one full 128-byte line from each of 8 rows and all U loads of a
// lane are in flight together.  Small per-wave tiles matter: a wave reads its whole tile before it
// can write anything, and only many short waves keep reads and writes mixed on the memory fabric.
// Minima and maxima are taken on the packed fp16 values (exact), meet across the eight row lanes
// through three exchanges and across the RW waves through 512 bytes of LDS (the only barrier).
// Lane (row lane r, chunk c) then works out the parameters of column 8c + r alone and the eight
// lanes of a chunk trade them.  In the scoring layout the 8 rows x 64 bytes that a store
// instruction writes for one 32-column block are contiguous.
//
// PB != 0 (2, 3 or 4 bits, U == 4): the bit stream is assembled here too.  A wave's 32 rows give
// PB whole words per column.  Each lane collects the four codes of each of its columns as bytes
// (byte u = row 8u + row lane), the wave turns them through a private LDS patch so that lane l
// holds all 32 codes of column l, and that lane shifts them into place and writes the PB words.
template <int U, int RW, bool SCALED, int PB>
__device__ __forceinline__ void quant_ic_body(
    unsigned bx, unsigned by, const __half* __restrict__ W, int64_t out, int64_t in, float clip, float qmax, float rqmax,
    int mfmt, uint8_t* __restrict__ codes, float* __restrict__ scales, uint8_t* __restrict__ zeros, void* __restrict__ dW,
    int dW_dtype, const float* __restrict__ colscale, uint32_t* __restrict__ packed, int64_t n_words) {
    constexpr int CSW = RW <= 4 ? 4 / RW : 1;                // 64-column sets per block
    constexpr int G = 8 * U * RW;
    static_assert(PB == 0 || (U == 4 && (PB == 2 || PB == 3 || PB == 4)), "fused packing: 32-row wave tiles, 2..4 bits");
    __shared__ uint32_t s_mm[CSW][RW][2][32];                // [set][row wave][min|max][chunk*4 + pair]
    __shared__ uint32_t s_pk[PB ? CSW * RW : 1][8][65];      // [wave][row lane][column], odd pitch
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int rw = wave % RW, cw = wave / RW;
    const int rl = lane >> 3, cl = lane & 7;
    const int64_t col0 = ((int64_t(bx) * CSW + cw) * 8 + cl) * 8;
    const int64_t row0 = int64_t(by) * G + rw * (8 * U) + rl;   // this lane's rows: row0 + 8u
    const bool col_ok = col0 < in;                           // in % 8 == 0: the whole chunk is inside

    uint4 raw[U];
#pragma unroll
    for (int u = 0; u < U; ++u)
        raw[u] = col_ok ? *reinterpret_cast<const uint4*>(W + (row0 + 8 * u) * in + col0) : make_uint4(0, 0, 0, 0);

    // column minima / maxima as packed fp16 pairs; the range contains zero anyway
    uint32_t mn2[4] = {0u, 0u, 0u, 0u}, mx2[4] = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint32_t v[4] = {raw[u].x, raw[u].y, raw[u].z, raw[u].w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            mn2[i] = pk_min(mn2[i], v[i]);
            mx2[i] = pk_max(mx2[i], v[i]);
        }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        mn2[i] = pk_min(mn2[i], dpp_u<0x128>(mn2[i]));     // row_ror:8 = the lane 8 away in its row of 16
        mx2[i] = pk_max(mx2[i], dpp_u<0x128>(mx2[i]));
        mn2[i] = pk_min(mn2[i], static_cast<uint32_t>(__shfl_xor(static_cast<int>(mn2[i]), 16, 64)));
        mx2[i] = pk_max(mx2[i], static_cast<uint32_t>(__shfl_xor(static_cast<int>(mx2[i]), 16, 64)));
        mn2[i] = pk_min(mn2[i], static_cast<uint32_t>(__shfl_xor(static_cast<int>(mn2[i]), 32, 64)));
        mx2[i] = pk_max(mx2[i], static_cast<uint32_t>(__shfl_xor(static_cast<int>(mx2[i]), 32, 64)));
    }
    // this lane's column: 8*cl + rl, i.e. half rl & 1 of pair rl >> 1
    uint32_t mnp, mxp;
    if constexpr (RW > 1) {
        if (rl == 0) {
            *reinterpret_cast<uint4*>(&s_mm[cw][rw][0][cl * 4]) = make_uint4(mn2[0], mn2[1], mn2[2], mn2[3]);
            *reinterpret_cast<uint4*>(&s_mm[cw][rw][1][cl * 4]) = make_uint4(mx2[0], mx2[1], mx2[2], mx2[3]);
        }
        __syncthreads();
        mnp = s_mm[cw][0][0][cl * 4 + (rl >> 1)];
        mxp = s_mm[cw][0][1][cl * 4 + (rl >> 1)];
#pragma unroll
        for (int w = 1; w < RW; ++w) {
            mnp = pk_min(mnp, s_mm[cw][w][0][cl * 4 + (rl >> 1)]);
            mxp = pk_max(mxp, s_mm[cw][w][1][cl * 4 + (rl >> 1)]);
        }
    } else {
        mnp = (rl & 4) ? ((rl & 2) ? mn2[3] : mn2[2]) : ((rl & 2) ? mn2[1] : mn2[0]);
        mxp = (rl & 4) ? ((rl & 2) ? mx2[3] : mx2[2]) : ((rl & 2) ? mx2[1] : mx2[0]);
    }
    const GroupParamsR gp = group_params_r(half_of(mnp, rl & 1), half_of(mxp, rl & 1), clip, qmax, rqmax, mfmt);
    const bool slow = __any(!gp.fast);
    if (col_ok && rw == 0) {
        const int64_t gi = int64_t(by) * in + col0 + rl;
        store_params(scales, zeros, gi, gp.scale, gp.zero, mfmt);
    }
    const bool do_pack = PB != 0 && packed != nullptr;
    if (!codes && !dW && !do_pack) return;
    QConst qc[8];
    float cs[8], nscs[8];
    uint32_t cbytes[8] = {0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u};  // codes of rows 8u + rl, byte u, per column
    const float n0 = opaque_negzero();
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        qc[i].n0 = n0;
        const int src = (i << 3) | cl;                      // the lane that worked out column 8*cl + i
        const float sc = __shfl(gp.scale, src, 64);
        const float zp = __shfl(gp.zero, src, 64);
        qc[i].y = __shfl(gp.rcp, src, 64);
        qc[i].ns = -sc;
        qc[i].nz = -zp;
        qc[i].pz = qmax - zp;
        cs[i] = 1.0f;
        nscs[i] = -sc;
    }
    if constexpr (SCALED) {
        if (col_ok) {
            const float4 a = *reinterpret_cast<const float4*>(colscale + col0);
            const float4 b = *reinterpret_cast<const float4*>(colscale + col0 + 4);
            cs[0] = a.x; cs[1] = a.y; cs[2] = a.z; cs[3] = a.w;
            cs[4] = b.x; cs[5] = b.y; cs[6] = b.z; cs[7] = b.w;
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) nscs[i] = qc[i].ns * cs[i];
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t row = row0 + 8 * u;
        const int64_t elem = row * in + col0;
        const uint32_t v[4] = {raw[u].x, raw[u].y, raw[u].z, raw[u].w};
        float k[8];
        quant_k8(v, qc, slow, k);
        if constexpr (PB != 0) {
            if (do_pack) {
#pragma unroll
                for (int i = 0; i < 8; ++i) cbytes[i] = __builtin_amdgcn_cvt_pk_u8_f32(k[i] - qc[i].nz, u, cbytes[i]);
            }
        }
        if (!col_ok) continue;
        if (codes) {
            uint32_t lo = 0, hi = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                lo |= static_cast<uint32_t>(k[i] - qc[i].nz) << (8 * i);
                hi |= static_cast<uint32_t>(k[4 + i] - qc[4 + i].nz) << (8 * i);
            }
            *reinterpret_cast<uint2*>(codes + elem) = make_uint2(lo, hi);
        }
        if (dW) {
            float d[8];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                d[2 * i] = fma_hff<0>(v[i], cs[2 * i], nscs[2 * i] * k[2 * i]);
                d[2 * i + 1] = fma_hff<1>(v[i], cs[2 * i + 1], nscs[2 * i + 1] * k[2 * i + 1]);
            }
            if (!SCALED && dW_dtype == ADADIM_DW_F32) {
                float4* p = reinterpret_cast<float4*>(static_cast<float*>(dW) + elem);
                p[0] = make_float4(d[0], d[1], d[2], d[3]);
                p[1] = make_float4(d[4], d[5], d[6], d[7]);
            } else {
                const uint4 o = make_uint4(pack_h2(d[0], d[1]), pack_h2(d[2], d[3]), pack_h2(d[4], d[5]), pack_h2(d[6], d[7]));
                const int64_t at = SCALED ? score_index(row, col0, out, in) : elem;
                *reinterpret_cast<uint4*>(static_cast<__half*>(dW) + at) = o;
            }
        }
    }
    if constexpr (PB != 0) {
        if (!do_pack) return;                                // uniform
#pragma unroll
        for (int i = 0; i < 8; ++i) s_pk[wave][rl][cl * 8 + i] = cbytes[i];
        // the patch is private to the wave and the LDS serves a wave's accesses in order
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        // lane l now takes column l of the wave: pair the row lanes (2*PB <= 8 bits per byte), then
        // field u = the 8 codes of rows 8u..8u+7, 8*PB bits, belongs at bit 8*PB*u of the PB words
        uint32_t pr[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) pr[j] = s_pk[wave][2 * j][lane] | (s_pk[wave][2 * j + 1][lane] << PB);
        uint32_t f[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            f[u] = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) f[u] |= ((pr[j] >> (8 * u)) & 0xffu) << (2 * PB * j);
        }
        uint32_t w[PB];
        if constexpr (PB == 4) {
            w[0] = f[0]; w[1] = f[1]; w[2] = f[2]; w[3] = f[3];
        } else if constexpr (PB == 2) {
            w[0] = f[0] | (f[1] << 16);
            w[1] = f[2] | (f[3] << 16);
        } else {
            w[0] = f[0] | (f[1] << 24);
            w[1] = (f[1] >> 8) | (f[2] << 16);
            w[2] = (f[2] >> 16) | (f[3] << 8);
        }
        const int64_t col = (int64_t(bx) * CSW + cw) * 64 + lane;
        if (col < in) {
            uint32_t* dst = packed + col * n_words + (int64_t(by) * (G / 32) + rw) * PB;
#pragma unroll
            for (int j = 0; j < PB; ++j) dst[j] = w[j];
        }
    }
}

template <int U, int RW, bool SCALED, int PB>
__global__ __launch_bounds__(RW <= 4 ? 256 : 64 * RW) void quant_ic_stream(
    const __half* __restrict__ W, int64_t out, int64_t in, float clip, float qmax, float rqmax, int mfmt,
    uint8_t* __restrict__ codes, float* __restrict__ scales, uint8_t* __restrict__ zeros, void* __restrict__ dW,
    int dW_dtype, const float* __restrict__ colscale, uint32_t* __restrict__ packed, int64_t n_words) {
    quant_ic_body<U, RW, SCALED, PB>(blockIdx.x, blockIdx.y, W, out, in, clip, qmax, rqmax, mfmt, codes, scales, zeros, dW,
                                     dW_dtype, colscale, packed, n_words);
}

// Both grouping dimensions of one weight in one launch (groups of g = 8*LPG in either direction, at most
// 128).  Short kernels spend a good part of their time filling and draining the chip; one launch does
// that once.  The two passes over W are arranged so that HBM is read once: W is cut into regions of g rows
// x 512 columns, a region's g/16 per-OC tiles (16 rows x 512 columns) and g/16 per-IC tiles (g rows x
// 512*16/g columns) are consecutive workgroups of ONE XCD (workgroups go to the eight XCDs round-robin by
// launch index, so XCD x takes the regions x, x + 8, ...), and they run at the same time: whichever tile
// asks for a line first brings it into that XCD's L2, the other finds it there.
struct QuantOut {
    uint8_t* codes;
    float* scales;
    uint8_t* zeros;
    void* dW;
    uint32_t* packed;
};
template <int LPG, int PB>
__global__ __launch_bounds__(256) void quant_both(const __half* __restrict__ W, int64_t out, int64_t in, float clip,
                                                  float qmax, float rqmax, int mfmt, QuantOut oc, QuantOut ic,
                                                  const float* __restrict__ colscale, int64_t n_words_ic, unsigned regions_x,
                                                  unsigned n_regions) {
    constexpr int U = LPG < 4 ? LPG : 4, RW = LPG / U;
    static_assert(RW <= 4 && LPG >= 4, "256 threads per workgroup in both halves; groups of 32 and up");
    constexpr unsigned PER = LPG / 2;                         // per-OC tiles per region = per-IC tiles per region = g/16
    const unsigned xcd = blockIdx.x % 8, seq = blockIdx.x / 8;
    const unsigned region = (seq / (2 * PER)) * 8 + xcd, within = seq % (2 * PER);
    if (region >= n_regions) return;                          // whole workgroup
    const unsigned rx = region % regions_x, ry = region / regions_x;
    if (within < PER) {
        quant_oc_body<LPG, PB, true>(rx, ry * PER + within, reinterpret_cast<const uint4*>(W), out,
                                     static_cast<int>(in / 8), clip, qmax, rqmax, mfmt, oc.codes, oc.scales, oc.zeros, oc.dW,
                                     ADADIM_DW_F16_SCALED, colscale, oc.packed);
    } else {
        quant_ic_body<U, RW, true, PB>(rx * PER + (within - PER), ry, W, out, in, clip, qmax, rqmax, mfmt, ic.codes, ic.scales,
                                       ic.zeros, ic.dW, ADADIM_DW_F16_SCALED, colscale, ic.packed, n_words_ic);
    }
}

// ---------------------------------------------------------------------------
// Wide groups (whole-channel quantization, groups longer than one workgroup can hold): three
// passes with 16-byte accesses.  (1) partial (min, -max) pairs per piece of a group, (2) one
// thread per group reduces the pieces and computes the parameters, (3) an element-wise pass
// looks the parameters up (they sit in L2) and quantizes with the streaming arithmetic.
// Group numbering is that of the scales array: per-OC row*(in/g) + column group, per-IC
// (row group)*in + column.

// per-OC pieces: one wavefront per (group, piece of up to 64 chunks = 512 columns)
__global__ __launch_bounds__(256) void wide_minmax_oc(const uint4* __restrict__ W, int64_t n_groups, int cpg,
                                                      int n_pieces, uint32_t* __restrict__ part) {
    const int lane = threadIdx.x & 63;
    const int64_t id = int64_t(blockIdx.x) * 4 + (threadIdx.x >> 6);      // (group, piece)
    if (id >= n_groups * n_pieces) return;                                 // whole wavefront leaves together
    const int64_t grp = id / n_pieces;
    const int ch = static_cast<int>(id % n_pieces) * 64 + lane;            // chunk within the group
    uint32_t m = 0u;                                                       // (0, -0): the range contains zero
    if (ch < cpg) {
        const uint4 raw = W[grp * cpg + ch];                               // groups are consecutive chunks of the flat matrix
        const uint32_t mnp = pk_min(pk_min(raw.x, raw.y), pk_min(raw.z, raw.w));
        const uint32_t nmx = pk_max(pk_max(raw.x, raw.y), pk_max(raw.z, raw.w)) ^ 0x80008000u;
        m = pk_min(__builtin_amdgcn_perm(nmx, mnp, 0x05040100u), __builtin_amdgcn_perm(nmx, mnp, 0x07060302u));
        m = pk_min(m, 0x80000000u);                                        // fold in (0, -0)
    } else {
        m = 0x80000000u;
    }
    m = cluster_min2<64>(m);
    if (lane == 0) part[id] = m;
}

// per-IC pieces: a wavefront owns 64 rows x 64 columns of one group (8 row lanes x 8 chunk lanes,
// 8 loads per lane); partials are stored [row group][piece][column]
__global__ __launch_bounds__(256) void wide_minmax_ic(const __half* __restrict__ W, int64_t out, int64_t in, int g,
                                                      int n_pieces, uint32_t* __restrict__ part) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int rl = lane >> 3, cl = lane & 7;
    const int64_t col0 = (int64_t(blockIdx.x) * 4 + wave) * 64 + cl * 8;
    const int64_t rg = blockIdx.y / n_pieces;
    const int piece = blockIdx.y % n_pieces;
    const int64_t r_end = min(out, (rg + 1) * int64_t(g));
    const int64_t r_first = rg * int64_t(g) + piece * 64 + rl;
    const bool col_ok = col0 < in;
    uint32_t mn2[4] = {0u, 0u, 0u, 0u}, mx2[4] = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        const int64_t row = r_first + 8 * u;
        if (col_ok && row < r_end) {
            const uint4 raw = *reinterpret_cast<const uint4*>(W + row * in + col0);
            const uint32_t v[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                mn2[i] = pk_min(mn2[i], v[i]);
                mx2[i] = pk_max(mx2[i], v[i]);
            }
        }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        mn2[i] = pk_min(mn2[i], dpp_u<0x128>(mn2[i]));
        mx2[i] = pk_max(mx2[i], dpp_u<0x128>(mx2[i]));
        mn2[i] = pk_min(mn2[i], static_cast<uint32_t>(__shfl_xor(static_cast<int>(mn2[i]), 16, 64)));
        mx2[i] = pk_max(mx2[i], static_cast<uint32_t>(__shfl_xor(static_cast<int>(mx2[i]), 16, 64)));
        mn2[i] = pk_min(mn2[i], static_cast<uint32_t>(__shfl_xor(static_cast<int>(mn2[i]), 32, 64)));
        mx2[i] = pk_max(mx2[i], static_cast<uint32_t>(__shfl_xor(static_cast<int>(mx2[i]), 32, 64)));
    }
    if (col_ok && rl == 0) {
        uint32_t o[8];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t nmx = mx2[i] ^ 0x80008000u;
            o[2 * i] = __builtin_amdgcn_perm(nmx, mn2[i], 0x05040100u);
            o[2 * i + 1] = __builtin_amdgcn_perm(nmx, mn2[i], 0x07060302u);
        }
        uint4* dst = reinterpret_cast<uint4*>(part + (rg * n_pieces + piece) * in + col0);
        dst[0] = make_uint4(o[0], o[1], o[2], o[3]);
        dst[1] = make_uint4(o[4], o[5], o[6], o[7]);
    }
}

// one thread per group: pieces -> parameters.  piece p of group grp is part[grp*ps_g + p*ps_p + off(grp)]
// (per-OC: grp*n_pieces + p; per-IC: (rg*n_pieces + p)*in + col)
__global__ __launch_bounds__(256) void wide_params(const uint32_t* __restrict__ part, int64_t n_groups, int n_pieces,
                                                   int64_t in, int is_ic, float clip, float qmax, float rqmax, int mfmt,
                                                   float* __restrict__ par, float* __restrict__ scales,
                                                   uint8_t* __restrict__ zeros) {
    const int64_t grp = int64_t(blockIdx.x) * 256 + threadIdx.x;
    const bool ok = grp < n_groups;                          // every lane reaches the wave-wide tests inside
    uint32_t m = 0x80000000u;
    if (ok) {
        const int64_t base = is_ic ? (grp / in) * n_pieces * in + grp % in : grp * n_pieces;
        const int64_t step = is_ic ? in : 1;
        for (int p = 0; p < n_pieces; ++p) m = pk_min(m, part[base + p * step]);
    }
    const GroupParamsR gp = group_params_r(half_of(m, 0), -half_of(m, 1), clip, qmax, rqmax, mfmt);
    if (!ok) return;
    par[grp] = gp.scale;
    par[n_groups + grp] = gp.zero;
    par[2 * n_groups + grp] = gp.rcp;
    store_params(scales, zeros, grp, gp.scale, gp.zero, mfmt);
}

// element-wise pass: one thread per 16-byte chunk of W
// PB != 0 (per-OC only; 2, 3, 4 or 8 bits, in % 32 == 0): the bit stream is written here too, as in the lane kernel.
template <bool IC, bool SCALED, int PB = 0>
__global__ __launch_bounds__(256) void wide_apply(const uint4* __restrict__ W, int64_t out, int cpr, int g,
                                                  int64_t n_groups, const float* __restrict__ par, float qmax,
                                                  uint8_t* __restrict__ codes, void* __restrict__ dW, int dW_dtype,
                                                  const float* __restrict__ colscale, uint32_t* __restrict__ packed) {
    static_assert(PB == 0 || !IC, "the per-IC stream runs across rows");
    const int64_t c = int64_t(blockIdx.x) * 256 + threadIdx.x;
    const bool valid = c < out * cpr;
    const int64_t row = valid ? c / cpr : 0;
    const int cc = valid ? static_cast<int>(c % cpr) : 0;
    const int64_t in = int64_t(cpr) * 8, col0 = int64_t(cc) * 8;
    const uint4 raw = valid ? W[c] : make_uint4(0, 0, 0, 0);
    const float n0 = opaque_negzero();
    QConst qc[8];
    float sc[8];
    bool fast = true;
    if constexpr (IC) {
        const int64_t p0 = (row / g) * in + col0;
        const float4 s0 = *reinterpret_cast<const float4*>(par + p0), s1 = *reinterpret_cast<const float4*>(par + p0 + 4);
        const float4 z0 = *reinterpret_cast<const float4*>(par + n_groups + p0);
        const float4 z1 = *reinterpret_cast<const float4*>(par + n_groups + p0 + 4);
        const float4 r0 = *reinterpret_cast<const float4*>(par + 2 * n_groups + p0);
        const float4 r1 = *reinterpret_cast<const float4*>(par + 2 * n_groups + p0 + 4);
        const float s[8] = {s0.x, s0.y, s0.z, s0.w, s1.x, s1.y, s1.z, s1.w};
        const float z[8] = {z0.x, z0.y, z0.z, z0.w, z1.x, z1.y, z1.z, z1.w};
        const float r[8] = {r0.x, r0.y, r0.z, r0.w, r1.x, r1.y, r1.z, r1.w};
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            sc[i] = s[i];
            qc[i] = {r[i], -s[i], -z[i], qmax - z[i], n0};
            fast = fast && fastdiv_ok(s[i]);
        }
    } else {
        const int64_t p = row * (in / g) + col0 / g;
        const float s = par[p], z = par[n_groups + p], r = par[2 * n_groups + p];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            sc[i] = s;
            qc[i] = {r, -s, -z, qmax - z, n0};
        }
        fast = fastdiv_ok(s);
    }
    const bool slow = __any(!fast);
    const uint32_t v[4] = {raw.x, raw.y, raw.z, raw.w};
    float k[8];
    quant_k8(v, qc, slow, k);
    if constexpr (PB != 0) {                                  // all lanes take part in the DPP
        float q[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) q[i] = k[i] - qc[i].nz;
        pack8_store<PB>(q, c, valid, packed);
    }
    if (!valid) return;
    if (codes) {
        uint32_t lo = 0, hi = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            lo |= static_cast<uint32_t>(k[i] - qc[i].nz) << (8 * i);
            hi |= static_cast<uint32_t>(k[4 + i] - qc[4 + i].nz) << (8 * i);
        }
        reinterpret_cast<uint2*>(codes)[c] = make_uint2(lo, hi);
    }
    if (dW) {
        float cs[8] = {1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f};
        if constexpr (SCALED) {
            const float4 a = *reinterpret_cast<const float4*>(colscale + col0);
            const float4 b = *reinterpret_cast<const float4*>(colscale + col0 + 4);
            cs[0] = a.x; cs[1] = a.y; cs[2] = a.z; cs[3] = a.w;
            cs[4] = b.x; cs[5] = b.y; cs[6] = b.z; cs[7] = b.w;
        }
        float d[8];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            d[2 * i] = fma_hff<0>(v[i], cs[2 * i], -(sc[2 * i] * cs[2 * i]) * k[2 * i]);
            d[2 * i + 1] = fma_hff<1>(v[i], cs[2 * i + 1], -(sc[2 * i + 1] * cs[2 * i + 1]) * k[2 * i + 1]);
        }
        if (!SCALED && dW_dtype == ADADIM_DW_F32) {
            float4* p = reinterpret_cast<float4*>(static_cast<float*>(dW) + c * 8);
            p[0] = make_float4(d[0], d[1], d[2], d[3]);
            p[1] = make_float4(d[4], d[5], d[6], d[7]);
        } else {
            const uint4 o = make_uint4(pack_h2(d[0], d[1]), pack_h2(d[2], d[3]), pack_h2(d[4], d[5]), pack_h2(d[6], d[7]));
            *reinterpret_cast<uint4*>(static_cast<__half*>(dW) + (SCALED ? score_index(row, col0, out, in) : c * 8)) = o;
        }
    }
}

// ---------------------------------------------------------------------------
// Bit-packing: one thread assembles one 32-bit word of a channel's stream.
// channel stride / element stride describe where code k of channel ch lives:
// OC: ch*in + k;  IC: k*in + ch.
__global__ __launch_bounds__(256) void pack_words(const uint8_t* __restrict__ codes, int64_t n_ch, int64_t len,
                                                  int64_t ch_stride, int64_t el_stride, int bits,
                                                  int64_t n_words, int ch_fastest,
                                                  uint32_t* __restrict__ packed) {
    const int64_t t = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (t >= n_ch * n_words) return;
    int64_t ch, wd;
    if (ch_fastest) {
        ch = t % n_ch;
        wd = t / n_ch;
    } else {
        wd = t % n_words;
        ch = t / n_words;
    }
    const int64_t bit0 = wd * 32;
    uint32_t word = 0;
    for (int64_t k = bit0 / bits; k < len && k * bits < bit0 + 32; ++k) {
        const uint32_t code = codes[ch * ch_stride + k * el_stride];
        const int sh = static_cast<int>(k * bits - bit0);
        word |= sh >= 0 ? (code << sh) : (code >> (-sh));
    }
    packed[ch * n_words + wd] = word;
}

template <int LPG>
void launch_oc_lanes(adadim_ctx* ctx, const __half* W, int64_t out, int64_t in, float clip, float qmax, int mfmt, int pb,
                     uint8_t* codes, float* scales, uint8_t* zeros, void* dW, int dW_dtype,
                     const float* colscale, uint32_t* packed) {
    const uint4* W4 = reinterpret_cast<const uint4*>(W);
    const int cpr = static_cast<int>(in / 8);
    const dim3 blocks(static_cast<unsigned>((cpr + 63) / 64), static_cast<unsigned>((out + 15) / 16));
    ProfScope prof(ctx, "quant_oc");
#define OC_GO(PB)                                                                                                  \
    do {                                                                                                           \
        if (dW && dW_dtype == ADADIM_DW_F16_SCALED)                                                                \
            hipLaunchKernelGGL((quant_oc_fast<LPG, PB, true>), blocks, dim3(256), 0, ctx->stream, W4, out, cpr,    \
                               clip, qmax, 1.0f / qmax, mfmt, codes, scales, zeros, dW, dW_dtype, colscale, packed);     \
        else                                                                                                       \
            hipLaunchKernelGGL((quant_oc_fast<LPG, PB, false>), blocks, dim3(256), 0, ctx->stream, W4, out, cpr,   \
                               clip, qmax, 1.0f / qmax, mfmt, codes, scales, zeros, dW, dW_dtype, colscale, packed);     \
    } while (0)
    switch (pb) {
        case 2: OC_GO(2); break;
        case 3: OC_GO(3); break;
        case 4: OC_GO(4); break;
        case 8: OC_GO(8); break;
        default: OC_GO(0); break;
    }
#undef OC_GO
}

// fused packing in the streaming per-IC kernel: 32-row wave tiles (groups of 32 rows and up), 2..4 bits
constexpr bool ic_stream_pack_ok(int lpg, int pb) { return lpg >= 4 && (pb == 2 || pb == 3 || pb == 4); }

// streaming per-IC kernel for a group of 8*LPG rows; pb != 0 also writes the packed stream
template <int LPG>
void launch_ic_stream(adadim_ctx* ctx, const __half* W, int64_t out, int64_t in, float clip, float qmax, int mfmt, int pb,
                      uint8_t* codes, float* scales, uint8_t* zeros, void* dW, int dW_dtype, const float* colscale,
                      uint32_t* packed, int64_t n_words) {
    const bool scaled = dW && dW_dtype == ADADIM_DW_F16_SCALED;
    const float rq = 1.0f / qmax;
    constexpr int U = LPG < 4 ? LPG : 4, RW = LPG / U, CSW = RW <= 4 ? 4 / RW : 1, TH = RW <= 4 ? 256 : 64 * RW;
    dim3 grid(static_cast<unsigned>((in + 64 * CSW - 1) / (64 * CSW)), static_cast<unsigned>(out / (8 * LPG)));
    ProfScope prof(ctx, "quant_ic");
#define IC_S(S, PB)                                                                                             \
    hipLaunchKernelGGL((quant_ic_stream<U, RW, S, PB>), grid, dim3(TH), 0, ctx->stream, W, out, in, clip, qmax,  \
                       rq, mfmt, codes, scales, zeros, dW, dW_dtype, colscale, packed, n_words)
    if constexpr (LPG >= 4) {
        if (scaled) {
            switch (pb) {
                case 2: IC_S(true, 2); return;
                case 3: IC_S(true, 3); return;
                case 4: IC_S(true, 4); return;
                default: break;
            }
        } else {
            switch (pb) {
                case 2: IC_S(false, 2); return;
                case 3: IC_S(false, 3); return;
                case 4: IC_S(false, 4); return;
                default: break;
            }
        }
    }
    if (scaled) IC_S(true, 0); else IC_S(false, 0);
#undef IC_S
}

// wide-group path (see wide_minmax_oc): in % 8 == 0; per-OC also g % 8 == 0
// pb: bits of the per-OC stream to write into `packed` along with the rest (0: none)
int launch_wide(adadim_ctx* ctx, const __half* W, int64_t out, int64_t in, int dim, int g, float clip, float qmax, int mfmt,
                uint8_t* codes, float* scales, uint8_t* zeros, void* dW, int dW_dtype, const float* colscale,
                int pb = 0, uint32_t* packed = nullptr) {
    const bool ic = dim == ADADIM_DIM_IC;
    const int64_t n_groups = ic ? (out / g) * in : out * (in / g);
    const int cpr = static_cast<int>(in / 8);
    const int n_pieces = ic ? (g + 63) / 64 : (g / 8 + 63) / 64;
    uint32_t* part = static_cast<uint32_t*>(adadim_workspace(ctx, WS_QPART, size_t(n_groups) * n_pieces * 4));
    float* par = static_cast<float*>(adadim_workspace(ctx, WS_QPAR, size_t(n_groups) * 3 * 4));
    if (!part || !par) return ADADIM_EHIP;
    ProfScope prof(ctx, ic ? "quant_ic_wide" : "quant_oc_wide");
    if (ic) {
        dim3 grid(static_cast<unsigned>((in + 255) / 256), static_cast<unsigned>((out / g) * n_pieces));
        hipLaunchKernelGGL(wide_minmax_ic, grid, dim3(256), 0, ctx->stream, W, out, in, g, n_pieces, part);
    } else {
        const int64_t waves = n_groups * n_pieces;
        hipLaunchKernelGGL(wide_minmax_oc, dim3(static_cast<unsigned>((waves + 3) / 4)), dim3(256), 0, ctx->stream,
                           reinterpret_cast<const uint4*>(W), n_groups, g / 8, n_pieces, part);
    }
    hipLaunchKernelGGL(wide_params, dim3(static_cast<unsigned>((n_groups + 255) / 256)), dim3(256), 0, ctx->stream, part,
                       n_groups, n_pieces, in, ic ? 1 : 0, clip, qmax, 1.0f / qmax, mfmt, par, scales, zeros);
    if (codes || dW || pb) {
        const unsigned blocks = static_cast<unsigned>((out * cpr + 255) / 256);
        const bool scaled = dW && dW_dtype == ADADIM_DW_F16_SCALED;
        const uint4* W4 = reinterpret_cast<const uint4*>(W);
#define WIDE_GO(IC, S, PB)                                                                                          \
    hipLaunchKernelGGL((wide_apply<IC, S, PB>), dim3(blocks), dim3(256), 0, ctx->stream, W4, out, cpr, g, n_groups, \
                       par, qmax, codes, dW, dW_dtype, colscale, packed)
#define WIDE_OC(PB)                                                                                                 \
    do {                                                                                                            \
        if (scaled) WIDE_GO(false, true, PB);                                                                       \
        else WIDE_GO(false, false, PB);                                                                             \
    } while (0)
        if (ic) { if (scaled) WIDE_GO(true, true, 0); else WIDE_GO(true, false, 0); }
        else if (pb == 2) WIDE_OC(2);
        else if (pb == 3) WIDE_OC(3);
        else if (pb == 4) WIDE_OC(4);
        else if (pb == 8) WIDE_OC(8);
        else WIDE_OC(0);
#undef WIDE_OC
#undef WIDE_GO
    }
    return ADADIM_OK;
}

}  // namespace

int launch_pack(adadim_ctx* ctx, const uint8_t* codes, int64_t out, int64_t in, int dim, int bits,
                uint32_t* packed) {
    const int64_t n_ch = dim == ADADIM_DIM_OC ? out : in;
    const int64_t len = dim == ADADIM_DIM_OC ? in : out;
    const int64_t n_words = (len * bits + 31) / 32;
    const int64_t total = n_ch * n_words;
    const unsigned blocks = static_cast<unsigned>((total + 255) / 256);
    {
        ProfScope prof(ctx, "pack_words");
        hipLaunchKernelGGL(pack_words, dim3(blocks), dim3(256), 0, ctx->stream, codes, n_ch, len,
                           dim == ADADIM_DIM_OC ? in : int64_t(1), dim == ADADIM_DIM_OC ? int64_t(1) : in, bits,
                           n_words, dim == ADADIM_DIM_IC ? 1 : 0, packed);
    }
    ADADIM_LAUNCH_CHECK(ctx, "pack_words");
    return ADADIM_OK;
}

// Both dimensions with the same group length.  One launch when both fast kernels take the shape
// (column-scaled dW for both, groups of 32, 64 or 128, in % 32 == 0, 2..4 bits if packed), else two.
int launch_quantize_both(adadim_ctx* ctx, const __half* W, int64_t out, int64_t in, int bits, int g_oc, int g_ic, float clip,
                         int mfmt, const float* colscale, uint8_t* codes_oc, float* scales_oc, uint8_t* zeros_oc,
                         void* dW_oc, uint32_t* packed_oc, uint8_t* codes_ic, float* scales_ic, uint8_t* zeros_ic,
                         void* dW_ic, uint32_t* packed_ic) {
    const int lpg = g_oc / 8;
    const bool want_pack = packed_oc || packed_ic;
    const bool fused = g_oc == g_ic && dW_oc && dW_ic && colscale && (g_oc == 32 || g_oc == 64 || g_oc == 128) &&
                       (in % 32) == 0 && (in % g_oc) == 0 && (out % g_ic) == 0 && out <= 16 * 65535 &&
                       (!want_pack || (packed_oc && packed_ic && bits >= 2 && bits <= 4));
    if (!fused) {
        int rc = launch_quantize(ctx, W, out, in, ADADIM_DIM_OC, bits, g_oc, clip, codes_oc, scales_oc, zeros_oc, dW_oc,
                                 ADADIM_DW_F16_SCALED, colscale, packed_oc, mfmt);
        if (rc != ADADIM_OK) return rc;
        return launch_quantize(ctx, W, out, in, ADADIM_DIM_IC, bits, g_ic, clip, codes_ic, scales_ic, zeros_ic, dW_ic,
                               ADADIM_DW_F16_SCALED, colscale, packed_ic, mfmt);
    }
    const float qmax = static_cast<float>((1 << bits) - 1);
    // regions of g rows x 512 columns, 2 * (g / 16) workgroups each, dealt to the XCDs round-robin
    const unsigned regions_x = static_cast<unsigned>((in + 511) / 512), regions_y = static_cast<unsigned>(out / g_oc);
    const unsigned n_regions = regions_x * regions_y, per_region = 2u * static_cast<unsigned>(lpg / 2);
    const unsigned grid = 8u * ((n_regions + 7u) / 8u) * per_region;
    const QuantOut oc = {codes_oc, scales_oc, zeros_oc, dW_oc, packed_oc}, ic = {codes_ic, scales_ic, zeros_ic, dW_ic, packed_ic};
    const int64_t n_words_ic = (out * bits + 31) / 32;
    {
        ProfScope prof(ctx, "quant_both");
#define QB_GO(L, PB)                                                                                                  \
    hipLaunchKernelGGL((quant_both<L, PB>), dim3(grid), dim3(256), 0, ctx->stream, W, out, in, clip, qmax,            \
                       1.0f / qmax, mfmt, oc, ic, colscale, n_words_ic, regions_x, n_regions)
#define QB_PB(L)                                                                                                      \
    do {                                                                                                              \
        if (!want_pack) QB_GO(L, 0);                                                                                  \
        else if (bits == 2) QB_GO(L, 2);                                                                              \
        else if (bits == 3) QB_GO(L, 3);                                                                              \
        else QB_GO(L, 4);                                                                                             \
    } while (0)
        if (lpg == 4) QB_PB(4);
        else if (lpg == 8) QB_PB(8);
        else QB_PB(16);
#undef QB_PB
#undef QB_GO
    }
    ADADIM_LAUNCH_CHECK(ctx, "quant_both");
    return ADADIM_OK;
}

int launch_quantize(adadim_ctx* ctx, const __half* W, int64_t out, int64_t in, int dim, int bits, int g,
                    float clip, uint8_t* codes, float* scales, uint8_t* zeros, void* dW, int dW_dtype,
                    const float* colscale, uint32_t* packed, int mfmt) {
    const float qmax = static_cast<float>((1 << bits) - 1);
    const bool vec = (in % 8) == 0;
    const int lpg = g / 8;
    const bool oc_lanes = dim == ADADIM_DIM_OC && vec && (g % 8) == 0 && lpg <= 64 && (lpg & (lpg - 1)) == 0 &&
                          out <= 16 * 65535;
    const bool ic_stream = dim == ADADIM_DIM_IC && vec && (g % 8) == 0 && lpg <= 32 && (lpg & (lpg - 1)) == 0;
    // the fast kernels assemble the bit stream themselves for these widths
    const bool oc_wide = dim == ADADIM_DIM_OC && !oc_lanes && vec && (g % 8) == 0 && g >= 512 &&
                         out * (in / g) <= (int64_t(1) << 30);
    const bool fused_pack =
        packed && (((oc_lanes || oc_wide) && (in % 32) == 0 && (bits == 2 || bits == 3 || bits == 4 || bits == 8)) ||
                   (ic_stream && ic_stream_pack_ok(lpg, bits)));
    if (packed && !fused_pack && !codes) {
        codes = static_cast<uint8_t*>(adadim_workspace(ctx, WS_CODES, size_t(out) * size_t(in)));
        if (!codes) return ADADIM_EHIP;
    }
    if (dim == ADADIM_DIM_OC) {
        if (oc_lanes) {
            const int pb = fused_pack ? bits : 0;
            uint32_t* pk = fused_pack ? packed : nullptr;
            switch (lpg) {
#define OC_CASE(n) case n: launch_oc_lanes<n>(ctx, W, out, in, clip, qmax, mfmt, pb, codes, scales, zeros, dW, dW_dtype, colscale, pk); break;
                OC_CASE(1) OC_CASE(2) OC_CASE(4) OC_CASE(8) OC_CASE(16) OC_CASE(32) OC_CASE(64)
#undef OC_CASE
            }
            ADADIM_LAUNCH_CHECK(ctx, "quant_oc_fast");
        } else if (oc_wide) {
            const int rc = launch_wide(ctx, W, out, in, dim, g, clip, qmax, mfmt, codes, scales, zeros, dW, dW_dtype, colscale,
                                       fused_pack ? bits : 0, fused_pack ? packed : nullptr);
            if (rc != ADADIM_OK) return rc;
            ADADIM_LAUNCH_CHECK(ctx, "quant_oc_wide");
        } else {
            const int64_t n_groups = out * (in / g);
            const unsigned blocks = static_cast<unsigned>((n_groups + 3) / 4);
            {
                ProfScope prof(ctx, "quant_oc_generic");
                hipLaunchKernelGGL(quant_oc_generic, dim3(blocks), dim3(256), 0, ctx->stream, W, n_groups, g, out, in,
                                   clip, qmax, mfmt, codes, scales, zeros, dW, dW_dtype, colscale);
            }
            ADADIM_LAUNCH_CHECK(ctx, "quant_oc_generic");
        }
    } else {
        const int64_t row_groups = out / g;
        if (row_groups > 65535)
            return adadim_fail(ctx, ADADIM_EINVAL, "adadim_quantize: more than 65535 row groups per column");
        if (ic_stream) {
            const int pb = fused_pack ? bits : 0;
            uint32_t* pk = fused_pack ? packed : nullptr;
            const int64_t n_words = (out * bits + 31) / 32;
            switch (lpg) {
#define IC_CASE(n)                                                                                              \
    case n:                                                                                                     \
        launch_ic_stream<n>(ctx, W, out, in, clip, qmax, mfmt, pb, codes, scales, zeros, dW, dW_dtype, colscale, pk,  \
                            n_words);                                                                           \
        break;
                IC_CASE(1) IC_CASE(2) IC_CASE(4) IC_CASE(8) IC_CASE(16) IC_CASE(32)
#undef IC_CASE
            }
            ADADIM_LAUNCH_CHECK(ctx, "quant_ic_stream");
        } else if (vec && g >= 256 && row_groups * ((g + 63) / 64) <= 65535) {
            const int rc = launch_wide(ctx, W, out, in, dim, g, clip, qmax, mfmt, codes, scales, zeros, dW, dW_dtype, colscale);
            if (rc != ADADIM_OK) return rc;
            ADADIM_LAUNCH_CHECK(ctx, "quant_ic_wide");
        } else if (vec) {
            dim3 grid(static_cast<unsigned>((in + 255) / 256), static_cast<unsigned>(row_groups));
            {
                ProfScope prof(ctx, "quant_ic_tile");
                hipLaunchKernelGGL(quant_ic_tile<8>, grid, dim3(256), 0, ctx->stream, W, out, in, g, clip, qmax, mfmt, codes,
                                   scales, zeros, dW, dW_dtype, colscale);
            }
            ADADIM_LAUNCH_CHECK(ctx, "quant_ic_tile");
        } else {
            dim3 grid(static_cast<unsigned>((in + 31) / 32), static_cast<unsigned>(row_groups));
            {
                ProfScope prof(ctx, "quant_ic_tile");
                hipLaunchKernelGGL(quant_ic_tile<1>, grid, dim3(256), 0, ctx->stream, W, out, in, g, clip, qmax, mfmt, codes,
                                   scales, zeros, dW, dW_dtype, colscale);
            }
            ADADIM_LAUNCH_CHECK(ctx, "quant_ic_tile");
        }
    }
    if (packed && !fused_pack) return launch_pack(ctx, codes, out, in, dim, bits, packed);
    return ADADIM_OK;
}
