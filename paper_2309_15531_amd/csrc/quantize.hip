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

namespace {

struct GroupParams {
    float scale;
    float zero;
};

__device__ __forceinline__ GroupParams group_params(float mn, float mx, float clip, float qmax) {
    mx = fmaxf(mx, 0.0f);
    mn = fminf(mn, 0.0f);
    mx = clip * mx;
    mn = clip * mn;
    const float range = mx - mn;
    float scale = range / qmax;
    if (range == 0.0f) scale = 1.0f;
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

// Stores 8 consecutive dW values of one row starting at column `col`.
__device__ __forceinline__ void store_dw8(void* dW, int dW_dtype, const float* __restrict__ colscale,
                                          int64_t elem, int64_t col, const float (&d)[8]) {
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
        *reinterpret_cast<uint4*>(static_cast<__half*>(dW) + elem) = o;
    }
}

__device__ __forceinline__ void store_dw1(void* dW, int dW_dtype, const float* __restrict__ colscale,
                                          int64_t elem, int64_t col, float d) {
    if (dW_dtype == ADADIM_DW_F32) {
        static_cast<float*>(dW)[elem] = d;
    } else {
        if (dW_dtype == ADADIM_DW_F16_SCALED) d = d * colscale[col];
        static_cast<__half*>(dW)[elem] = __float2half_rn(d);
    }
}

// ---------------------------------------------------------------------------
// per-OC, group = 8*LPG contiguous halfs: LPG adjacent lanes own one group,
// each lane 8 halfs (one 16-byte load).  W is addressed as a flat array of
// 16-byte chunks because groups never straddle rows.
template <int LPG>
__global__ __launch_bounds__(256) void quant_oc_lanes(const uint4* __restrict__ W, int64_t n_chunks,
                                                      int chunks_per_row, float clip, float qmax,
                                                      uint8_t* __restrict__ codes, float* __restrict__ scales,
                                                      uint8_t* __restrict__ zeros, void* __restrict__ dW,
                                                      int dW_dtype, const float* __restrict__ colscale) {
    const int64_t c = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    const bool valid = c < n_chunks;
    float w[8];
    uint4 raw = make_uint4(0, 0, 0, 0);
    if (valid) raw = W[c];
    unpack8(raw, w);
    float mn = w[0], mx = w[0];
#pragma unroll
    for (int i = 1; i < 8; ++i) {
        mn = fminf(mn, w[i]);
        mx = fmaxf(mx, w[i]);
    }
#pragma unroll
    for (int m = 1; m < LPG; m <<= 1) {
        mn = fminf(mn, __shfl_xor(mn, m, 64));
        mx = fmaxf(mx, __shfl_xor(mx, m, 64));
    }
    if (!valid) return;
    const GroupParams gp = group_params(mn, mx, clip, qmax);
    if ((c & (LPG - 1)) == 0) {
        const int64_t grp = c / LPG;
        if (scales) scales[grp] = gp.scale;
        if (zeros) zeros[grp] = static_cast<uint8_t>(gp.zero);
    }
    float q[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) q[i] = quant_code(w[i], gp.scale, gp.zero, qmax);
    if (codes) {
        uint32_t lo = 0, hi = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            lo |= static_cast<uint32_t>(q[i]) << (8 * i);
            hi |= static_cast<uint32_t>(q[4 + i]) << (8 * i);
        }
        reinterpret_cast<uint2*>(codes)[c] = make_uint2(lo, hi);
    }
    if (dW) {
        float d[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) d[i] = weight_error(w[i], q[i], gp.scale, gp.zero);
        const int64_t col = (c % chunks_per_row) * 8;
        store_dw8(dW, dW_dtype, colscale, c * 8, col, d);
    }
}

// per-OC, any group length: one wavefront per group, element-wise accesses.
__global__ __launch_bounds__(256) void quant_oc_generic(const __half* __restrict__ W, int64_t n_groups, int g,
                                                        int64_t in, float clip, float qmax,
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
    const GroupParams gp = group_params(mn, mx, clip, qmax);
    if (lane == 0) {
        if (scales) scales[grp] = gp.scale;
        if (zeros) zeros[grp] = static_cast<uint8_t>(gp.zero);
    }
    for (int i = lane; i < g; i += 64) {
        const float w = __half2float(W[base + i]);
        const float q = quant_code(w, gp.scale, gp.zero, qmax);
        if (codes) codes[base + i] = static_cast<uint8_t>(q);
        if (dW) store_dw1(dW, dW_dtype, colscale, base + i, (base + i) % in, weight_error(w, q, gp.scale, gp.zero));
    }
}

// ---------------------------------------------------------------------------
// per-IC: a block owns the g rows of one row-group and COLS = 32*VEC adjacent
// columns.  Lane x of row-slice y scans rows y, y+8, ... of its VEC columns,
// the 8 slices are combined through LDS, the column parameters are computed
// once, and a second sweep (served by L2) quantizes.
template <int VEC>
__global__ __launch_bounds__(256) void quant_ic_tile(const __half* __restrict__ W, int64_t in, int g,
                                                     float clip, float qmax, uint8_t* __restrict__ codes,
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
        const GroupParams gp = group_params(a, b, clip, qmax);
        s_scale[cidx] = gp.scale;
        s_zero[cidx] = gp.zero;
        const int64_t col = int64_t(blockIdx.x) * COLS + cidx;
        if (col < in) {
            const int64_t gi = int64_t(blockIdx.y) * in + col;
            if (scales) scales[gi] = gp.scale;
            if (zeros) zeros[gi] = static_cast<uint8_t>(gp.zero);
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
                store_dw8(dW, dW_dtype, colscale, elem, col0, d);
            }
        } else {
            const float w = __half2float(W[elem]);
            const float q = quant_code(w, sc[0], zp[0], qmax);
            if (codes) codes[elem] = static_cast<uint8_t>(q);
            if (dW) store_dw1(dW, dW_dtype, colscale, elem, col0, weight_error(w, q, sc[0], zp[0]));
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
void launch_oc_lanes(adadim_ctx* ctx, const __half* W, int64_t out, int64_t in, float clip, float qmax,
                     uint8_t* codes, float* scales, uint8_t* zeros, void* dW, int dW_dtype,
                     const float* colscale) {
    const int64_t n_chunks = out * in / 8;
    const unsigned blocks = static_cast<unsigned>((n_chunks + 255) / 256);
    {
        ProfScope prof(ctx, "quant_oc_lanes");
        hipLaunchKernelGGL(quant_oc_lanes<LPG>, dim3(blocks), dim3(256), 0, ctx->stream,
                           reinterpret_cast<const uint4*>(W), n_chunks, static_cast<int>(in / 8), clip, qmax, codes,
                           scales, zeros, dW, dW_dtype, colscale);
    }
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

int launch_quantize(adadim_ctx* ctx, const __half* W, int64_t out, int64_t in, int dim, int bits, int g,
                    float clip, uint8_t* codes, float* scales, uint8_t* zeros, void* dW, int dW_dtype,
                    const float* colscale, uint32_t* packed) {
    const float qmax = static_cast<float>((1 << bits) - 1);
    if (packed && !codes) {
        codes = static_cast<uint8_t*>(adadim_workspace(ctx, WS_CODES, size_t(out) * size_t(in)));
        if (!codes) return ADADIM_EHIP;
    }
    const bool vec = (in % 8) == 0;
    if (dim == ADADIM_DIM_OC) {
        const int lpg = g / 8;
        const bool lanes = vec && (g % 8) == 0 && lpg <= 64 && (lpg & (lpg - 1)) == 0;
        if (lanes) {
            switch (lpg) {
#define OC_CASE(n) case n: launch_oc_lanes<n>(ctx, W, out, in, clip, qmax, codes, scales, zeros, dW, dW_dtype, colscale); break;
                OC_CASE(1) OC_CASE(2) OC_CASE(4) OC_CASE(8) OC_CASE(16) OC_CASE(32) OC_CASE(64)
#undef OC_CASE
            }
            ADADIM_LAUNCH_CHECK(ctx, "quant_oc_lanes");
        } else {
            const int64_t n_groups = out * (in / g);
            const unsigned blocks = static_cast<unsigned>((n_groups + 3) / 4);
            {
                ProfScope prof(ctx, "quant_oc_generic");
                hipLaunchKernelGGL(quant_oc_generic, dim3(blocks), dim3(256), 0, ctx->stream, W, n_groups, g, in,
                                   clip, qmax, codes, scales, zeros, dW, dW_dtype, colscale);
            }
            ADADIM_LAUNCH_CHECK(ctx, "quant_oc_generic");
        }
    } else {
        const int64_t row_groups = out / g;
        if (row_groups > 65535)
            return adadim_fail(ctx, ADADIM_EINVAL, "adadim_quantize: more than 65535 row groups per column");
        if (vec) {
            dim3 grid(static_cast<unsigned>((in + 255) / 256), static_cast<unsigned>(row_groups));
            {
                ProfScope prof(ctx, "quant_ic_tile");
                hipLaunchKernelGGL(quant_ic_tile<8>, grid, dim3(256), 0, ctx->stream, W, in, g, clip, qmax, codes,
                                   scales, zeros, dW, dW_dtype, colscale);
            }
        } else {
            dim3 grid(static_cast<unsigned>((in + 31) / 32), static_cast<unsigned>(row_groups));
            {
                ProfScope prof(ctx, "quant_ic_tile");
                hipLaunchKernelGGL(quant_ic_tile<1>, grid, dim3(256), 0, ctx->stream, W, in, g, clip, qmax, codes,
                                   scales, zeros, dW, dW_dtype, colscale);
            }
        }
        ADADIM_LAUNCH_CHECK(ctx, "quant_ic_tile");
    }
    if (packed) return launch_pack(ctx, codes, out, in, dim, bits, packed);
    return ADADIM_OK;
}
