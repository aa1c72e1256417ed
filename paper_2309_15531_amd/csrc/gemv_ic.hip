// De-quantizing matrix-vector product for per-IC quantized weights (paper Sec. 4.5, App. D):
//     y[o] = sum_j scale[o/g, j] * (code[o, j] - zero[o/g, j]) * x[j]
// from the packed stream adadim_quantize(dim = IC) writes: [in, out*b/32] words, the codes of
// one input column consecutive along the output axis.  Batch 1: every weight bit is read once
// and used once, so the kernel is bound by HBM reads.
//
// The paper's kernel builds look-up tables of scale*activation products; on gfx950 a direct
// form is simpler and reads the same bytes: with a[r, j] = scale[r, j] * x[j] (the per-IC
// scale folded into the activation, as the paper does when it fills its tables)
//     y[o] = sum_j a[o/g, j] * code[o, j]  -  sum_j a[o/g, j] * zero[o/g, j].
// A lane owns 32 consecutive outputs (b words of every column, one 16-byte load for b = 4), a
// wavefront 2048, so the codes of a column are read in contiguous kilobytes and no sum crosses
// lanes; the second sum costs one fma per lane and column.  Columns are split over the eight
// waves of a block and over blocks; partial outputs are added up in a fixed order (LDS inside
// a block; across blocks by a second small kernel, chunk by chunk), so the result is
// reproducible.  (Letting the last block of an output tile do that sum needs device-scope
// fences, which write back and invalidate the XCD's whole L2 each time: 3x slower overall.)
#include "common.h"

#include <algorithm>

namespace {

constexpr int GV_WAVES = 8, GV_OUT_PER_BLOCK = 64 * 32;
// Two blocks fit a compute unit (registers and LDS), 512 on the chip.  The columns are dealt to
// blocks so that one launch is a whole number of such rounds as nearly as can be: a grid a little
// larger than that would run a second, mostly empty round (576 blocks took two rounds for the work
// of 1.1), and the kernel is short enough for that to cost a third of its time.
constexpr int GV_BLOCK_SLOTS = 512, GV_MIN_COLS_PER_WAVE = 32;

template <int PB>
struct Words {
    uint32_t w[PB];
};

template <int PB>
__device__ __forceinline__ Words<PB> load_words(const uint32_t* p) {
    Words<PB> r;
    if constexpr (PB == 4) {
        const uint4 v = *reinterpret_cast<const uint4*>(p);
        r.w[0] = v.x; r.w[1] = v.y; r.w[2] = v.z; r.w[3] = v.w;
    } else if constexpr (PB == 2) {
        const uint2 v = *reinterpret_cast<const uint2*>(p);
        r.w[0] = v.x; r.w[1] = v.y;
    } else {
#pragma unroll
        for (int i = 0; i < PB; ++i) r.w[i] = p[i];
    }
    return r;
}

// float(byte n of v).  `v` must be opaque to the optimiser (see hide()), or it rewrites the
// mask-then-byte sequence into a bit-field extract plus a conversion, one instruction more per code.
__device__ __forceinline__ float ubyte(uint32_t v, int n) { return static_cast<float>((v >> (8 * n)) & 0xffu); }
__device__ __forceinline__ uint32_t hide(uint32_t v) {
    asm("" : "+v"(v));
    return v;
}
// (v & mask) | orc in one instruction: the encoding takes one scalar operand, so the mask travels in a scalar
// register and the or-constant in a vector register (see hide()); left alone the compiler emits an and and an or,
// each with a literal
__device__ __forceinline__ uint32_t and_or(uint32_t v, uint32_t mask, uint32_t orc) {
    uint32_t r;
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(r) : "v"(v), "s"(mask), "v"(orc));
    return r;
}

__device__ __forceinline__ __half2 as_half2(uint32_t v) { return *reinterpret_cast<const __half2*>(&v); }
// bit pattern of the fp16 value 2^e
__host__ __device__ constexpr uint32_t f16_exp2(int e) { return static_cast<uint32_t>(e + 15) << 10; }

// 3-bit extraction plan.  Stream t (0: as stored, 1: shifted right by 8), word w, step q takes the field that starts
// at bit f3_s(c, q, 0) of the low half and the one at f3_s(c, q, 1) of the high half (-1: none), c = f3_class(t, w);
// the code's index follows from its bit position.
__host__ __device__ constexpr int f3_s(int c, int q, int h) {
    constexpr int S[3][3][2] = {{{0, 2}, {3, 5}, {6, -1}}, {{1, 0}, {4, 3}, {7, 6}}, {{2, 1}, {5, 4}, {-1, 7}}};
    return S[c][q][h];
}
__host__ __device__ constexpr int f3_class(int t, int w) { return (w + t) % 3; }
__host__ __device__ constexpr uint32_t f3_mask(int c, int q) {
    return (f3_s(c, q, 0) >= 0 ? 7u << f3_s(c, q, 0) : 0u) | (f3_s(c, q, 1) >= 0 ? 7u << (16 + f3_s(c, q, 1)) : 0u);
}
__host__ __device__ constexpr uint32_t f3_orc(int c, int q) {
    return (f3_s(c, q, 0) >= 0 ? f16_exp2(10 - f3_s(c, q, 0)) : 0u) |
           (f3_s(c, q, 1) >= 0 ? f16_exp2(10 - f3_s(c, q, 1)) << 16 : 0u);
}
// index of the code whose field starts at bit s of half h of word w of stream t
__host__ __device__ constexpr int f3_code(int t, int w, int h, int s) { return (32 * w + 16 * h + s + 8 * t) / 3; }

// what a code was read as, minus the code: the constant that leaves with the zero-point sum
template <int PB>
__host__ __device__ constexpr float code_offset(int k) {
    if (PB == 4) return (k & 1) ? 64.0f : 1024.0f;
    if (PB == 2) {
        const int f = k & 7;                                  // field within its half: 0..4 direct, 5..7 shifted by 10
        return static_cast<float>(1024 >> (2 * (f < 5 ? f : f - 5)));
    }
    const int b = 3 * k, t = (b & 15) <= 7 ? 0 : 1;           // PB == 3
    return static_cast<float>(1024 >> ((b - 8 * t) & 15));
}

// one step of the plan; t, w, q are constants where this is called (fully unrolled loops)
__device__ __forceinline__ void f3_step(int t, int w, int q, uint32_t word, const uint32_t (&orc)[9], float a,
                                        float (&acc)[32]) {
    const int c = f3_class(t, w);
    const __half2 h = as_half2(and_or(word, f3_mask(c, q), orc[3 * c + q]));
    if (f3_s(c, q, 0) >= 0) {
        const int k = f3_code(t, w, 0, f3_s(c, q, 0));
        acc[k] = fmaf(__low2float(h), a, acc[k]);
    }
    if (f3_s(c, q, 1) >= 0) {
        const int k = f3_code(t, w, 1, f3_s(c, q, 1));
        acc[k] = fmaf(__high2float(h), a, acc[k]);
    }
}

// acc[k] += a * (code k of the lane's 32 codes + code_offset(k))
template <int PB>
__device__ __forceinline__ void accumulate(const Words<PB>& wd, float a, float (&acc)[32]) {
    if constexpr (PB == 4) {
        // A nibble placed in the low fraction bits of an fp16 pattern is that code plus a constant: bits 0..3
        // under the exponent of [1024, 2048) read 1024 + code, bits 4..7 under that of [64, 128) read 64 + code.
        // One and-or builds two such halves, and v_fma_mix_f32 takes either half as an operand, so a code costs
        // 5/8 + 1 instructions and no conversion.  The constants leave with the zero-point sum (see OFFSET).
        const uint32_t c1024 = hide(0x64006400u), c64 = hide(0x54005400u);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t w0 = wd.w[i], w8 = w0 >> 8;
            const uint32_t p[4] = {and_or(w0, 0x000F000Fu, c1024), and_or(w0, 0x00F000F0u, c64),
                                   and_or(w8, 0x000F000Fu, c1024), and_or(w8, 0x00F000F0u, c64)};
#pragma unroll
            for (int n = 0; n < 4; ++n) {
                const __half2 h = *reinterpret_cast<const __half2*>(&p[n]);
                acc[8 * i + n] = fmaf(__low2float(h), a, acc[8 * i + n]);           // nibble n
                acc[8 * i + n + 4] = fmaf(__high2float(h), a, acc[8 * i + n + 4]);   // nibble n + 4
            }
        }
    } else if constexpr (PB == 2) {
        // same scheme: a field at bits s..s+1 of a 16-bit half, s = 0, 2, .. 8, reads code + 2^(10-s); the fields
        // at 10, 12, 14 are taken from the word shifted right by 10
        uint32_t orc[5];
#pragma unroll
        for (int q = 0; q < 5; ++q) orc[q] = hide(f16_exp2(10 - 2 * q) * 0x10001u);
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const uint32_t w0 = wd.w[i], w10 = w0 >> 10;
#pragma unroll
            for (int q = 0; q < 5; ++q) {                    // fields 0..4 of either half
                const __half2 h = as_half2(and_or(w0, 0x00030003u << (2 * q), orc[q]));
                acc[16 * i + q] = fmaf(__low2float(h), a, acc[16 * i + q]);
                acc[16 * i + 8 + q] = fmaf(__high2float(h), a, acc[16 * i + 8 + q]);
            }
#pragma unroll
            for (int q = 0; q < 3; ++q) {                    // fields 5..7
                const __half2 h = as_half2(and_or(w10, 0x00030003u << (2 * q), orc[q]));
                acc[16 * i + 5 + q] = fmaf(__low2float(h), a, acc[16 * i + 5 + q]);
                acc[16 * i + 13 + q] = fmaf(__high2float(h), a, acc[16 * i + 13 + q]);
            }
        }
    } else {
        static_assert(PB == 3, "2, 3 or 4 bits");
        // 3-bit codes: code k sits at bit 3k of the 96-bit stream.  A field can be read as an fp16 pattern when it
        // starts at bit 0..7 of a 16-bit half (code + 2^(10-s)); every code does so either in the stream as it is
        // (3k mod 16 < 8) or in the stream shifted right by 8 bits.  One and-or takes a field from each half of a
        // word, so the 32 codes cost 18 of them and three funnel shifts.
        const uint32_t st[2][3] = {{wd.w[0], wd.w[1], wd.w[2]},
                                   {__builtin_amdgcn_alignbit(wd.w[1], wd.w[0], 8), __builtin_amdgcn_alignbit(wd.w[2], wd.w[1], 8),
                                    wd.w[2] >> 8}};
        uint32_t orc[9];
#pragma unroll
        for (int q = 0; q < 9; ++q) orc[q] = hide(f3_orc(q / 3, q % 3));
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int w = 0; w < 3; ++w)
#pragma unroll
                for (int q = 0; q < 3; ++q) f3_step(t, w, q, st[t][w], orc, a, acc);
    }
}

// M16: the group parameters come as one 16-bit word per (group, column) in `scales` (the
// fp16 pattern of the scale without its sign bit and its PB-1 lowest bits, above the PB-bit
// zero-point) instead of an fp32 scale and a u8 zero-point.
template <int PB, bool M16>
__global__ __launch_bounds__(64 * GV_WAVES) void gemv_ic_tiles(const uint32_t* __restrict__ packed,
                                                               const void* __restrict__ scales,
                                                               const uint8_t* __restrict__ zeros,
                                                               const __half* __restrict__ x, int64_t out, int64_t in,
                                                               int g, int64_t n_words, float* __restrict__ part) {
    __shared__ float s_acc[GV_WAVES][32][65];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t o_lane = int64_t(blockIdx.x) * GV_OUT_PER_BLOCK + lane * 32;
    const bool valid = o_lane < out;                         // out % 32 == 0: a lane's outputs are inside together
    // (32-bit divisions: out and in are below 2^24)
    const int64_t r = valid ? static_cast<uint32_t>(o_lane) / static_cast<uint32_t>(g) : 0;
    // the in/4 column quads split evenly over the gridDim.y * 8 waves that share this output tile: the first
    // `quads % waves` waves take one quad more
    const uint32_t n_wv = gridDim.y * GV_WAVES, wv = blockIdx.y * GV_WAVES + wave, quads = static_cast<uint32_t>(in >> 2);
    const uint32_t q_each = quads / n_wv, q_more = quads - q_each * n_wv;
    const int64_t j_begin = int64_t(wv * q_each + min(wv, q_more)) << 2;
    const int64_t j_end = int64_t((wv + 1) * q_each + min(wv + 1, q_more)) << 2;
    const uint32_t* wp = packed + (valid ? (o_lane >> 5) * PB : 0);
    float acc[32];
#pragma unroll
    for (int k = 0; k < 32; ++k) acc[k] = 0.0f;
    float zsum = 0.0f, asum = 0.0f;                           // sums of a * zero and of a
    // four columns per step, the next step's loads issued before this step's arithmetic
    struct Step {
        Words<PB> wd[4];
        float4 s4;
        uint32_t z4;
        uint2 m4;
        uint2 xr;
    };
    auto fetch = [&](Step& st, int64_t j0) {
#pragma unroll
        for (int c = 0; c < 4; ++c) st.wd[c] = load_words<PB>(wp + (j0 + c) * n_words);
        if constexpr (M16) {
            st.m4 = *reinterpret_cast<const uint2*>(static_cast<const uint16_t*>(scales) + r * in + j0);
        } else {
            st.s4 = *reinterpret_cast<const float4*>(static_cast<const float*>(scales) + r * in + j0);
            st.z4 = *reinterpret_cast<const uint32_t*>(zeros + r * in + j0);
        }
        st.xr = *reinterpret_cast<const uint2*>(x + j0);
    };
    auto consume = [&](const Step& st) {
        const float2 x01 = __half22float2(*reinterpret_cast<const __half2*>(&st.xr.x));
        const float2 x23 = __half22float2(*reinterpret_cast<const __half2*>(&st.xr.y));
        float a[4], z[4];
        if constexpr (M16) {
            // both words of a register at once: shifted right by one, the kept pattern bits of each
            // word land on their fp16 positions and the mask clears what crossed over
            constexpr uint32_t KEEP = (0x7FFFu & ~((1u << (PB - 1)) - 1u)) * 0x10001u, ZM = (1u << PB) - 1u;
            const uint32_t h01 = (st.m4.x >> 1) & KEEP, h23 = (st.m4.y >> 1) & KEEP;
            const float2 s01 = __half22float2(*reinterpret_cast<const __half2*>(&h01));
            const float2 s23 = __half22float2(*reinterpret_cast<const __half2*>(&h23));
            a[0] = s01.x * x01.x; a[1] = s01.y * x01.y; a[2] = s23.x * x23.x; a[3] = s23.y * x23.y;
            z[0] = static_cast<float>(st.m4.x & ZM); z[1] = static_cast<float>((st.m4.x >> 16) & ZM);
            z[2] = static_cast<float>(st.m4.y & ZM); z[3] = static_cast<float>((st.m4.y >> 16) & ZM);
        } else {
            a[0] = st.s4.x * x01.x; a[1] = st.s4.y * x01.y; a[2] = st.s4.z * x23.x; a[3] = st.s4.w * x23.y;
#pragma unroll
            for (int c = 0; c < 4; ++c) z[c] = ubyte(st.z4, c);
        }
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            zsum = fmaf(a[c], z[c], zsum);
            asum += a[c];
            accumulate<PB>(st.wd[c], a[c], acc);
        }
    };
    if (valid && j_begin < j_end) {
        // three buffers, no copies: one is consumed while the other two are in flight (two steps of 2 to 4 KB per
        // wave are too little to keep the memory system busy with 2- and 3-bit codes).  Fetches past the end
        // re-read the chunk's last columns and are not consumed.
        const int64_t j_last = j_end - 4;
        Step A, B2, C;
        fetch(A, j_begin);
        fetch(B2, min(j_begin + 4, j_last));
        for (int64_t j0 = j_begin; j0 < j_end; j0 += 12) {   // in % 4 == 0
            fetch(C, min(j0 + 8, j_last));
            consume(A);
            fetch(A, min(j0 + 12, j_last));
            if (j0 + 4 < j_end) consume(B2);
            fetch(B2, min(j0 + 16, j_last));
            if (j0 + 8 < j_end) consume(C);
        }
    }
    // OFFSET: the codes were read as code + code_offset(k)
#pragma unroll
    for (int k = 0; k < 32; ++k) {
        s_acc[wave][k][lane] = (acc[k] - code_offset<PB>(k) * asum) - zsum;
    }
    __syncthreads();
    // thread t adds up the waves for outputs 4t .. 4t+3 of the block's 2048
    const int t = threadIdx.x;
    const int64_t o0 = int64_t(blockIdx.x) * GV_OUT_PER_BLOCK + 4 * t;
    const bool o_ok = o0 < out;                               // out % 4 == 0
    if (o_ok) {
        float v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int ol = 4 * t + e, ln = ol >> 5, k = ol & 31;
            float sum = 0.0f;
#pragma unroll
            for (int w = 0; w < GV_WAVES; ++w) sum += s_acc[w][k][ln];
            v[e] = sum;
        }
        *reinterpret_cast<float4*>(part + int64_t(blockIdx.y) * out + o0) = make_float4(v[0], v[1], v[2], v[3]);
    }
}

// y[o] = fp16 of the chunk sums in chunk order; one thread per four outputs
__global__ __launch_bounds__(256) void gemv_ic_finish(const float* __restrict__ part, int n_chunks, int64_t out,
                                                      __half* __restrict__ y) {
    const int64_t o0 = (int64_t(blockIdx.x) * 256 + threadIdx.x) * 4;
    if (o0 >= out) return;                                    // out % 4 == 0
    float4 sum = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
#pragma unroll 4
    for (int c = 0; c < n_chunks; ++c) {
        const float4 p = *reinterpret_cast<const float4*>(part + int64_t(c) * out + o0);
        sum.x += p.x; sum.y += p.y; sum.z += p.z; sum.w += p.w;
    }
    uint2 o;
    *reinterpret_cast<__half2*>(&o.x) = __floats2half2_rn(sum.x, sum.y);
    *reinterpret_cast<__half2*>(&o.y) = __floats2half2_rn(sum.z, sum.w);
    *reinterpret_cast<uint2*>(y + o0) = o;
}

}  // namespace

int launch_gemv_ic(adadim_ctx* ctx, const uint32_t* packed, const void* scales, const uint8_t* zeros, const __half* x,
                   int64_t out, int64_t in, int bits, int g, __half* y, bool meta16) {
    const int n_tiles = static_cast<int>((out + GV_OUT_PER_BLOCK - 1) / GV_OUT_PER_BLOCK);
    // whole rounds of GV_BLOCK_SLOTS blocks, each wave keeping at least GV_MIN_COLS_PER_WAVE columns
    const int64_t max_chunks = std::max<int64_t>(1, in / (GV_WAVES * GV_MIN_COLS_PER_WAVE));
    const int64_t rounds = (n_tiles + GV_BLOCK_SLOTS - 1) / GV_BLOCK_SLOTS;
    const int n_chunks = static_cast<int>(std::min<int64_t>(max_chunks, std::max<int64_t>(1, rounds * GV_BLOCK_SLOTS / n_tiles)));
    float* part = static_cast<float*>(adadim_workspace(ctx, WS_GEMV_PART, size_t(n_chunks) * size_t(out) * sizeof(float)));
    if (!part) return ADADIM_EHIP;
    const int64_t n_words = out * bits / 32;
    const dim3 grid(static_cast<unsigned>(n_tiles), static_cast<unsigned>(n_chunks));
    {
        ProfScope prof(ctx, "gemv_ic_tiles");
#define GV_GO(PB)                                                                                                   \
    do {                                                                                                            \
        if (meta16)                                                                                                 \
            hipLaunchKernelGGL((gemv_ic_tiles<PB, true>), grid, dim3(64 * GV_WAVES), 0, ctx->stream, packed, scales, \
                               zeros, x, out, in, g, n_words, part);                                                \
        else                                                                                                        \
            hipLaunchKernelGGL((gemv_ic_tiles<PB, false>), grid, dim3(64 * GV_WAVES), 0, ctx->stream, packed, scales, \
                               zeros, x, out, in, g, n_words, part);                                                \
    } while (0)
        switch (bits) {
            case 2: GV_GO(2); break;
            case 3: GV_GO(3); break;
            default: GV_GO(4); break;
        }
#undef GV_GO
    }
    ADADIM_LAUNCH_CHECK(ctx, "gemv_ic_tiles");
    {
        ProfScope prof(ctx, "gemv_ic_finish");
        hipLaunchKernelGGL(gemv_ic_finish, dim3(static_cast<unsigned>((out / 4 + 255) / 256)), dim3(256), 0, ctx->stream,
                           part, n_chunks, out, y);
    }
    ADADIM_LAUNCH_CHECK(ctx, "gemv_ic_finish");
    return ADADIM_OK;
}
