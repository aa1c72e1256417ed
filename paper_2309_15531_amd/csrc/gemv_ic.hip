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
#include "code_fields.h"

#include <algorithm>

namespace {

constexpr int GV_WAVES = 8, GV_OUT_PER_BLOCK = 64 * 32;
// One block per compute unit, 256 on the chip (two would fit by registers and LDS, but half as many blocks with
// twice the columns each are 5 % faster on the App. D shape: half the dispatches, half the partial sums, and eight
// waves with two steps in flight each already keep the memory system busy).  The columns are dealt to blocks so
// that one launch is a whole number of such rounds as nearly as can be: a grid a little larger than that would run
// a second, mostly empty round, and the kernel is short enough for that to cost a third of its time.
constexpr int GV_BLOCK_SLOTS = 256, GV_MIN_COLS_PER_WAVE = 32;
constexpr int GV_NBUF = 3;                 // load buffers taken in turn (4 to 6 were measured: no faster)

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

// float(byte n of v)
__device__ __forceinline__ float ubyte(uint32_t v, int n) { return static_cast<float>((v >> (8 * n)) & 0xffu); }
// the value in a vector register, opaque to the optimiser (a constant stays a register operand)
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
// acc[k] += a * (code k of the lane's 32 codes + code_offset(k)): the plan of code_fields.h, unrolled.  The
// exponent constants sit in vector registers, the masks become scalar operands (see and_or).
template <int PB>
__device__ __forceinline__ void accumulate(const Words<PB>& wd, float a, float (&acc)[32]) {
    static_assert(PB >= 2 && PB <= 4, "2, 3 or 4 bits");
    constexpr int NS = field_steps<PB>(), NO = field_orcs<PB>();
    uint32_t orc[NO];
#pragma unroll
    for (int q = 0; q < NO; ++q) orc[q] = hide(field_orc<PB>(q));
    // the words as stored and shifted: per word for 4 and 2 bits (by 8, by 10), across words for 3 bits (by 8)
    uint32_t src[PB][2];
#pragma unroll
    for (int w = 0; w < PB; ++w) {
        src[w][0] = wd.w[w];
        if constexpr (PB == 3) src[w][1] = w + 1 < PB ? __builtin_amdgcn_alignbit(wd.w[w + 1 < PB ? w + 1 : w], wd.w[w], 8) : wd.w[w] >> 8;
        else src[w][1] = wd.w[w] >> (PB == 4 ? 8 : 10);
    }
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        const FieldStep f = field_step<PB>(s);
        const __half2 h = as_half2(and_or(src[f.word][f.shift != 0], f.mask, orc[f.orc_id]));
        if (f.k_lo >= 0) acc[f.k_lo] = fmaf(__low2float(h), a, acc[f.k_lo]);
        if (f.k_hi >= 0) acc[f.k_hi] = fmaf(__high2float(h), a, acc[f.k_hi]);
    }
}

// M16: the group parameters come as one 16-bit word per (group, column) in `scales` (the
// fp16 pattern of the scale without its sign bit and its PB-1 lowest bits, above the PB-bit
// zero-point) instead of an fp32 scale and a u8 zero-point.
template <int PB, bool M16>
__global__ __launch_bounds__(64 * GV_WAVES, 4) void gemv_ic_tiles(const uint32_t* __restrict__ packed,
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
        // GV_NBUF buffers taken in turn, no copies: one is consumed while the others are in flight (a step is 2 to
        // 4 KB per wave; the memory system wants several of them outstanding per wave).  Fetches past the end
        // re-read the chunk's last columns and are not consumed.
        const int64_t j_last = j_end - 4;
        Step st[GV_NBUF];
#pragma unroll
        for (int b = 0; b < GV_NBUF - 1; ++b) fetch(st[b], min(j_begin + 4 * b, j_last));
        for (int64_t j0 = j_begin; j0 < j_end; j0 += 4 * GV_NBUF) {   // in % 4 == 0
#pragma unroll
            for (int b = 0; b < GV_NBUF; ++b) {
                fetch(st[(b + GV_NBUF - 1) % GV_NBUF], min(j0 + 4 * (b + GV_NBUF - 1), j_last));
                if (j0 + 4 * b < j_end) consume(st[b]);
            }
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

// Measurement aid: the same code words read by the same grid, waves and column ranges as gemv_ic_tiles, with one
// xor per word in place of the arithmetic and no parameters, x, LDS reduction or partial sums: what the kernel's
// access pattern alone costs.  Each thread leaves one word in `sink` so that the loads are not dropped.
template <int PB>
__global__ __launch_bounds__(64 * GV_WAVES, 4) void gemv_bare_read(const uint32_t* __restrict__ packed, int64_t out,
                                                                int64_t in, int64_t n_words,
                                                                uint32_t* __restrict__ sink) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t o_lane = int64_t(blockIdx.x) * GV_OUT_PER_BLOCK + lane * 32;
    const bool valid = o_lane < out;
    const uint32_t n_wv = gridDim.y * GV_WAVES, wv = blockIdx.y * GV_WAVES + wave, quads = static_cast<uint32_t>(in >> 2);
    const uint32_t q_each = quads / n_wv, q_more = quads - q_each * n_wv;
    const int64_t j_begin = int64_t(wv * q_each + min(wv, q_more)) << 2;
    const int64_t j_end = int64_t((wv + 1) * q_each + min(wv + 1, q_more)) << 2;
    const uint32_t* wp = packed + (valid ? (o_lane >> 5) * PB : 0);
    uint32_t acc = 0;
    if (valid) {
        for (int64_t j0 = j_begin; j0 < j_end; j0 += 4) {
            Words<PB> wd[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) wd[c] = load_words<PB>(wp + (j0 + c) * n_words);
#pragma unroll
            for (int c = 0; c < 4; ++c)
#pragma unroll
                for (int w = 0; w < PB; ++w) acc ^= wd[c].w[w];
        }
    }
    sink[(int64_t(blockIdx.y) * gridDim.x + blockIdx.x) * (64 * GV_WAVES) + threadIdx.x] = acc;
}

}  // namespace

extern "C" int adadim_probe_gemv_read(adadim_ctx* ctx, const void* packed, int64_t out, int64_t in, int bits,
                                      double* us) {
    if (!ctx) return ADADIM_ENULL;
    if (!packed || !us) return adadim_fail(ctx, ADADIM_ENULL, "adadim_probe_gemv_read: NULL argument");
    if (bits < 2 || bits > 4 || out <= 0 || in <= 0 || out > (int64_t(1) << 24) || in > (int64_t(1) << 24) ||
        (out % 32) != 0 || (in % 4) != 0)
        return adadim_fail(ctx, ADADIM_EINVAL, "adadim_probe_gemv_read: bits 2..4, out a multiple of 32, in of 4, both "
                                               "at most 2^24");
    if (reinterpret_cast<uintptr_t>(packed) & 15u)
        return adadim_fail(ctx, ADADIM_EALIGN, "adadim_probe_gemv_read: packed must be 16-byte aligned");
    if (ctx->capturing) return adadim_fail(ctx, ADADIM_EINVAL, "adadim_probe_gemv_read: not while a graph is being recorded");
    // the grid of launch_gemv_ic
    const int n_tiles = static_cast<int>((out + GV_OUT_PER_BLOCK - 1) / GV_OUT_PER_BLOCK);
    const int64_t max_chunks = std::max<int64_t>(1, in / (GV_WAVES * GV_MIN_COLS_PER_WAVE));
    const int64_t rounds = (n_tiles + GV_BLOCK_SLOTS - 1) / GV_BLOCK_SLOTS;
    const int n_chunks = static_cast<int>(std::min<int64_t>(max_chunks, std::max<int64_t>(1, rounds * GV_BLOCK_SLOTS / n_tiles)));
    uint32_t* sink = static_cast<uint32_t*>(
        adadim_workspace(ctx, WS_GEMV_PART, size_t(n_tiles) * size_t(n_chunks) * 64 * GV_WAVES * sizeof(uint32_t)));
    if (!sink) return ADADIM_EHIP;
    const int64_t n_words = out * bits / 32;
    const dim3 grid(static_cast<unsigned>(n_tiles), static_cast<unsigned>(n_chunks));
    hipEvent_t e0, e1;
    ADADIM_HIP_TRY(ctx, hipEventCreate(&e0));
    ADADIM_HIP_TRY(ctx, hipEventCreate(&e1));
    ADADIM_HIP_TRY(ctx, hipEventRecord(e0, ctx->stream));
    const uint32_t* pk = static_cast<const uint32_t*>(packed);
    switch (bits) {
        case 2: hipLaunchKernelGGL(gemv_bare_read<2>, grid, dim3(64 * GV_WAVES), 0, ctx->stream, pk, out, in, n_words, sink); break;
        case 3: hipLaunchKernelGGL(gemv_bare_read<3>, grid, dim3(64 * GV_WAVES), 0, ctx->stream, pk, out, in, n_words, sink); break;
        default: hipLaunchKernelGGL(gemv_bare_read<4>, grid, dim3(64 * GV_WAVES), 0, ctx->stream, pk, out, in, n_words, sink); break;
    }
    const hipError_t le = hipGetLastError();
    hipError_t e = hipEventRecord(e1, ctx->stream);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    float ms = 0.0f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (le != hipSuccess) return adadim_fail(ctx, ADADIM_EHIP, "adadim_probe_gemv_read: launch: %s", hipGetErrorString(le));
    if (e != hipSuccess) return adadim_fail(ctx, ADADIM_EHIP, "adadim_probe_gemv_read: %s", hipGetErrorString(e));
    *us = double(ms) * 1e3;
    return ADADIM_OK;
}

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
