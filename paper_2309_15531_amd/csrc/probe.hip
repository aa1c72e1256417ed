// Measurement aid (not part of the method): what the matrix cores of this chip sustain on an instruction stream
// of nothing but v_mfma_f32_32x32x16_f16 with register-resident operands, for operands of all zeros and for
// random fp16 operands (and, further down, of nothing but v_mfma_f64_16x16x4_f64).  The two differ because the chip holds a power limit by lowering its clock, and the power
// a multiplier array draws depends on the bits that toggle in it; the figure for random operands, not the
// published peak, is what a real fp16 contraction can approach.  The kernel also reads the shader clock
// (clock64) against the constant 100 MHz counter (wall_clock64) to report the clock the loop ran at.
#include "common.h"

namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int PROBE_ACC = 16, PROBE_OPS = 4;

__global__ __launch_bounds__(256) void mfma_probe(float* __restrict__ out, int iters, unsigned seed, int random_operands) {
    half8 a[PROBE_OPS], b[PROBE_OPS];
    unsigned s = seed + threadIdx.x * 2654435761u + blockIdx.x * 40503u;
    for (int v = 0; v < PROBE_OPS; ++v)
        for (int i = 0; i < 8; ++i) {
            s = s * 1664525u + 1013904223u;
            float x = ((s >> 8) & 0xffff) / 16384.0f - 2.0f;     // uniform in [-2, 2)
            s = s * 1664525u + 1013904223u;
            float y = ((s >> 8) & 0xffff) / 16384.0f - 2.0f;
            if (!random_operands) x = y = 0.0f;
            a[v][i] = static_cast<_Float16>(x);
            b[v][i] = static_cast<_Float16>(y);
        }
    floatx16 acc[PROBE_ACC];
    for (int t = 0; t < PROBE_ACC; ++t)
        for (int r = 0; r < 16; ++r) acc[t][r] = 0.0f;
    const long long c0 = clock64(), w0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int v = 0; v < PROBE_OPS; ++v)
#pragma unroll
            for (int t = 0; t < PROBE_ACC; ++t)
                acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[v], b[(v + t) % PROBE_OPS], acc[t], 0, 0, 0);
    }
    const long long c1 = clock64(), w1 = wall_clock64();
    float sum = 0.0f;
    for (int t = 0; t < PROBE_ACC; ++t)
        for (int r = 0; r < 16; ++r) sum += acc[t][r];
    out[8 + blockIdx.x * 256 + threadIdx.x] = sum;            // keeps the loop alive
    if (threadIdx.x == 0 && blockIdx.x == 7) {
        out[0] = static_cast<float>(c1 - c0);
        out[1] = static_cast<float>(w1 - w0);
    }
}

// The same for the fp64 instruction of the GPTQ factor: eight independent v_mfma_f64_16x16x4_f64 chains per wave.
typedef double double4_t __attribute__((ext_vector_type(4)));
constexpr int PROBE64_ACC = 8;
__global__ __launch_bounds__(256) void mfma_probe_f64(float* __restrict__ out, int iters) {
    const double a = 1.000001 + threadIdx.x * 1e-3, b = 0.999999 - threadIdx.x * 1e-3;
    double4_t acc[PROBE64_ACC];
    for (int t = 0; t < PROBE64_ACC; ++t) acc[t] = double4_t{0.0, 0.0, 0.0, 0.0};
    const long long c0 = clock64(), w0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int t = 0; t < PROBE64_ACC; ++t) acc[t] = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, acc[t], 0, 0, 0);
    }
    const long long c1 = clock64(), w1 = wall_clock64();
    double sum = 0.0;
    for (int t = 0; t < PROBE64_ACC; ++t) sum += acc[t][0] + acc[t][1] + acc[t][2] + acc[t][3];
    out[8 + blockIdx.x * 256 + threadIdx.x] = static_cast<float>(sum);   // keeps the loop alive
    if (threadIdx.x == 0 && blockIdx.x == 7) {
        out[0] = static_cast<float>(c1 - c0);
        out[1] = static_cast<float>(w1 - w0);
    }
}

// launches `launch(out)` between two events and reads the two clock counts back
template <class L>
int run_probe(adadim_ctx* ctx, const char* who, int blocks, L launch, float* ms, double* clock_mhz) {
    float* out = static_cast<float*>(adadim_workspace(ctx, WS_PROBE, (8 + size_t(blocks) * 256) * sizeof(float)));
    if (!out) return ADADIM_EHIP;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    ADADIM_HIP_TRY(ctx, hipEventCreate(&e0));
    hipError_t e = hipEventCreate(&e1);
    if (e == hipSuccess) e = hipEventRecord(e0, ctx->stream);
    if (e == hipSuccess) {
        launch(out);
        e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipEventRecord(e1, ctx->stream);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    float clk[2] = {0.0f, 1.0f};
    if (e == hipSuccess) e = hipEventElapsedTime(ms, e0, e1);
    if (e == hipSuccess) e = hipMemcpy(clk, out, sizeof(clk), hipMemcpyDeviceToHost);
    (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (e != hipSuccess) return adadim_fail(ctx, ADADIM_EHIP, "%s: %s", who, hipGetErrorString(e));
    *clock_mhz = double(clk[0]) / double(clk[1]) * 100.0;
    return ADADIM_OK;
}

}  // namespace

extern "C" int adadim_probe_mfma_f64(adadim_ctx* ctx, int iters, double* tflops, double* clock_mhz) {
    if (!ctx) return ADADIM_ENULL;
    if (!tflops || !clock_mhz) return adadim_fail(ctx, ADADIM_ENULL, "adadim_probe_mfma_f64: NULL output");
    if (iters <= 0 || iters > 1000000) return adadim_fail(ctx, ADADIM_EINVAL, "adadim_probe_mfma_f64: iters in [1, 1000000]");
    if (ctx->capturing) return adadim_fail(ctx, ADADIM_EINVAL, "adadim_probe_mfma_f64: not while a graph is being recorded");
    constexpr int BLOCKS = 1024;                              // four workgroups of four waves per compute unit
    float ms = 0.0f;
    const int rc = run_probe(ctx, "adadim_probe_mfma_f64", BLOCKS, [&](float* out) {
        hipLaunchKernelGGL(mfma_probe_f64, dim3(BLOCKS), dim3(256), 0, ctx->stream, out, iters);
    }, &ms, clock_mhz);
    if (rc != ADADIM_OK) return rc;
    *tflops = 2.0 * 16 * 16 * 4 * double(PROBE64_ACC) * iters * BLOCKS * 4 / (double(ms) * 1e-3) / 1e12;
    return ADADIM_OK;
}

extern "C" int adadim_probe_mfma(adadim_ctx* ctx, int random_operands, int iters, double* tflops, double* clock_mhz) {
    if (!ctx) return ADADIM_ENULL;
    if (!tflops || !clock_mhz) return adadim_fail(ctx, ADADIM_ENULL, "adadim_probe_mfma: NULL output");
    if (iters <= 0 || iters > 1000000 || (random_operands != 0 && random_operands != 1))
        return adadim_fail(ctx, ADADIM_EINVAL, "adadim_probe_mfma: iters in [1, 1000000], random_operands 0 or 1");
    if (ctx->capturing) return adadim_fail(ctx, ADADIM_EINVAL, "adadim_probe_mfma: not while a graph is being recorded");
    constexpr int BLOCKS = 1024;                              // four workgroups of four waves per compute unit
    float ms = 0.0f;
    const int rc = run_probe(ctx, "adadim_probe_mfma", BLOCKS, [&](float* out) {
        hipLaunchKernelGGL(mfma_probe, dim3(BLOCKS), dim3(256), 0, ctx->stream, out, iters, 12345u, random_operands);
    }, &ms, clock_mhz);
    if (rc != ADADIM_OK) return rc;
    const double flops = 2.0 * 32 * 32 * 16 * double(PROBE_ACC) * PROBE_OPS * iters * BLOCKS * 4;
    *tflops = flops / (double(ms) * 1e-3) / 1e12;
    return ADADIM_OK;
}
