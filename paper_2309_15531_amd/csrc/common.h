// Internal declarations shared by the library's translation units (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <mutex>

#include "../../include/adadim.h"
#include "gram_plan.h"

// Scratch slots owned by a context; each grows on demand and is reused.
enum {
    WS_HESS_PART = 0,   // split-K partial tiles of the Gram matrix
    WS_ERR_PART,        // per-column-block partial row losses
    WS_DW16,            // fp16 column-scaled copy of dW
    WS_HS,              // prepared fp16 H when the caller passes the fp32 one
    WS_HMETA,           // column scales and diagonal of the above
    WS_CODES,           // u8 codes when only the packed stream is requested
    WS_SELECT,          // device int for adadim_select without a device output
    WS_ERR_FIN,         // block totals and ticket of the loss reduction
    WS_ZERO,            // zero-filled buffer: source of out-of-range token rows for LDS DMA
    WS_QPART,           // partial (min, -max) pairs of the wide-group quantizer
    WS_QPAR,            // its per-group scale, zero and reciprocal
    WS_GEMV_PART,       // per-column-chunk partial outputs of the de-quantizing matrix-vector product
    WS_GPTQ_A,          // fp64 reversed, permuted, damped Hessian and its Cholesky factor
    WS_GPTQ_M,          // fp64 inverse of that factor
    WS_GPTQ_D,          // fp64 diagonal and damping term
    WS_GPTQ_T,          // fp64 products of the triangular inverse's doubling levels
    WS_GPTQ_W,          // fp32 working copy of the weight in visiting order
    WS_GPTQ_E,          // fp32 propagated errors in visiting order
    WS_GPTQ_Q,          // u8 codes in visiting order
    WS_GPTQ_V,          // int32 position of each original channel in the visiting order
    WS_PROBE,           // output of the matrix-core rate probe
    WS_COUNT
};

// Per-kernel event timing (adadim_profile).  Events are created once, on the
// first enable, and reused.
constexpr int PROF_MAX_LAUNCHES = 8192;
constexpr int PROF_MAX_KERNELS = 32;
struct adadim_prof {
    bool enabled;
    int n_events;                    // event pairs created so far
    int n_used;                      // pairs used since the last enable
    int64_t dropped;
    hipEvent_t* start;
    hipEvent_t* stop;
    int* kernel_of;                  // pair -> kernel slot
    int n_kernels;
    const char* names[PROF_MAX_KERNELS];
    char only[32];                   // when not empty: the one kernel that is bracketed
};

struct adadim_ctx {
    hipStream_t stream;
    char err[512];
    void* ws[WS_COUNT];
    size_t ws_bytes[WS_COUNT];
    size_t zero_ready_bytes;         // size of WS_ZERO when it was last cleared
    // Gram launch plans already chosen, keyed by (token count, tile count, whether whole tiles may store): choosing
    // one simulates the launch's schedule (milliseconds of host time), and a model driver alternates between a few
    // input widths
    struct GramSplit { GramPlan plan; GramOrder order; bool whole_ok; } gram_split[8];
    int gram_split_n, gram_split_next;
    bool capturing;                  // between adadim_capture_begin and adadim_capture_end
    hipStream_t side;                // second stream for work that may overlap the main one (created on first use)
    hipEvent_t side_ev[2];           // main -> side and side -> main hand-overs
    adadim_prof prof;
};

// Brackets one kernel launch with events when profiling is on.
struct ProfScope {
    adadim_ctx* ctx;
    int pair;
    ProfScope(adadim_ctx* c, const char* name);
    ~ProfScope();
};

int adadim_fail(adadim_ctx* ctx, int code, const char* fmt, ...);

// Creates the context's side stream and its two events on first use (default priority, like every
// stream here).  Returns false with the error recorded.
bool adadim_side_stream(adadim_ctx* ctx);

// Returns a device buffer of at least `bytes` for `slot`, or nullptr (error recorded).
void* adadim_workspace(adadim_ctx* ctx, int slot, size_t bytes);

#define ADADIM_HIP_TRY(ctx, expr)                                                          \
    do {                                                                                   \
        hipError_t e__ = (expr);                                                           \
        if (e__ != hipSuccess)                                                             \
            return adadim_fail((ctx), ADADIM_EHIP, "%s: %s", #expr, hipGetErrorString(e__)); \
    } while (0)

#define ADADIM_LAUNCH_CHECK(ctx, what)                                                     \
    do {                                                                                   \
        hipError_t e__ = hipGetLastError();                                                \
        if (e__ != hipSuccess)                                                             \
            return adadim_fail((ctx), ADADIM_EHIP, "launch %s: %s", (what), hipGetErrorString(e__)); \
    } while (0)

// Scoring layout of an fp16 [rows, cols] operand of the error GEMM (the column-scaled dW and the
// prepared H).  The GEMM consumes 32 contraction elements (64 bytes) from each of 256 consecutive
// rows per pipeline stage.  When cols is a multiple of 32 the operand is therefore stored as
// [row tile of 256][column block of 32][256 rows][32 columns]: a stage is one contiguous 16 KB
// piece (whole 128-byte lines per request), successive stages of a tile follow each other in
// memory, and no pitch is a large power of two (a [column block][rows][32] layout had a pitch of
// rows*64 bytes between column blocks, which for 4096 rows put every block of a producer's tile
// on the same memory channels).  The last row tile is padded to 256 rows: a buffer holds
// score_elems(rows, cols) elements.  Otherwise plain row-major.
__host__ __device__ inline bool score_blocked(int64_t cols) { return (cols & 31) == 0; }
__host__ __device__ inline int64_t score_elems(int64_t rows, int64_t cols) {
    return score_blocked(cols) ? ((rows + 255) & ~int64_t(255)) * cols : rows * cols;
}
__host__ __device__ inline int64_t score_index(int64_t row, int64_t col, int64_t rows, int64_t cols) {
    (void)rows;
    return score_blocked(cols) ? (((row >> 8) * (cols >> 5) + (col >> 5)) * 256 + (row & 255)) * 32 + (col & 31)
                               : row * cols + col;
}

// Runs `fn` (a sequence of hipFuncSetAttribute calls returning hipError_t) once per device and thread-safely:
// function attributes belong to the device that is current when they are set, and several host threads may
// make their first call at the same time.  A failed run is tried again by the next call.
struct PerDeviceOnce {
    std::mutex m;
    bool done[128] = {};
    template <class F>
    hipError_t run(F fn) {
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return e;
        if (dev < 0 || dev >= 128) return hipErrorInvalidDevice;
        std::lock_guard<std::mutex> lock(m);
        if (done[dev]) return hipSuccess;
        e = fn();
        if (e == hipSuccess) done[dev] = true;
        return e;
    }
};

static inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Launchers implemented in the .hip files.  All validate nothing: the API layer does.
int launch_quantize(adadim_ctx* ctx, const __half* W, int64_t out, int64_t in, int dim, int bits, int g,
                    float clip, uint8_t* codes, float* scales, uint8_t* zeros, void* dW, int dW_dtype,
                    const float* colscale, uint32_t* packed, int mfmt);
int launch_quantize_both(adadim_ctx* ctx, const __half* W, int64_t out, int64_t in, int bits, int g_oc, int g_ic, float clip,
                         int mfmt, const float* colscale, uint8_t* codes_oc, float* scales_oc, uint8_t* zeros_oc,
                         void* dW_oc, uint32_t* packed_oc, uint8_t* codes_ic, float* scales_ic, uint8_t* zeros_ic,
                         void* dW_ic, uint32_t* packed_ic);
int launch_pack(adadim_ctx* ctx, const uint8_t* codes, int64_t out, int64_t in, int dim, int bits,
                uint32_t* packed);
int launch_hessian(adadim_ctx* ctx, const __half* X, int64_t tokens, int64_t in, int64_t ldx, float* H,
                   int accumulate);
int launch_hessian_prepare(adadim_ctx* ctx, const float* H, int64_t in, __half* Hs, float* hmeta);
int launch_hessian_prepared(adadim_ctx* ctx, const __half* X, int64_t tokens, int64_t in, int64_t ldx, float* H,
                            __half* Hs, float* hmeta);
int launch_layer_error(adadim_ctx* ctx, int n, const void* const* dW, int dW_dtype, int64_t out, int64_t in,
                       const __half* Hs, const float* hmeta, float* loss_rows, float* losses,
                       int32_t* best_dev = nullptr);
// The same launch group (n <= 8 candidates, column-scaled fp16 dW) with its scratch in the library's fixed device
// array; _bytes gives what such a launch needs of it.
int launch_layer_error_noalloc(adadim_ctx* ctx, int n, const void* const* dW, int64_t out, int64_t in, const __half* Hs,
                               const float* hmeta, float* loss_rows, float* losses, int32_t* best_dev);
int64_t launch_layer_error_noalloc_bytes(int n, int64_t out, int64_t in);
int launch_select(adadim_ctx* ctx, const float* losses, int n, int32_t* best_dev);
int launch_gptq_prepare(adadim_ctx* ctx, const float* H, int64_t n, float percdamp, int act_order, int32_t* perm,
                        uint8_t* dead, float* U);
int launch_gptq_quantize(adadim_ctx* ctx, const __half* W, int64_t out, int64_t in, int dim, int bits, int g,
                         const float* U, const int32_t* perm, const uint8_t* dead, const float* st_scales,
                         const uint8_t* st_zeros, uint8_t* codes, float* scales_out, uint8_t* zeros_out, float* dW, int mfmt);
int launch_gemv_ic(adadim_ctx* ctx, const uint32_t* packed, const void* scales, const uint8_t* zeros, const __half* x,
                   int64_t out, int64_t in, int bits, int g, __half* y, bool meta16);
