// C-ABI entry points: context handling and argument validation.  Every check
// runs before the first HIP call so that a rejected call touches no device.
#include "common.h"

#include <algorithm>
#include <vector>

#include <cmath>
#include <cstdlib>
#include <cstring>
#include <new>

static char g_create_error[256] = "";

int adadim_fail(adadim_ctx* ctx, int code, const char* fmt, ...) {
    char* dst = ctx ? ctx->err : g_create_error;
    size_t cap = ctx ? sizeof(ctx->err) : sizeof(g_create_error);
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(dst, cap, fmt, ap);
    va_end(ap);
    return code;
}

void* adadim_workspace(adadim_ctx* ctx, int slot, size_t bytes) {
    if (bytes == 0) bytes = 256;
    if (ctx->ws_bytes[slot] >= bytes) return ctx->ws[slot];
    if (ctx->capturing) {
        adadim_fail(ctx, ADADIM_EINVAL,
                    "scratch slot %d would have to grow while a graph is being recorded: make the same call once "
                    "before adadim_capture_begin", slot);
        return nullptr;
    }
    if (ctx->ws[slot]) {
        // Earlier kernels on the stream may still read the old buffer.
        if (hipStreamSynchronize(ctx->stream) != hipSuccess || hipFree(ctx->ws[slot]) != hipSuccess) {
            adadim_fail(ctx, ADADIM_EHIP, "releasing scratch slot %d failed", slot);
            return nullptr;
        }
        ctx->ws[slot] = nullptr;
        ctx->ws_bytes[slot] = 0;
    }
    size_t want = (bytes + 255) & ~size_t(255);
    void* p = nullptr;
    hipError_t e = hipMalloc(&p, want);
    if (e != hipSuccess) {
        adadim_fail(ctx, ADADIM_EHIP, "hipMalloc(%zu bytes) for scratch slot %d: %s", want, slot,
                    hipGetErrorString(e));
        return nullptr;
    }
    ctx->ws[slot] = p;
    ctx->ws_bytes[slot] = want;
    return p;
}

bool adadim_side_stream(adadim_ctx* ctx) {
    if (ctx->side) return true;
    hipStream_t st = nullptr;
    hipError_t e = hipStreamCreateWithFlags(&st, hipStreamNonBlocking);
    for (int i = 0; e == hipSuccess && i < 2; ++i) e = hipEventCreateWithFlags(&ctx->side_ev[i], hipEventDisableTiming);
    if (e != hipSuccess) {
        adadim_fail(ctx, ADADIM_EHIP, "creating the side stream: %s", hipGetErrorString(e));
        for (int i = 0; i < 2; ++i)
            if (ctx->side_ev[i]) {
                (void)hipEventDestroy(ctx->side_ev[i]);
                ctx->side_ev[i] = nullptr;
            }
        if (st) (void)hipStreamDestroy(st);
        return false;
    }
    ctx->side = st;
    return true;
}

ProfScope::ProfScope(adadim_ctx* c, const char* name) : ctx(c), pair(-1) {
    adadim_prof& p = c->prof;
    if (!p.enabled || c->capturing) return;
    if (p.only[0] && std::strcmp(p.only, name) != 0) return;
    if (p.n_used >= p.n_events) {
        ++p.dropped;
        return;
    }
    int k = 0;
    while (k < p.n_kernels && p.names[k] != name && std::strcmp(p.names[k], name) != 0) ++k;
    if (k == p.n_kernels) {
        if (k == PROF_MAX_KERNELS) {
            ++p.dropped;
            return;
        }
        p.names[p.n_kernels++] = name;
    }
    pair = p.n_used++;
    p.kernel_of[pair] = k;
    (void)hipEventRecord(p.start[pair], c->stream);
}

ProfScope::~ProfScope() {
    if (pair >= 0) (void)hipEventRecord(ctx->prof.stop[pair], ctx->stream);
}

extern "C" {

int adadim_profile(adadim_ctx* ctx, int enable) {
    if (!ctx) return ADADIM_ENULL;
    adadim_prof& p = ctx->prof;
    if (enable && !p.start) {
        p.start = new (std::nothrow) hipEvent_t[PROF_MAX_LAUNCHES];
        p.stop = new (std::nothrow) hipEvent_t[PROF_MAX_LAUNCHES];
        p.kernel_of = new (std::nothrow) int[PROF_MAX_LAUNCHES];
        if (!p.start || !p.stop || !p.kernel_of) return adadim_fail(ctx, ADADIM_EINVAL, "adadim_profile: out of host memory");
        p.n_events = 0;
        for (int i = 0; i < PROF_MAX_LAUNCHES; ++i) {
            ADADIM_HIP_TRY(ctx, hipEventCreate(&p.start[i]));
            ADADIM_HIP_TRY(ctx, hipEventCreate(&p.stop[i]));
            p.n_events = i + 1;
        }
    }
    if (enable) {
        p.n_used = 0;
        p.dropped = 0;
        p.n_kernels = 0;
    }
    p.enabled = enable != 0;
    return ADADIM_OK;
}

int adadim_profile_only(adadim_ctx* ctx, const char* name) {
    if (!ctx) return ADADIM_ENULL;
    const size_t len = name ? std::strlen(name) : 0;
    if (len >= sizeof(ctx->prof.only))
        return adadim_fail(ctx, ADADIM_EINVAL, "adadim_profile_only: a kernel name has at most %d characters", int(sizeof(ctx->prof.only)) - 1);
    std::memcpy(ctx->prof.only, name ? name : "", len);
    ctx->prof.only[len] = 0;
    return ADADIM_OK;
}

int adadim_profile_read(adadim_ctx* ctx, int idx, char* name, int cap, double* total_ms, int64_t* launches) {
    if (!ctx) return ADADIM_ENULL;
    adadim_prof& p = ctx->prof;
    if (idx < 0 || idx >= p.n_kernels) return adadim_fail(ctx, ADADIM_EINVAL, "adadim_profile_read: no record %d", idx);
    ADADIM_HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    double tot = 0.0;
    int64_t n = 0;
    for (int i = 0; i < p.n_used; ++i) {
        if (p.kernel_of[i] != idx) continue;
        float ms = 0.0f;
        ADADIM_HIP_TRY(ctx, hipEventElapsedTime(&ms, p.start[i], p.stop[i]));
        tot += ms;
        ++n;
    }
    if (name && cap > 0) {
        std::strncpy(name, p.names[idx], cap - 1);
        name[cap - 1] = 0;
    }
    if (total_ms) *total_ms = tot;
    if (launches) *launches = n;
    return ADADIM_OK;
}

int adadim_profile_read_spread(adadim_ctx* ctx, int idx, double* min_ms, double* median_ms, double* max_ms) {
    if (!ctx) return ADADIM_ENULL;
    adadim_prof& p = ctx->prof;
    if (idx < 0 || idx >= p.n_kernels)
        return adadim_fail(ctx, ADADIM_EINVAL, "adadim_profile_read_spread: no record %d", idx);
    ADADIM_HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    std::vector<float> ms;
    for (int i = 0; i < p.n_used; ++i) {
        if (p.kernel_of[i] != idx) continue;
        float t = 0.0f;
        ADADIM_HIP_TRY(ctx, hipEventElapsedTime(&t, p.start[i], p.stop[i]));
        ms.push_back(t);
    }
    std::sort(ms.begin(), ms.end());
    const size_t n = ms.size();
    if (min_ms) *min_ms = n ? ms.front() : 0.0;
    if (max_ms) *max_ms = n ? ms.back() : 0.0;
    if (median_ms) *median_ms = n ? 0.5 * (double(ms[(n - 1) / 2]) + double(ms[n / 2])) : 0.0;
    return ADADIM_OK;
}

const char* adadim_version(void) { return "adadim-gfx950 0.3"; }

int64_t adadim_score_elems(int64_t rows, int64_t cols) {
    if (rows <= 0 || cols <= 0) return 0;
    return score_elems(rows, cols);
}

int adadim_create(adadim_ctx** out, void* hip_stream) {
    if (!out) return adadim_fail(nullptr, ADADIM_ENULL, "adadim_create: out is NULL");
    adadim_ctx* c = new (std::nothrow) adadim_ctx;
    if (!c) return adadim_fail(nullptr, ADADIM_EINVAL, "adadim_create: out of host memory");
    std::memset(c, 0, sizeof(*c));
    c->stream = static_cast<hipStream_t>(hip_stream);
    std::strcpy(c->err, "no error");
    *out = c;
    return ADADIM_OK;
}

void adadim_destroy(adadim_ctx* ctx) {
    if (!ctx) return;
    if (ctx->capturing) {                                     // an unfinished recording: end and drop it
        hipGraph_t g = nullptr;
        if (hipStreamEndCapture(ctx->stream, &g) == hipSuccess && g) (void)hipGraphDestroy(g);
        ctx->capturing = false;
    }
    if (ctx->side) {
        (void)hipStreamSynchronize(ctx->side);
        for (int i = 0; i < 2; ++i) (void)hipEventDestroy(ctx->side_ev[i]);
        (void)hipStreamDestroy(ctx->side);
    }
    bool any = false;
    for (int i = 0; i < WS_COUNT; ++i) any = any || ctx->ws[i];
    if (any) {
        (void)hipStreamSynchronize(ctx->stream);
        for (int i = 0; i < WS_COUNT; ++i)
            if (ctx->ws[i]) (void)hipFree(ctx->ws[i]);
    }
    if (ctx->prof.start) {
        for (int i = 0; i < ctx->prof.n_events; ++i) {
            (void)hipEventDestroy(ctx->prof.start[i]);
            (void)hipEventDestroy(ctx->prof.stop[i]);
        }
        delete[] ctx->prof.start;
        delete[] ctx->prof.stop;
        delete[] ctx->prof.kernel_of;
    }
    delete ctx;
}

const char* adadim_last_error(const adadim_ctx* ctx) { return ctx ? ctx->err : g_create_error; }

int adadim_hessian(adadim_ctx* ctx, const void* X, int64_t tokens, int64_t in, int64_t ldx, float* H,
                   int accumulate) {
    if (!ctx) return ADADIM_ENULL;
    if (!H) return adadim_fail(ctx, ADADIM_ENULL, "adadim_hessian: H is NULL");
    if (tokens < 0 || in <= 0 || ldx < in || (accumulate != 0 && accumulate != 1))
        return adadim_fail(ctx, ADADIM_EINVAL,
                           "adadim_hessian: need tokens >= 0, in > 0, ldx >= in, accumulate in {0,1} "
                           "(tokens=%lld in=%lld ldx=%lld accumulate=%d)",
                           (long long)tokens, (long long)in, (long long)ldx, accumulate);
    if (in > (int64_t(1) << 20) || tokens > (int64_t(1) << 40))
        return adadim_fail(ctx, ADADIM_EINVAL, "adadim_hessian: size out of range");
    if (tokens > 0 && !X) return adadim_fail(ctx, ADADIM_ENULL, "adadim_hessian: X is NULL");
    if ((in % 8) != 0 || (ldx % 8) != 0 || !aligned16(X) || !aligned16(H))
        return adadim_fail(ctx, ADADIM_EALIGN,
                           "adadim_hessian: in and ldx must be multiples of 8, X and H 16-byte aligned");
    return launch_hessian(ctx, static_cast<const __half*>(X), tokens, in, ldx, H, accumulate);
}

// shared by the two quantizer entry points; mfmt = 0: fp32 scales and u8 zeros, else the 16-bit group word
static int quantize_checked(adadim_ctx* ctx, const void* W, int64_t out, int64_t in, int dim, int bits, int group,
                            float clip, uint8_t* codes, float* scales, uint8_t* zeros, void* dW, int dW_dtype,
                            const float* colscale, uint32_t* packed, int mfmt) {
    if (!ctx) return ADADIM_ENULL;
    if (!W) return adadim_fail(ctx, ADADIM_ENULL, "adadim_quantize: W is NULL");
    if (out <= 0 || in <= 0 || out > (int64_t(1) << 24) || in > (int64_t(1) << 24))
        return adadim_fail(ctx, ADADIM_EINVAL, "adadim_quantize: bad shape out=%lld in=%lld",
                           (long long)out, (long long)in);
    if (dim != ADADIM_DIM_OC && dim != ADADIM_DIM_IC)
        return adadim_fail(ctx, ADADIM_EINVAL, "adadim_quantize: dim must be 0 (OC) or 1 (IC), got %d", dim);
    if (bits < 2 || bits > 8)
        return adadim_fail(ctx, ADADIM_EINVAL, "adadim_quantize: bits must be in [2,8], got %d", bits);
    if (!(clip > 0.0f && clip <= 1.0f))
        return adadim_fail(ctx, ADADIM_EINVAL, "adadim_quantize: clip must be in (0,1], got %g", (double)clip);
    const int64_t axis = dim == ADADIM_DIM_OC ? in : out;
    if (group < 0 || (group > 0 && (axis % group) != 0))
        return adadim_fail(ctx, ADADIM_EINVAL,
                           "adadim_quantize: group %d must be 0 or divide the grouped axis (%lld)", group,
                           (long long)axis);
    if (dW && dW_dtype != ADADIM_DW_F32 && dW_dtype != ADADIM_DW_F16 && dW_dtype != ADADIM_DW_F16_SCALED)
        return adadim_fail(ctx, ADADIM_EINVAL, "adadim_quantize: unknown dW_dtype %d", dW_dtype);
    if (dW && dW_dtype == ADADIM_DW_F16_SCALED && !colscale)
        return adadim_fail(ctx, ADADIM_ENULL, "adadim_quantize: colscale is NULL with dW_dtype F16_SCALED");
    if (dW && dW_dtype == ADADIM_DW_F16_SCALED && (in % 8) == 0 && !aligned16(colscale))
        return adadim_fail(ctx, ADADIM_EALIGN, "adadim_quantize: colscale must be 16-byte aligned");
    if ((in % 8) == 0 && (!aligned16(W) || (dW && !aligned16(dW)) || (codes && (reinterpret_cast<uintptr_t>(codes) & 7u))))
        return adadim_fail(ctx, ADADIM_EALIGN,
                           "adadim_quantize: W and dW must be 16-byte, codes 8-byte aligned");
    const int g = group == 0 ? (int)axis : group;
    return launch_quantize(ctx, static_cast<const __half*>(W), out, in, dim, bits, g, clip, codes, scales,
                           zeros, dW, dW_dtype, colscale, packed, mfmt);
}

int adadim_quantize(adadim_ctx* ctx, const void* W, int64_t out, int64_t in, int dim, int bits, int group,
                    float clip, uint8_t* codes, float* scales, uint8_t* zeros, void* dW, int dW_dtype,
                    const float* colscale, uint32_t* packed) {
    return quantize_checked(ctx, W, out, in, dim, bits, group, clip, codes, scales, zeros, dW, dW_dtype, colscale,
                            packed, 0);
}

int adadim_quantize_both(adadim_ctx* ctx, const void* W, int64_t out, int64_t in, int bits, int group, float clip,
                         int meta16, const float* colscale, uint8_t* codes_oc, void* scales_oc, uint8_t* zeros_oc,
                         void* dW_oc, uint32_t* packed_oc, uint8_t* codes_ic, void* scales_ic, uint8_t* zeros_ic,
                         void* dW_ic, uint32_t* packed_ic) {
    if (!ctx) return ADADIM_ENULL;
    if (!W || !colscale) return adadim_fail(ctx, ADADIM_ENULL, "adadim_quantize_both: W or colscale is NULL");
    if (out <= 0 || in <= 0 || out > (int64_t(1) << 24) || in > (int64_t(1) << 24))
        return adadim_fail(ctx, ADADIM_EINVAL, "adadim_quantize_both: bad shape out=%lld in=%lld", (long long)out,
                           (long long)in);
    if (bits < 2 || bits > (meta16 ? 4 : 8) || (meta16 != 0 && meta16 != 1))
        return adadim_fail(ctx, ADADIM_EINVAL, "adadim_quantize_both: bits must be in [2,8] ([2,4] for group words), "
                                               "meta16 0 or 1 (bits=%d meta16=%d)", bits, meta16);
    if (!(clip > 0.0f && clip <= 1.0f))
        return adadim_fail(ctx, ADADIM_EINVAL, "adadim_quantize_both: clip must be in (0,1], got %g", (double)clip);
    if (group < 0 || (group > 0 && ((in % group) != 0 || (out % group) != 0)))
        return adadim_fail(ctx, ADADIM_EINVAL, "adadim_quantize_both: group %d must be 0 or divide both out and in", group);
    if ((in % 8) != 0)
        return adadim_fail(ctx, ADADIM_EINVAL, "adadim_quantize_both: in must be a multiple of 8 (scoring layout)");
    if (!aligned16(W) || !aligned16(colscale) || (dW_oc && !aligned16(dW_oc)) || (dW_ic && !aligned16(dW_ic)) ||
        (codes_oc && (reinterpret_cast<uintptr_t>(codes_oc) & 7u)) || (codes_ic && (reinterpret_cast<uintptr_t>(codes_ic) & 7u)))
        return adadim_fail(ctx, ADADIM_EALIGN, "adadim_quantize_both: W, colscale and dW must be 16-byte, codes 8-byte aligned");
    const int g_oc = group == 0 ? (int)in : group, g_ic = group == 0 ? (int)out : group;
    return launch_quantize_both(ctx, static_cast<const __half*>(W), out, in, bits, g_oc, g_ic, clip, meta16 ? bits : 0,
                                colscale, codes_oc, static_cast<float*>(scales_oc), meta16 ? nullptr : zeros_oc, dW_oc,
                                packed_oc, codes_ic, static_cast<float*>(scales_ic), meta16 ? nullptr : zeros_ic, dW_ic,
                                packed_ic);
}

int adadim_quantize_meta16(adadim_ctx* ctx, const void* W, int64_t out, int64_t in, int dim, int bits, int group,
                           float clip, uint8_t* codes, uint16_t* meta, void* dW, int dW_dtype,
                           const float* colscale, uint32_t* packed) {
    if (!ctx) return ADADIM_ENULL;
    if (bits < 2 || bits > 4)
        return adadim_fail(ctx, ADADIM_EINVAL, "adadim_quantize_meta16: bits must be 2, 3 or 4, got %d", bits);
    return quantize_checked(ctx, W, out, in, dim, bits, group, clip, codes, reinterpret_cast<float*>(meta), nullptr, dW,
                            dW_dtype, colscale, packed, bits);
}

int adadim_hessian_prepare(adadim_ctx* ctx, const float* H, int64_t in, void* Hs, float* hmeta) {
    if (!ctx) return ADADIM_ENULL;
    if (!H || !Hs || !hmeta) return adadim_fail(ctx, ADADIM_ENULL, "adadim_hessian_prepare: NULL argument");
    if (in <= 0 || in > (int64_t(1) << 20))
        return adadim_fail(ctx, ADADIM_EINVAL, "adadim_hessian_prepare: bad in=%lld", (long long)in);
    if ((in % 8) != 0 || !aligned16(H) || !aligned16(Hs) || !aligned16(hmeta))
        return adadim_fail(ctx, ADADIM_EALIGN,
                           "adadim_hessian_prepare: in must be a multiple of 8, H, Hs and hmeta 16-byte aligned");
    return launch_hessian_prepare(ctx, H, in, static_cast<__half*>(Hs), hmeta);
}

int adadim_hessian_prepared(adadim_ctx* ctx, const void* X, int64_t tokens, int64_t in, int64_t ldx, float* H, void* Hs,
                            float* hmeta) {
    if (!ctx) return ADADIM_ENULL;
    if (!Hs || !hmeta) return adadim_fail(ctx, ADADIM_ENULL, "adadim_hessian_prepared: Hs or hmeta is NULL");
    if (!aligned16(Hs) || !aligned16(hmeta))
        return adadim_fail(ctx, ADADIM_EALIGN, "adadim_hessian_prepared: Hs and hmeta must be 16-byte aligned");
    // the checks of adadim_hessian, then the fused launch
    if (!H) return adadim_fail(ctx, ADADIM_ENULL, "adadim_hessian_prepared: H is NULL");
    if (tokens < 0 || in <= 0 || ldx < in)
        return adadim_fail(ctx, ADADIM_EINVAL, "adadim_hessian_prepared: need tokens >= 0, in > 0, ldx >= in "
                                               "(tokens=%lld in=%lld ldx=%lld)",
                           (long long)tokens, (long long)in, (long long)ldx);
    if (in > (int64_t(1) << 20) || tokens > (int64_t(1) << 40))
        return adadim_fail(ctx, ADADIM_EINVAL, "adadim_hessian_prepared: size out of range");
    if (tokens > 0 && !X) return adadim_fail(ctx, ADADIM_ENULL, "adadim_hessian_prepared: X is NULL");
    if ((in % 8) != 0 || (ldx % 8) != 0 || !aligned16(X) || !aligned16(H))
        return adadim_fail(ctx, ADADIM_EALIGN,
                           "adadim_hessian_prepared: in and ldx must be multiples of 8, X and H 16-byte aligned");
    return launch_hessian_prepared(ctx, static_cast<const __half*>(X), tokens, in, ldx, H, static_cast<__half*>(Hs), hmeta);
}

static int check_error_args(adadim_ctx* ctx, const char* who, const void* dW, int dW_dtype, int64_t out,
                            int64_t in, const void* Hany, const float* loss, bool allow_scaled) {
    if (!dW || !Hany || !loss) return adadim_fail(ctx, ADADIM_ENULL, "%s: dW, H or loss is NULL", who);
    if (out <= 0 || in <= 0 || out > (int64_t(1) << 24) || in > (int64_t(1) << 20))
        return adadim_fail(ctx, ADADIM_EINVAL, "%s: bad shape out=%lld in=%lld", who, (long long)out,
                           (long long)in);
    const bool ok = dW_dtype == ADADIM_DW_F32 || dW_dtype == ADADIM_DW_F16 ||
                    (allow_scaled && dW_dtype == ADADIM_DW_F16_SCALED);
    if (!ok) return adadim_fail(ctx, ADADIM_EINVAL, "%s: dW_dtype %d not accepted here", who, dW_dtype);
    if ((in % 8) != 0 || !aligned16(dW) || !aligned16(Hany))
        return adadim_fail(ctx, ADADIM_EALIGN, "%s: in must be a multiple of 8, dW and H 16-byte aligned", who);
    return ADADIM_OK;
}

int adadim_layer_error(adadim_ctx* ctx, const void* dW, int dW_dtype, int64_t out, int64_t in, const float* H,
                       float* loss_rows, float* loss) {
    if (!ctx) return ADADIM_ENULL;
    int rc = check_error_args(ctx, "adadim_layer_error", dW, dW_dtype, out, in, H, loss, false);
    if (rc != ADADIM_OK) return rc;
    __half* Hs = static_cast<__half*>(adadim_workspace(ctx, WS_HS, size_t(score_elems(in, in)) * sizeof(__half)));
    float* hmeta = static_cast<float*>(adadim_workspace(ctx, WS_HMETA, size_t(in) * 2 * sizeof(float)));
    if (!Hs || !hmeta) return ADADIM_EHIP;
    rc = launch_hessian_prepare(ctx, H, in, Hs, hmeta);
    if (rc != ADADIM_OK) return rc;
    return launch_layer_error(ctx, 1, &dW, dW_dtype, out, in, Hs, hmeta, loss_rows, loss);
}

int adadim_layer_error_prepared(adadim_ctx* ctx, const void* dW, int dW_dtype, int64_t out, int64_t in,
                                const void* Hs, const float* hmeta, float* loss_rows, float* loss) {
    if (!ctx) return ADADIM_ENULL;
    int rc = check_error_args(ctx, "adadim_layer_error_prepared", dW, dW_dtype, out, in, Hs, loss, true);
    if (rc != ADADIM_OK) return rc;
    if (!hmeta) return adadim_fail(ctx, ADADIM_ENULL, "adadim_layer_error_prepared: hmeta is NULL");
    if (!aligned16(hmeta))
        return adadim_fail(ctx, ADADIM_EALIGN, "adadim_layer_error_prepared: hmeta must be 16-byte aligned");
    return launch_layer_error(ctx, 1, &dW, dW_dtype, out, in, static_cast<const __half*>(Hs), hmeta, loss_rows,
                              loss);
}

static int error_batch_checked(adadim_ctx* ctx, int n, const void* const* dW, int dW_dtype, int64_t out, int64_t in,
                               const void* Hs, const float* hmeta, float* loss_rows, float* losses, int32_t* best_dev) {
    if (!ctx) return ADADIM_ENULL;
    if (n <= 0 || n > 4096) return adadim_fail(ctx, ADADIM_EINVAL, "adadim_layer_error_batch: bad n=%d", n);
    if (!dW) return adadim_fail(ctx, ADADIM_ENULL, "adadim_layer_error_batch: dW is NULL");
    for (int c = 0; c < n; ++c) {
        int rc = check_error_args(ctx, "adadim_layer_error_batch", dW[c], dW_dtype, out, in, Hs, losses, true);
        if (rc != ADADIM_OK) return rc;
    }
    if (!hmeta) return adadim_fail(ctx, ADADIM_ENULL, "adadim_layer_error_batch: hmeta is NULL");
    if (!aligned16(hmeta))
        return adadim_fail(ctx, ADADIM_EALIGN, "adadim_layer_error_batch: hmeta must be 16-byte aligned");
    return launch_layer_error(ctx, n, dW, dW_dtype, out, in, static_cast<const __half*>(Hs), hmeta, loss_rows,
                              losses, best_dev);
}

int adadim_layer_error_batch(adadim_ctx* ctx, int n, const void* const* dW, int dW_dtype, int64_t out, int64_t in,
                             const void* Hs, const float* hmeta, float* loss_rows, float* losses) {
    return error_batch_checked(ctx, n, dW, dW_dtype, out, in, Hs, hmeta, loss_rows, losses, nullptr);
}

int adadim_layer_error_batch_select(adadim_ctx* ctx, int n, const void* const* dW, int dW_dtype, int64_t out,
                                    int64_t in, const void* Hs, const float* hmeta, float* loss_rows, float* losses,
                                    int32_t* best_dev) {
    if (ctx && !best_dev) return adadim_fail(ctx, ADADIM_ENULL, "adadim_layer_error_batch_select: best_dev is NULL");
    return error_batch_checked(ctx, n, dW, dW_dtype, out, in, Hs, hmeta, loss_rows, losses, best_dev);
}

int adadim_layer_error_batch_select_noalloc(adadim_ctx* ctx, int n, const void* const* dW, int64_t out, int64_t in,
                                            const void* Hs, const float* hmeta, float* loss_rows, float* losses,
                                            int32_t* best_dev) {
    if (!ctx) return ADADIM_ENULL;
    if (n <= 0 || n > 8)
        return adadim_fail(ctx, ADADIM_EINVAL, "adadim_layer_error_batch_select_noalloc: n must be in [1,8], got %d", n);
    if (!dW) return adadim_fail(ctx, ADADIM_ENULL, "adadim_layer_error_batch_select_noalloc: dW is NULL");
    if (!best_dev) return adadim_fail(ctx, ADADIM_ENULL, "adadim_layer_error_batch_select_noalloc: best_dev is NULL");
    for (int c = 0; c < n; ++c) {
        int rc = check_error_args(ctx, "adadim_layer_error_batch_select_noalloc", dW[c], ADADIM_DW_F16_SCALED, out, in, Hs,
                                  losses, true);
        if (rc != ADADIM_OK) return rc;
    }
    if (!hmeta) return adadim_fail(ctx, ADADIM_ENULL, "adadim_layer_error_batch_select_noalloc: hmeta is NULL");
    if (!aligned16(hmeta))
        return adadim_fail(ctx, ADADIM_EALIGN, "adadim_layer_error_batch_select_noalloc: hmeta must be 16-byte aligned");
    return launch_layer_error_noalloc(ctx, n, dW, out, in, static_cast<const __half*>(Hs), hmeta, loss_rows, losses,
                                      best_dev);
}

int64_t adadim_noalloc_scratch_bytes(int n, int64_t out, int64_t in) {
    if (n <= 0 || n > 8 || out <= 0 || in <= 0 || out > (int64_t(1) << 24) || in > (int64_t(1) << 20)) return -1;
    return launch_layer_error_noalloc_bytes(n, out, in);
}

int adadim_select(adadim_ctx* ctx, const float* losses, int n, int32_t* best_dev, int32_t* host_best) {
    if (!ctx) return ADADIM_ENULL;
    if (!losses) return adadim_fail(ctx, ADADIM_ENULL, "adadim_select: losses is NULL");
    if (n <= 0 || n > (1 << 20)) return adadim_fail(ctx, ADADIM_EINVAL, "adadim_select: bad n=%d", n);
    if (!best_dev && !host_best) return adadim_fail(ctx, ADADIM_ENULL, "adadim_select: no output given");
    int32_t* dst = best_dev;
    if (!dst) {
        dst = static_cast<int32_t*>(adadim_workspace(ctx, WS_SELECT, 256));
        if (!dst) return ADADIM_EHIP;
    }
    if (host_best && ctx->capturing)
        return adadim_fail(ctx, ADADIM_EINVAL, "adadim_select: no host output while a graph is being recorded");
    int rc = launch_select(ctx, losses, n, dst);
    if (rc != ADADIM_OK) return rc;
    if (host_best) {
        ADADIM_HIP_TRY(ctx, hipMemcpyAsync(host_best, dst, sizeof(int32_t), hipMemcpyDeviceToHost, ctx->stream));
        ADADIM_HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    }
    return ADADIM_OK;
}

int adadim_capture_begin(adadim_ctx* ctx) {
    if (!ctx) return ADADIM_ENULL;
    if (ctx->capturing) return adadim_fail(ctx, ADADIM_EINVAL, "adadim_capture_begin: already recording");
    if (!ctx->stream)
        return adadim_fail(ctx, ADADIM_EINVAL, "adadim_capture_begin: the context's stream is the default stream, "
                                               "which cannot be recorded; create the context on a stream of its own");
    ADADIM_HIP_TRY(ctx, hipStreamBeginCapture(ctx->stream, hipStreamCaptureModeRelaxed));
    ctx->capturing = true;
    return ADADIM_OK;
}

int adadim_capture_end(adadim_ctx* ctx, void** graph) {
    if (!ctx) return ADADIM_ENULL;
    if (!ctx->capturing) return adadim_fail(ctx, ADADIM_EINVAL, "adadim_capture_end: not recording");
    ctx->capturing = false;
    hipGraph_t g = nullptr;
    ADADIM_HIP_TRY(ctx, hipStreamEndCapture(ctx->stream, &g));   // also ends a recording that a failed call broke
    if (!graph) {
        (void)hipGraphDestroy(g);
        return adadim_fail(ctx, ADADIM_ENULL, "adadim_capture_end: graph is NULL");
    }
    hipGraphExec_t exec = nullptr;
    const hipError_t e = hipGraphInstantiate(&exec, g, nullptr, nullptr, 0);
    (void)hipGraphDestroy(g);
    if (e != hipSuccess) return adadim_fail(ctx, ADADIM_EHIP, "hipGraphInstantiate: %s", hipGetErrorString(e));
    *graph = exec;
    return ADADIM_OK;
}

int adadim_graph_launch(adadim_ctx* ctx, void* graph) {
    if (!ctx) return ADADIM_ENULL;
    if (!graph) return adadim_fail(ctx, ADADIM_ENULL, "adadim_graph_launch: graph is NULL");
    if (ctx->capturing) return adadim_fail(ctx, ADADIM_EINVAL, "adadim_graph_launch: still recording");
    ADADIM_HIP_TRY(ctx, hipGraphLaunch(static_cast<hipGraphExec_t>(graph), ctx->stream));
    return ADADIM_OK;
}

void adadim_graph_destroy(void* graph) {
    if (graph) (void)hipGraphExecDestroy(static_cast<hipGraphExec_t>(graph));
}

// shared by the two matrix-vector entry points; meta16: `scales` holds the 16-bit group words and zeros is unused
static int gemv_ic_checked(adadim_ctx* ctx, const char* who, const uint32_t* packed, const void* scales, const uint8_t* zeros,
                           const void* x, int64_t out, int64_t in, int bits, int group, void* y, bool meta16) {
    if (!ctx) return ADADIM_ENULL;
    if (!packed || !scales || (!meta16 && !zeros) || !x || !y) return adadim_fail(ctx, ADADIM_ENULL, "%s: NULL argument", who);
    if (out <= 0 || in <= 0 || out > (int64_t(1) << 24) || in > (int64_t(1) << 24))
        return adadim_fail(ctx, ADADIM_EINVAL, "%s: bad shape out=%lld in=%lld", who, (long long)out, (long long)in);
    if (bits < 2 || bits > 4) return adadim_fail(ctx, ADADIM_EINVAL, "%s: bits must be 2, 3 or 4, got %d", who, bits);
    const int64_t g = group == 0 ? out : group;
    if (group < 0 || (out % g) != 0 || (g % 32) != 0)
        return adadim_fail(ctx, ADADIM_EINVAL, "%s: group %d must be 0 or a multiple of 32 that divides out (%lld)", who,
                           group, (long long)out);
    if ((in % 4) != 0) return adadim_fail(ctx, ADADIM_EINVAL, "%s: in must be a multiple of 4", who);
    if (g > (int64_t(1) << 30)) return adadim_fail(ctx, ADADIM_EINVAL, "%s: group too long", who);
    if (!aligned16(packed) || (reinterpret_cast<uintptr_t>(x) & 7u) || (reinterpret_cast<uintptr_t>(y) & 1u))
        return adadim_fail(ctx, ADADIM_EALIGN, "%s: packed must be 16-byte, x 8-byte, y 2-byte aligned", who);
    if (meta16 ? (reinterpret_cast<uintptr_t>(scales) & 7u) != 0
               : (!aligned16(scales) || (reinterpret_cast<uintptr_t>(zeros) & 3u) != 0))
        return adadim_fail(ctx, ADADIM_EALIGN, "%s: scales must be 16-byte and zeros 4-byte aligned (group words: 8-byte)",
                           who);
    return launch_gemv_ic(ctx, packed, scales, zeros, static_cast<const __half*>(x), out, in, bits, static_cast<int>(g),
                          static_cast<__half*>(y), meta16);
}

int adadim_gemv_ic(adadim_ctx* ctx, const uint32_t* packed, const float* scales, const uint8_t* zeros, const void* x,
                   int64_t out, int64_t in, int bits, int group, void* y) {
    return gemv_ic_checked(ctx, "adadim_gemv_ic", packed, scales, zeros, x, out, in, bits, group, y, false);
}

int adadim_gemv_ic_meta16(adadim_ctx* ctx, const uint32_t* packed, const uint16_t* meta, const void* x, int64_t out,
                          int64_t in, int bits, int group, void* y) {
    return gemv_ic_checked(ctx, "adadim_gemv_ic_meta16", packed, meta, nullptr, x, out, in, bits, group, y, true);
}

int adadim_gptq_prepare(adadim_ctx* ctx, const float* H, int64_t in, float percdamp, int act_order, int32_t* perm,
                        uint8_t* dead, float* U) {
    if (!ctx) return ADADIM_ENULL;
    if (!H || !perm || !dead || !U) return adadim_fail(ctx, ADADIM_ENULL, "adadim_gptq_prepare: NULL argument");
    if (in <= 0 || in > 46340) return adadim_fail(ctx, ADADIM_EINVAL, "adadim_gptq_prepare: bad in=%lld", (long long)in);
    if (!(percdamp >= 0.0f && percdamp <= 1.0f) || (act_order != 0 && act_order != 1))
        return adadim_fail(ctx, ADADIM_EINVAL, "adadim_gptq_prepare: percdamp must be in [0,1], act_order 0 or 1");
    return launch_gptq_prepare(ctx, H, in, percdamp, act_order, perm, dead, U);
}

// shared by the two sweep entry points; mfmt != 0: parameters travel as 16-bit group words (static_scales / scales are
// then u16 arrays and the zero arrays are unused)
static int gptq_quantize_checked(adadim_ctx* ctx, const char* who, const void* W, int64_t out, int64_t in, int dim, int bits,
                                 int group, const float* U, const int32_t* perm, const uint8_t* dead,
                                 const float* static_scales, const uint8_t* static_zeros, uint8_t* codes, float* scales,
                                 uint8_t* zeros, float* dW, uint32_t* packed, int mfmt) {
    if (!ctx) return ADADIM_ENULL;
    if (!W || !U || !perm || !dead || !codes)
        return adadim_fail(ctx, ADADIM_ENULL, "%s: W, U, perm, dead or codes is NULL", who);
    if (out <= 0 || in <= 0 || out > 500000 || in > 46340)
        return adadim_fail(ctx, ADADIM_EINVAL, "%s: bad shape out=%lld in=%lld", who, (long long)out, (long long)in);
    if (dim != ADADIM_DIM_OC && dim != ADADIM_DIM_IC)
        return adadim_fail(ctx, ADADIM_EINVAL, "%s: dim must be 0 (OC) or 1 (IC), got %d", who, dim);
    if (bits < 2 || bits > (mfmt ? 4 : 8))
        return adadim_fail(ctx, ADADIM_EINVAL, "%s: bits must be in [2,%d]", who, mfmt ? 4 : 8);
    if (dim == ADADIM_DIM_OC) {
        const int64_t g = group == 0 ? in : group;
        if (group < 0 || (in % g) != 0) return adadim_fail(ctx, ADADIM_EINVAL, "%s: group %d must be 0 or divide in", who, group);
        if (!static_scales || (!mfmt && !static_zeros))
            return adadim_fail(ctx, ADADIM_ENULL, "%s: per-OC needs the static parameters", who);
        const int rc = launch_gptq_quantize(ctx, static_cast<const __half*>(W), out, in, dim, bits, static_cast<int>(g), U,
                                            perm, dead, static_scales, static_zeros, codes, nullptr, nullptr, dW, mfmt);
        if (rc != ADADIM_OK) return rc;
    } else {
        if ((group != 64 && group != 128) || (out % group) != 0)
            return adadim_fail(ctx, ADADIM_EINVAL, "%s: per-IC groups of 64 or 128 rows dividing out are supported, got %d", who,
                               group);
        if (!scales || (!mfmt && !zeros)) return adadim_fail(ctx, ADADIM_ENULL, "%s: per-IC needs the parameter outputs", who);
        const int rc = launch_gptq_quantize(ctx, static_cast<const __half*>(W), out, in, dim, bits, group, U, perm, dead,
                                            nullptr, nullptr, codes, scales, zeros, dW, mfmt);
        if (rc != ADADIM_OK) return rc;
    }
    if (packed) return launch_pack(ctx, codes, out, in, dim, bits, packed);
    return ADADIM_OK;
}

int adadim_gptq_quantize(adadim_ctx* ctx, const void* W, int64_t out, int64_t in, int dim, int bits, int group,
                         const float* U, const int32_t* perm, const uint8_t* dead, const float* static_scales,
                         const uint8_t* static_zeros, uint8_t* codes, float* scales, uint8_t* zeros, float* dW,
                         uint32_t* packed) {
    return gptq_quantize_checked(ctx, "adadim_gptq_quantize", W, out, in, dim, bits, group, U, perm, dead, static_scales,
                                 static_zeros, codes, scales, zeros, dW, packed, 0);
}

int adadim_gptq_quantize_meta16(adadim_ctx* ctx, const void* W, int64_t out, int64_t in, int dim, int bits, int group,
                                const float* U, const int32_t* perm, const uint8_t* dead, const uint16_t* static_meta,
                                uint8_t* codes, uint16_t* meta, float* dW, uint32_t* packed) {
    return gptq_quantize_checked(ctx, "adadim_gptq_quantize_meta16", W, out, in, dim, bits, group, U, perm, dead,
                                 reinterpret_cast<const float*>(static_meta), nullptr, codes,
                                 reinterpret_cast<float*>(meta), nullptr, dW, packed, bits);
}

}  // extern "C"
