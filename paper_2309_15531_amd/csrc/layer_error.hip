// Reconstruction error of a quantization candidate (Eq. 1 of Sec. 3.3, squared)
// as the quadratic form  L = tr(dW H dW^T) = sum_o dW_o H dW_o^T,  and the
// first-minimum selection over candidates (App. B procedure).
//
// H is symmetric, so with the scaled strictly-lower triangle Hs and the
// diagonal kept apart in fp32,
//     L_o = sum_j H_jj dW_oj^2  +  2 * sum_n ( sum_{k<n} dW'_ok Hs_nk ) dW'_on ,
// dW' = dW * colscale.  The inner sums are a GEMM E = dW' * Hs^T restricted to
// k < n (half the flops of the full product), run on the matrix cores with
// fp16 operands and fp32 accumulation; E is never stored: the epilogue
// multiplies each tile by the matching dW' entries and reduces along n.
// Row partials are combined in a fixed order (no atomics), so results are
// bit-reproducible.
#include "common.h"
#include "mfma_tile.h"
#include "error_dma.h"


namespace {

using namespace mfma;

// dW (fp32 / fp16 / already scaled fp16) -> dW16 = fp16(dW * d) in the scoring layout if needed, and
// diag[o] = sum_j H_jj dW_oj^2 in fp32.  One block per row.
struct SrcBatch {
    const void* dW[edma::MAX_BATCH];
};

// blockIdx.y = candidate; dW16 and diag are laid out [candidate][...].
__global__ __launch_bounds__(256) void error_prologue(SrcBatch src, int dW_dtype, int64_t out, int64_t in,
                                                      const float* __restrict__ hmeta,
                                                      __half* __restrict__ dW16_all, float* __restrict__ diag_all) {
    __shared__ float s_red[256];
    const int64_t o = blockIdx.x;
    const void* __restrict__ dW = src.dW[blockIdx.y];
    __half* __restrict__ dW16 = dW16_all ? dW16_all + int64_t(blockIdx.y) * score_elems(out, in) : nullptr;
    float* __restrict__ diag = diag_all + int64_t(blockIdx.y) * out;
    const float* d = hmeta;
    const float* hd = hmeta + in;
    float sum = 0.0f;
    for (int64_t j0 = int64_t(threadIdx.x) * 8; j0 < in; j0 += 256 * 8) {
        float w[8];
        if (dW_dtype == ADADIM_DW_F32) {
            const float4 a = *reinterpret_cast<const float4*>(static_cast<const float*>(dW) + o * in + j0);
            const float4 b = *reinterpret_cast<const float4*>(static_cast<const float*>(dW) + o * in + j0 + 4);
            w[0] = a.x; w[1] = a.y; w[2] = a.z; w[3] = a.w; w[4] = b.x; w[5] = b.y; w[6] = b.z; w[7] = b.w;
        } else {
            const int64_t at = dW_dtype == ADADIM_DW_F16_SCALED ? score_index(o, j0, out, in) : o * in + j0;
            const uint4 raw = *reinterpret_cast<const uint4*>(static_cast<const __half*>(dW) + at);
            const __half2* h = reinterpret_cast<const __half2*>(&raw);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float2 f = __half22float2(h[i]);
                w[2 * i] = f.x;
                w[2 * i + 1] = f.y;
            }
        }
        const float4 da = *reinterpret_cast<const float4*>(d + j0), db = *reinterpret_cast<const float4*>(d + j0 + 4);
        const float4 ha = *reinterpret_cast<const float4*>(hd + j0), hb = *reinterpret_cast<const float4*>(hd + j0 + 4);
        const float dd[8] = {da.x, da.y, da.z, da.w, db.x, db.y, db.z, db.w};
        const float hh[8] = {ha.x, ha.y, ha.z, ha.w, hb.x, hb.y, hb.z, hb.w};
        if (dW_dtype == ADADIM_DW_F16_SCALED) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const float u = w[i] / dd[i];  // exact: d is a power of two
                sum += hh[i] * (u * u);
            }
        } else {
            uint4 o16;
            __half2* h = reinterpret_cast<__half2*>(&o16);
#pragma unroll
            for (int i = 0; i < 8; ++i) sum += hh[i] * (w[i] * w[i]);
#pragma unroll
            for (int i = 0; i < 4; ++i) h[i] = __floats2half2_rn(w[2 * i] * dd[2 * i], w[2 * i + 1] * dd[2 * i + 1]);
            *reinterpret_cast<uint4*>(dW16 + score_index(o, j0, out, in)) = o16;
        }
    }
    s_red[threadIdx.x] = sum;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if (threadIdx.x < s) s_red[threadIdx.x] += s_red[threadIdx.x + s];
        __syncthreads();
    }
    if (threadIdx.x == 0) diag[o] = s_red[0];
}

// loss_rows[o] = diag[o] + 2*sum_slot part[slot,o] (no diag array: the tile kernel has put half
// the diagonal term into its row sums) for 256 rows per block, a per-block total,
// and, in the block that finishes last, loss = sum of the block totals in block order (so the
// result does not depend on which block that is).  `ticket` must be zero on entry and is zero
// again on exit.  With `best` given, the block that writes the launch's last loss also takes the
// argmin of sel_losses[0..n_sel) (first minimum, NaN never wins, as select_first_min): one launch
// and one kernel boundary less than a separate selection.
__global__ __launch_bounds__(256) void error_finish(const float* __restrict__ diag_all,
                                                    const float* __restrict__ part_all, int64_t out, int n_slots,
                                                    float* __restrict__ loss_rows_all, float* __restrict__ loss_all,
                                                    double* __restrict__ block_tot_all,
                                                    unsigned int* __restrict__ ticket_all,
                                                    const float* __restrict__ sel_losses, int n_sel,
                                                    int32_t* __restrict__ best) {
    __shared__ double s_red[256];
    __shared__ bool s_last;
    // blockIdx.y = candidate
    const float* __restrict__ diag = diag_all + int64_t(blockIdx.y) * out;
    const float* __restrict__ part = part_all + int64_t(blockIdx.y) * n_slots * out;
    float* __restrict__ loss_rows = loss_rows_all ? loss_rows_all + int64_t(blockIdx.y) * out : nullptr;
    float* __restrict__ loss = loss_all + blockIdx.y;
    double* __restrict__ block_tot = block_tot_all + int64_t(blockIdx.y) * gridDim.x;
    unsigned int* __restrict__ ticket = ticket_all + blockIdx.y;
    const int64_t o = int64_t(blockIdx.x) * 256 + threadIdx.x;
    double mine = 0.0;
    if (o < out) {
        float off = 0.0f;
        for (int sl = 0; sl < n_slots; ++sl) off += part[int64_t(sl) * out + o];
        const float l = (diag_all ? diag[o] : 0.0f) + 2.0f * off;
        if (loss_rows) loss_rows[o] = l;
        mine = static_cast<double>(l);
    }
    s_red[threadIdx.x] = mine;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if (threadIdx.x < s) s_red[threadIdx.x] += s_red[threadIdx.x + s];
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        block_tot[blockIdx.x] = s_red[0];
        __threadfence();
        s_last = atomicAdd(ticket, 1u) == gridDim.x - 1;
    }
    __syncthreads();
    if (!s_last) return;
    __threadfence();
    double tot = 0.0;
    for (unsigned b = threadIdx.x; b < gridDim.x; b += 256) tot += __builtin_nontemporal_load(block_tot + b);
    s_red[threadIdx.x] = tot;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if (threadIdx.x < s) s_red[threadIdx.x] += s_red[threadIdx.x + s];
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        *loss = static_cast<float>(s_red[0]);
        *ticket = 0u;
        if (best) {
            unsigned int* done = ticket_all + 32;             // candidates of this launch whose loss is written
            __threadfence();
            if (atomicAdd(done, 1u) == gridDim.y - 1) {
                __threadfence();
                int b = -1;
                float bv = 0.0f;
                for (int i = 0; i < n_sel; ++i) {
                    const float v = __builtin_nontemporal_load(sel_losses + i);
                    if (v != v) continue;
                    if (b < 0 || v < bv) {
                        b = i;
                        bv = v;
                    }
                }
                *best = b < 0 ? 0 : b;
                *done = 0u;
            }
        }
    }
}

__global__ void fill_zero_f32(float* p, int64_t n) {
    const int64_t i = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0.0f;
}

__global__ void select_first_min(const float* __restrict__ losses, int n, int32_t* __restrict__ best) {
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    int b = -1;
    float bv = 0.0f;
    for (int i = 0; i < n; ++i) {
        const float v = losses[i];
        if (v != v) continue;            // NaN never wins
        if (b < 0 || v < bv) {
            b = i;
            bv = v;
        }
    }
    *best = b < 0 ? 0 : b;
}

// Scratch of one scoring launch, wherever it lives (the context's growing slots, or the fixed device array of the
// entry point that may not allocate).
struct ErrScratch {
    float* part;             // per candidate [n_slots, out] row partials
    float* diag;             // per candidate [out] diagonal terms (prologue path only)
    double* block_tot;       // per candidate one double per 256 rows
    unsigned int* ticket;    // 64 counters, zero between launches
    const void* zero16;      // at least 256 zero bytes
    __half* dW16;            // per candidate scaled copy of dW (prologue path only)
};

// Contraction chunk of a launch of nc candidates, in 256-k blocks, and the number of (chunk, column block) slots:
// whole contractions (one workgroup per tile, the cheapest in prologues and epilogues) unless that leaves fewer
// than two workgroups per compute unit; then the largest chunk that gives that many.
void error_slots(int nc, int MB, int NB, int64_t in, int& kb, int& n_slots) {
    constexpr int BT = edma::BT;
    kb = NB;
    for (;;) {
        n_slots = 0;
        for (int nb = 0; nb < NB; ++nb) {
            const int64_t kend = in < int64_t(nb + 1) * BT ? in : int64_t(nb + 1) * BT;
            n_slots += static_cast<int>((kend + int64_t(kb) * BT - 1) / (int64_t(kb) * BT));
        }
        if (kb == 1 || int64_t(nc) * MB * n_slots >= 512) break;
        kb = kb > 2 ? kb / 2 : 1;
    }
}

int set_error_attr(adadim_ctx* ctx) {
    static PerDeviceOnce once;
    const hipError_t err = once.run([] {
        return hipFuncSetAttribute(reinterpret_cast<const void*>(edma::error_tiles_dma<0>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, edma::SMEM_BYTES);
    });
    if (err != hipSuccess)
        return adadim_fail(ctx, ADADIM_EHIP, "hipFuncSetAttribute(error_tiles): %s", hipGetErrorString(err));
    return ADADIM_OK;
}

// One launch group: nc <= MAX_BATCH candidates dW[0..nc) scored against Hs; losses_all / n_all are the whole
// call's loss array (for the fused selection, taken when best_dev is given).
int run_error_batch(adadim_ctx* ctx, int nc, const void* const* dW, int dW_dtype, int64_t out, int64_t in,
                    const __half* Hs, const float* hmeta, float* loss_rows, float* losses, const float* losses_all,
                    int n_all, int32_t* best_dev, const ErrScratch& sc, int kb, int n_slots) {
    constexpr int BT = edma::BT;
    const int MB = static_cast<int>((out + BT - 1) / BT), NB = static_cast<int>((in + BT - 1) / BT);
    const int kc_len = kb * BT;
    const unsigned fin_blocks = static_cast<unsigned>((out + 255) / 256);
    SrcBatch src;
    edma::Batch batch;
    batch.n = nc;
    for (int c = 0; c < edma::MAX_BATCH; ++c) {
        src.dW[c] = c < nc ? dW[c] : nullptr;
        batch.A[c] = c < nc ? (sc.dW16 ? sc.dW16 + size_t(c) * size_t(score_elems(out, in))
                                       : static_cast<const __half*>(dW[c]))
                            : nullptr;
    }
    // Column-scaled fp16 input is consumed as it is and the tile kernel adds the diagonal term;
    // other inputs go through the prologue, which scales them and takes that term in fp32.
    const bool direct = dW_dtype == ADADIM_DW_F16_SCALED;
    if (!direct) {
        ProfScope prof(ctx, "error_prologue");
        hipLaunchKernelGGL(error_prologue, dim3(static_cast<unsigned>(out), nc), dim3(256), 0, ctx->stream, src,
                           dW_dtype, out, in, hmeta, sc.dW16, sc.diag);
    }
    ADADIM_LAUNCH_CHECK(ctx, "error_prologue");
    {
        ProfScope prof(ctx, "error_tiles");
        // units of 4 slots x 8 (candidate, row block) pairs, 32 workgroups each, dealt to 8 XCDs
        const int n_units = ((n_slots + 3) / 4) * ((nc * MB + 7) / 8);
        const unsigned grid = 8u * static_cast<unsigned>((n_units + 7) / 8) * 32u;
        hipLaunchKernelGGL(edma::error_tiles_dma<0>, dim3(grid), dim3(256), edma::SMEM_BYTES, ctx->stream, batch, Hs,
                           out, in, MB, NB, kc_len, n_slots, sc.zero16, direct ? hmeta : nullptr, sc.part);
    }
    ADADIM_LAUNCH_CHECK(ctx, "error_tiles");
    {
        ProfScope prof(ctx, "error_finish");
        hipLaunchKernelGGL(error_finish, dim3(fin_blocks, nc), dim3(256), 0, ctx->stream,
                           direct ? static_cast<const float*>(nullptr) : sc.diag, sc.part, out, n_slots, loss_rows,
                           losses, sc.block_tot, sc.ticket, losses_all, n_all, best_dev);
    }
    ADADIM_LAUNCH_CHECK(ctx, "error_finish");
    return ADADIM_OK;
}

}  // namespace

int launch_layer_error(adadim_ctx* ctx, int n, const void* const* dW, int dW_dtype, int64_t out, int64_t in,
                       const __half* Hs, const float* hmeta, float* loss_rows, float* losses, int32_t* best_dev) {
    constexpr int BT = edma::BT;
    const int MB = static_cast<int>((out + BT - 1) / BT), NB = static_cast<int>((in + BT - 1) / BT);
    ErrScratch sc{};
    void* zero16 = adadim_workspace(ctx, WS_ZERO, 256);
    if (!zero16) return ADADIM_EHIP;
    sc.zero16 = zero16;
    if (ctx->zero_ready_bytes != ctx->ws_bytes[WS_ZERO]) {
        // a fill kernel rather than a memset node, so that the call stays safe to capture in a graph
        const int64_t nz = static_cast<int64_t>(ctx->ws_bytes[WS_ZERO] / 4);
        hipLaunchKernelGGL(fill_zero_f32, dim3(static_cast<unsigned>((nz + 255) / 256)), dim3(256), 0, ctx->stream,
                           static_cast<float*>(zero16), nz);
        ADADIM_LAUNCH_CHECK(ctx, "fill_zero_f32");
        ctx->zero_ready_bytes = ctx->ws_bytes[WS_ZERO];
    }
    int rc = set_error_attr(ctx);
    if (rc != ADADIM_OK) return rc;
    for (int c0 = 0; c0 < n; c0 += edma::MAX_BATCH) {
        const int nc = n - c0 < edma::MAX_BATCH ? n - c0 : edma::MAX_BATCH;
        int kb = 0, n_slots = 0;
        error_slots(nc, MB, NB, in, kb, n_slots);
        // scratch: per candidate [n_slots, out] row partials; then per candidate [out] diagonal terms
        sc.part = static_cast<float*>(adadim_workspace(
            ctx, WS_ERR_PART, size_t(nc) * size_t(n_slots + 1) * size_t(out) * sizeof(float)));
        if (!sc.part) return ADADIM_EHIP;
        sc.diag = sc.part + size_t(nc) * size_t(n_slots) * size_t(out);
        // scratch of the final reduction: per candidate one double per 256 rows; then the tickets
        const unsigned fin_blocks = static_cast<unsigned>((out + 255) / 256);
        const size_t fin_bytes = size_t(edma::MAX_BATCH) * fin_blocks * sizeof(double) + 256;
        const bool fin_fresh = ctx->ws_bytes[WS_ERR_FIN] < fin_bytes;
        sc.block_tot = static_cast<double*>(adadim_workspace(ctx, WS_ERR_FIN, fin_bytes));
        if (!sc.block_tot) return ADADIM_EHIP;
        sc.ticket = reinterpret_cast<unsigned int*>(sc.block_tot + (ctx->ws_bytes[WS_ERR_FIN] - 256) / sizeof(double));
        if (fin_fresh) {
            hipLaunchKernelGGL(fill_zero_f32, dim3(1), dim3(64), 0, ctx->stream, reinterpret_cast<float*>(sc.ticket),
                               int64_t(64));
            ADADIM_LAUNCH_CHECK(ctx, "fill_zero_f32");
        }
        sc.dW16 = nullptr;
        if (dW_dtype != ADADIM_DW_F16_SCALED) {
            sc.dW16 = static_cast<__half*>(
                adadim_workspace(ctx, WS_DW16, size_t(nc) * size_t(score_elems(out, in)) * sizeof(__half)));
            if (!sc.dW16) return ADADIM_EHIP;
        }
        rc = run_error_batch(ctx, nc, dW + c0, dW_dtype, out, in, Hs, hmeta,
                             loss_rows ? loss_rows + size_t(c0) * size_t(out) : nullptr, losses + c0, losses, n,
                             c0 + nc == n ? best_dev : nullptr, sc, kb, n_slots);
        if (rc != ADADIM_OK) return rc;
    }
    return ADADIM_OK;
}

int launch_select(adadim_ctx* ctx, const float* losses, int n, int32_t* best_dev) {
    {
        ProfScope prof(ctx, "select_first_min");
        hipLaunchKernelGGL(select_first_min, dim3(1), dim3(64), 0, ctx->stream, losses, n, best_dev);
    }
    ADADIM_LAUNCH_CHECK(ctx, "select_first_min");
    return ADADIM_OK;
}

// ---------------------------------------------------------------------------------------------
// The scoring call for callers that cannot allocate (code under graph capture, tight serving loops,
// harnesses that forbid hipMalloc): the scratch of the launch lives in a fixed device array instead
// of the context's growing slots.  Layout of the array: [0, 256) zero page (never written after the
// first clear), [256, 512) the 64 counters of error_finish, [512, 512 + 8*MAX_BATCH*fin_blocks)
// block totals, then the row partials.
namespace {

constexpr size_t NOALLOC_SCRATCH_BYTES = size_t(16) << 20;
constexpr int NOALLOC_MAX_DEVICES = 64;

}  // namespace

static __device__ __align__(256) unsigned char scratch[NOALLOC_SCRATCH_BYTES];

namespace {

// Device address of `scratch` on each GPU (every GPU holds its own copy of the array at its own address);
// looked up once per device, with that device current.
std::mutex g_scratch_mutex;
unsigned char* g_scratch_ptr[NOALLOC_MAX_DEVICES] = {};

int noalloc_scratch(adadim_ctx* ctx, unsigned char** out_ptr, bool* first_use) {
    int dev = -1;
    ADADIM_HIP_TRY(ctx, hipGetDevice(&dev));
    if (dev < 0 || dev >= NOALLOC_MAX_DEVICES)
        return adadim_fail(ctx, ADADIM_EINVAL, "adadim_layer_error_batch_select_noalloc: device index %d out of range", dev);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    *first_use = false;
    if (!g_scratch_ptr[dev]) {
        unsigned char* ptr = nullptr;
        const hipError_t e = hipGetSymbolAddress(reinterpret_cast<void**>(&ptr), HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr)
            return adadim_fail(ctx, ADADIM_EHIP, "hipGetSymbolAddress(scratch) on device %d: %s", dev, hipGetErrorString(e));
        g_scratch_ptr[dev] = ptr;
        *first_use = true;
    }
    *out_ptr = g_scratch_ptr[dev];
    return ADADIM_OK;
}

}  // namespace

int64_t launch_layer_error_noalloc_bytes(int n, int64_t out, int64_t in) {
    constexpr int BT = edma::BT;
    const int MB = static_cast<int>((out + BT - 1) / BT), NB = static_cast<int>((in + BT - 1) / BT);
    int kb = 0, n_slots = 0;
    error_slots(n, MB, NB, in, kb, n_slots);
    const int64_t fin_blocks = (out + 255) / 256;
    return 512 + int64_t(edma::MAX_BATCH) * fin_blocks * 8 + int64_t(n) * n_slots * out * 4;
}

int launch_layer_error_noalloc(adadim_ctx* ctx, int n, const void* const* dW, int64_t out, int64_t in, const __half* Hs,
                               const float* hmeta, float* loss_rows, float* losses, int32_t* best_dev) {
    constexpr int BT = edma::BT;
    const int MB = static_cast<int>((out + BT - 1) / BT), NB = static_cast<int>((in + BT - 1) / BT);
    int kb = 0, n_slots = 0;
    error_slots(n, MB, NB, in, kb, n_slots);
    const int64_t need = launch_layer_error_noalloc_bytes(n, out, in);
    if (need > int64_t(NOALLOC_SCRATCH_BYTES))
        return adadim_fail(ctx, ADADIM_EINVAL,
                           "adadim_layer_error_batch_select_noalloc: %d candidates of [%lld, %lld] need %lld bytes of scratch, "
                           "the fixed array holds %lld", n, (long long)out, (long long)in, (long long)need,
                           (long long)NOALLOC_SCRATCH_BYTES);
    unsigned char* ptr = nullptr;
    bool first_use = false;
    int rc = noalloc_scratch(ctx, &ptr, &first_use);
    if (rc != ADADIM_OK) return rc;
    rc = set_error_attr(ctx);
    if (rc != ADADIM_OK) return rc;
    // The zero page and the counters must be zero on entry.  The array keeps the last call's contents (the
    // counters are left at zero by a launch that ran to its end, but not by one that was abandoned), so the
    // first 512 bytes are cleared on every call, by a fill kernel (a memset node would not be safe to record).
    hipLaunchKernelGGL(fill_zero_f32, dim3(1), dim3(128), 0, ctx->stream, reinterpret_cast<float*>(ptr), int64_t(128));
    ADADIM_LAUNCH_CHECK(ctx, "fill_zero_f32");
    const int64_t fin_blocks = (out + 255) / 256;
    ErrScratch sc{};
    sc.zero16 = ptr;
    sc.ticket = reinterpret_cast<unsigned int*>(ptr + 256);
    sc.block_tot = reinterpret_cast<double*>(ptr + 512);
    sc.part = reinterpret_cast<float*>(ptr + 512 + size_t(edma::MAX_BATCH) * size_t(fin_blocks) * 8);
    sc.diag = nullptr;
    sc.dW16 = nullptr;
    return run_error_batch(ctx, n, dW, ADADIM_DW_F16_SCALED, out, in, Hs, hmeta, loss_rows, losses, losses, n, best_dev, sc,
                           kb, n_slots);
}
