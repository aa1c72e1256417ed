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

namespace {

using namespace mfma;

// dW (fp32 / fp16 / already scaled fp16) -> dW16 = fp16(dW * d) if needed, and
// diag[o] = sum_j H_jj dW_oj^2 in fp32.  One block per row.
__global__ __launch_bounds__(256) void error_prologue(const void* __restrict__ dW, int dW_dtype, int64_t in,
                                                      const float* __restrict__ hmeta,
                                                      __half* __restrict__ dW16, float* __restrict__ diag) {
    __shared__ float s_red[256];
    const int64_t o = blockIdx.x;
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
            const uint4 raw = *reinterpret_cast<const uint4*>(static_cast<const __half*>(dW) + o * in + j0);
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
            *reinterpret_cast<uint4*>(dW16 + o * in + j0) = o16;
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

// One workgroup per (row block, column block) tile of E, longest contraction
// first.  part[nb*out + o] = sum over the tile's columns n of E[o,n]*dW'[o,n].
template <int BM, int BN, int WGM, int WGN>
__global__ __launch_bounds__(THREADS) void error_tiles(const __half* __restrict__ A, const __half* __restrict__ Hs,
                                                       int64_t out, int64_t in, int MB, int NB,
                                                       float* __restrict__ part) {
    static_assert(WGM * WGN == 4, "four wavefronts");
    constexpr int WM = BM / WGM, WN = BN / WGN, TM = WM / 32, TN = WN / 32;
    extern __shared__ __align__(16) char smem[];
    constexpr int A_BYTES = BM * ROW_BYTES, B_BYTES = BN * ROW_BYTES;
    auto sA = [&](int b) { return smem + b * (A_BYTES + B_BYTES); };
    auto sB = [&](int b) { return smem + b * (A_BYTES + B_BYTES) + A_BYTES; };
    __shared__ float s_rows[WGN][BM];

    const int nb = NB - 1 - static_cast<int>(blockIdx.x / MB);
    const int mb = static_cast<int>(blockIdx.x % MB);
    const int64_t row0 = int64_t(mb) * BM, col0 = int64_t(nb) * BN;
    const int64_t k_end = min(in, col0 + BN);  // Hs[n,k] = 0 for k >= n

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    DirectStage<BM> ga;
    DirectStage<BN> gb;
    ga.load(A, in, row0, out, 0, k_end, tid);
    gb.load(Hs, in, col0, in, 0, k_end, tid);
    ga.store(sA(0), tid);
    gb.store(sB(0), tid);
    __syncthreads();
    int buf = 0;
    for (int64_t k0 = 0; k0 < k_end; k0 += KT) {
        const bool more = k0 + KT < k_end;
        if (more) {
            ga.load(A, in, row0, out, k0 + KT, k_end, tid);
            gb.load(Hs, in, col0, in, k0 + KT, k_end, tid);
        }
        mma_stage<TM, TN>(sA(buf), sB(buf), wm * WM, wn * WN, lane, acc);
        if (more) {
            ga.store(sA(buf ^ 1), tid);
            gb.store(sB(buf ^ 1), tid);
        }
        __syncthreads();
        buf ^= 1;
    }

    // epilogue: row sums of E .* dW' over this tile's columns
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int lrow = wm * WM + 32 * i + acc_row(r, lane);
            const int64_t row = row0 + lrow;
            float v = 0.0f;
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int64_t col = col0 + wn * WN + 32 * j + (lane & 31);
                if (row < out && col < in) v += acc[i][j][r] * __half2float(A[row * in + col]);
            }
#pragma unroll
            for (int m = 1; m < 32; m <<= 1) v += __shfl_xor(v, m, 64);
            if ((lane & 31) == 0) s_rows[wn][lrow] = v;
        }
    }
    __syncthreads();
    for (int r = tid; r < BM; r += THREADS) {
        float v = s_rows[0][r];
#pragma unroll
        for (int w = 1; w < WGN; ++w) v += s_rows[w][r];
        if (row0 + r < out) part[int64_t(nb) * out + row0 + r] = v;
    }
}

// loss_rows[o] = diag[o] + 2*sum_nb part[nb,o];  loss = sum_o loss_rows[o].  One block.
__global__ __launch_bounds__(1024) void error_finish(const float* __restrict__ diag, const float* __restrict__ part,
                                                     int64_t out, int NB, float* __restrict__ loss_rows,
                                                     float* __restrict__ loss) {
    __shared__ double s_red[1024];
    double tot = 0.0;
    for (int64_t o = threadIdx.x; o < out; o += 1024) {
        float off = 0.0f;
        for (int nb = 0; nb < NB; ++nb) off += part[int64_t(nb) * out + o];
        const float l = diag[o] + 2.0f * off;
        if (loss_rows) loss_rows[o] = l;
        tot += static_cast<double>(l);
    }
    s_red[threadIdx.x] = tot;
    __syncthreads();
    for (int s = 512; s > 0; s >>= 1) {
        if (threadIdx.x < s) s_red[threadIdx.x] += s_red[threadIdx.x + s];
        __syncthreads();
    }
    if (threadIdx.x == 0) *loss = static_cast<float>(s_red[0]);
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

template <int BM, int BN, int WGM, int WGN>
int run_error_tiles(adadim_ctx* ctx, const __half* A, const __half* Hs, int64_t out, int64_t in, float* part,
                    int* NB_out) {
    const int MB = static_cast<int>((out + BM - 1) / BM), NB = static_cast<int>((in + BN - 1) / BN);
    constexpr int smem = 2 * (BM + BN) * ROW_BYTES;
    static bool attr_set = false;
    if (!attr_set) {
        ADADIM_HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(error_tiles<BM, BN, WGM, WGN>),
                                                hipFuncAttributeMaxDynamicSharedMemorySize, smem));
        attr_set = true;
    }
    {
        ProfScope prof(ctx, "error_tiles");
        hipLaunchKernelGGL((error_tiles<BM, BN, WGM, WGN>), dim3(static_cast<unsigned>(int64_t(MB) * NB)),
                           dim3(THREADS), smem, ctx->stream, A, Hs, out, in, MB, NB, part);
    }
    ADADIM_LAUNCH_CHECK(ctx, "error_tiles");
    *NB_out = NB;
    return ADADIM_OK;
}

}  // namespace

int launch_layer_error(adadim_ctx* ctx, const void* dW, int dW_dtype, int64_t out, int64_t in, const __half* Hs,
                       const float* hmeta, float* loss_rows, float* loss) {
    constexpr int BN = 256;
    const int NB = static_cast<int>((in + BN - 1) / BN);
    // scratch: [NB+1, out] floats: row partials per column block, then the diagonal term
    float* part = static_cast<float*>(adadim_workspace(ctx, WS_ERR_PART, size_t(NB + 1) * size_t(out) * sizeof(float)));
    if (!part) return ADADIM_EHIP;
    float* diag = part + size_t(NB) * size_t(out);
    const __half* A = static_cast<const __half*>(dW);
    __half* dW16 = nullptr;
    if (dW_dtype != ADADIM_DW_F16_SCALED) {
        dW16 = static_cast<__half*>(adadim_workspace(ctx, WS_DW16, size_t(out) * size_t(in) * sizeof(__half)));
        if (!dW16) return ADADIM_EHIP;
        A = dW16;
    }
    {
        ProfScope prof(ctx, "error_prologue");
        hipLaunchKernelGGL(error_prologue, dim3(static_cast<unsigned>(out)), dim3(256), 0, ctx->stream, dW, dW_dtype,
                           in, hmeta, dW16, diag);
    }
    ADADIM_LAUNCH_CHECK(ctx, "error_prologue");
    int nb_used = 0;
    int rc;
    if (out <= 2048 || (out / 256) * NB < 512)
        rc = run_error_tiles<128, BN, 1, 4>(ctx, A, Hs, out, in, part, &nb_used);
    else
        rc = run_error_tiles<256, BN, 2, 2>(ctx, A, Hs, out, in, part, &nb_used);
    if (rc != ADADIM_OK) return rc;
    {
        ProfScope prof(ctx, "error_finish");
        hipLaunchKernelGGL(error_finish, dim3(1), dim3(1024), 0, ctx->stream, diag, part, out, nb_used, loss_rows, loss);
    }
    ADADIM_LAUNCH_CHECK(ctx, "error_finish");
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
