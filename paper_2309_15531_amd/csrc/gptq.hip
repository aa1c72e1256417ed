// GPTQ in the dimension AdaDim selected (paper Sec. 3.3 "Augmenting RTN and GPTQ", App. A.1,
// App. B `gptq_ada`; GPTQ itself is Frantar et al. 2022).  Two calls:
//
//   adadim_gptq_prepare : dead channels, damping, activation order, and the factor U of the
//                         inverse Hessian (inv(H) = U^T U, U upper triangular, visiting order);
//   adadim_gptq_quantize: the channel-by-channel sweep with error feedback.
//
// Factor.  With J the index reversal, A = J H J, A = L L^T (lower Cholesky), H = V V^T for the
// upper triangular V = J L J, hence U = inv(V) = J inv(L) J: one Cholesky and one triangular
// inverse instead of Cholesky / inverse / Cholesky.  Both run in fp64: on this chip an fp64 fma
// costs what an unpacked fp32 fma costs, and the sweep's rounding decisions then see the same
// U (rounded once to fp32) as an fp64 reference.  Blocked right-looking Cholesky (64-wide
// panels: diagonal block in LDS, row-parallel triangular solve, tiled trailing update) and a
// block-row triangular inverse.
//
// Sweep.  Rows (per-OC) or row groups (per-IC) are independent, so a workgroup keeps its rows'
// 128-channel block in LDS and walks the channels alone: quantize channel i, e = (w - q)/U_ii,
// w_j -= e*U_ij for the rest of the block; a second kernel applies the block's errors to the
// channels behind the block, one channel's error at a time.  Every update is a rounded product
// followed by a rounded difference (no fma), in channel order, which fixes the result bit for
// bit.  Per-OC uses static groups (parameters computed beforehand from the original weight and
// looked up by the channel's original index); per-IC recomputes each (row group, channel)'s
// parameters from the channel's current values when it is visited.
#include "common.h"

namespace {

constexpr int NB = 64;        // panel width of the factorization
constexpr int GB = 128;       // channels per sweep block

// ------------------------------------------------------------------ prepare: order and matrix
__global__ void gq_diag(const float* __restrict__ H, int64_t n, double* __restrict__ d, uint8_t* __restrict__ dead) {
    const int64_t j = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (j >= n) return;
    const float h = H[j * n + j];
    const bool dd = h == 0.0f;
    dead[j] = dd ? 1 : 0;
    d[j] = dd ? 1.0 : static_cast<double>(h);
}

// damp = percdamp * mean(d), summed in index order by one thread block (fixed tree)
__global__ __launch_bounds__(256) void gq_damp(const double* __restrict__ d, int64_t n, double percdamp,
                                               double* __restrict__ damp) {
    __shared__ double s[256];
    double acc = 0.0;
    for (int64_t j = threadIdx.x; j < n; j += 256) acc += d[j];
    s[threadIdx.x] = acc;
    __syncthreads();
    for (int k = 128; k > 0; k >>= 1) {
        if (threadIdx.x < k) s[threadIdx.x] += s[threadIdx.x + k];
        __syncthreads();
    }
    if (threadIdx.x == 0) *damp = percdamp * (s[0] / static_cast<double>(n));
}

// perm[rank] = j with rank = number of channels that come before j: larger diagonal first,
// equal diagonals by index (a stable descending sort); identity without act_order
__global__ void gq_rank(const double* __restrict__ d, int64_t n, int act_order, int32_t* __restrict__ perm) {
    const int64_t j = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (j >= n) return;
    if (!act_order) {
        perm[j] = static_cast<int32_t>(j);
        return;
    }
    const double dj = d[j];
    int64_t rank = 0;
    for (int64_t k = 0; k < n; ++k) {
        const double dk = d[k];
        rank += (dk > dj || (dk == dj && k < j)) ? 1 : 0;
    }
    perm[rank] = static_cast<int32_t>(j);
}

// A = J (P (H' + damp I) P^T) J in fp64: A[a][b] = H'[perm[n-1-a]][perm[n-1-b]] (+ damp on the diagonal),
// H' = H with dead channels' diagonal set to 1
__global__ void gq_gather(const float* __restrict__ H, int64_t n, const int32_t* __restrict__ perm,
                          const double* __restrict__ d, const double* __restrict__ damp, double* __restrict__ A) {
    const int64_t idx = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (idx >= n * n) return;
    const int64_t a = idx / n, b = idx % n;
    const int64_t pa = perm[n - 1 - a], pb = perm[n - 1 - b];
    double v = static_cast<double>(H[pa * n + pb]);
    if (a == b) v = d[pa] + *damp;
    A[idx] = v;
}

// ------------------------------------------------------------------ Cholesky, lower, in place
// diagonal block A[k0.., k0..] of width w <= NB
__global__ __launch_bounds__(256) void chol_diag(double* __restrict__ A, int64_t n, int64_t k0, int w) {
    __shared__ double t[NB][NB + 1];
    const int tid = threadIdx.x;
    for (int e = tid; e < w * w; e += 256) t[e / w][e % w] = A[(k0 + e / w) * n + k0 + e % w];
    __syncthreads();
    for (int c = 0; c < w; ++c) {
        if (tid == 0) t[c][c] = sqrt(t[c][c]);
        __syncthreads();
        for (int r = c + 1 + tid; r < w; r += 256) t[r][c] /= t[c][c];
        __syncthreads();
        const int m = w - c - 1;                              // trailing rows/columns c+1..w-1, lower part
        for (int e = tid; e < m * m; e += 256) {
            const int r = c + 1 + e / m, cc = c + 1 + e % m;
            if (cc <= r) t[r][cc] -= t[r][c] * t[cc][c];
        }
        __syncthreads();
    }
    for (int e = tid; e < w * w; e += 256) {
        const int r = e / w, c = e % w;
        A[(k0 + r) * n + k0 + c] = c <= r ? t[r][c] : 0.0;
    }
}

// rows below the diagonal block: X L_kk^T = A[r, k0..k0+w), one thread per row
__global__ __launch_bounds__(64) void chol_trsm(double* __restrict__ A, int64_t n, int64_t k0, int w) {
    __shared__ double L[NB][NB + 1];
    for (int e = threadIdx.x; e < w * w; e += 64) L[e / w][e % w] = A[(k0 + e / w) * n + k0 + e % w];
    __syncthreads();
    const int64_t r = k0 + w + int64_t(blockIdx.x) * 64 + threadIdx.x;
    if (r >= n) return;
    double x[NB];
#pragma unroll
    for (int c = 0; c < NB; ++c) x[c] = c < w ? A[r * n + k0 + c] : 0.0;
#pragma unroll
    for (int c = 0; c < NB; ++c) {
        if (c < w) {
            double v = x[c];
#pragma unroll
            for (int t2 = 0; t2 < c; ++t2) v = fma(-x[t2], L[c][t2], v);
            x[c] = v / L[c][c];
        }
    }
#pragma unroll
    for (int c = 0; c < NB; ++c)
        if (c < w) A[r * n + k0 + c] = x[c];
}

// trailing update: C[r][c] -= sum_t P[r][t] P[c][t] for the 64 x 64 tile (tr, tc), tc <= tr, of the
// rows/columns from k1 on; P = A[.., k0..k0+w)
__global__ __launch_bounds__(256) void chol_syrk(double* __restrict__ A, int64_t n, int64_t k0, int w, int64_t k1) {
    __shared__ double Pr[NB][NB + 1], Pc[NB][NB + 1];
    // blockIdx.x enumerates the lower-triangular tile pairs
    int tr = 0, rem = blockIdx.x;
    while (rem > tr) {
        rem -= tr + 1;
        ++tr;
    }
    const int tc = rem;
    const int64_t r0 = k1 + int64_t(tr) * NB, c0 = k1 + int64_t(tc) * NB;
    for (int e = threadIdx.x; e < NB * NB; e += 256) {
        const int i = e / NB, t2 = e % NB;
        Pr[i][t2] = (r0 + i < n && t2 < w) ? A[(r0 + i) * n + k0 + t2] : 0.0;
        Pc[i][t2] = (c0 + i < n && t2 < w) ? A[(c0 + i) * n + k0 + t2] : 0.0;
    }
    __syncthreads();
    const int ty = threadIdx.x / 16, tx = threadIdx.x % 16;   // 4 x 4 outputs each: rows 4ty.., cols 4tx..
    double acc[4][4] = {};
    for (int t2 = 0; t2 < NB; ++t2) {
        double a[4], b[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            a[i] = Pr[4 * ty + i][t2];
            b[i] = Pc[4 * tx + i][t2];
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[i][j] = fma(a[i], b[j], acc[i][j]);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int64_t r = r0 + 4 * ty + i, c = c0 + 4 * tx + j;
            if (r < n && c <= r) A[r * n + c] -= acc[i][j];
        }
}

// ------------------------------------------------------------------ M = inv(L), lower, block rows
// diagonal block: column c of inv(L_ii) by forward substitution, one thread per column
__global__ __launch_bounds__(64) void trinv_diag(const double* __restrict__ A, double* __restrict__ M, int64_t n,
                                                 int64_t k0, int w) {
    __shared__ double L[NB][NB + 1];
    for (int e = threadIdx.x; e < w * w; e += 64) L[e / w][e % w] = A[(k0 + e / w) * n + k0 + e % w];
    __syncthreads();
    const int c = threadIdx.x;
    if (c >= w) return;
    double x[NB];
#pragma unroll
    for (int r = 0; r < NB; ++r) {
        x[r] = 0.0;
        if (r < w && r >= c) {
            double v = r == c ? 1.0 : 0.0;
#pragma unroll
            for (int t2 = 0; t2 < r; ++t2) v = fma(-L[r][t2], x[t2], v);
            x[r] = v / L[r][r];
        }
    }
#pragma unroll
    for (int r = 0; r < NB; ++r)
        if (r < w) M[(k0 + r) * n + k0 + c] = r >= c ? x[r] : 0.0;
}

// block row i0 (rows k0..k0+w): M[i][j] = -M_ii * sum_{t=j}^{i-1} L[i][t] M[t][j] for the block column
// blockIdx.x = j (64 columns from 64j); tiles through LDS
__global__ __launch_bounds__(256) void trinv_row(const double* __restrict__ A, double* __restrict__ M, int64_t n,
                                                 int64_t k0, int w) {
    __shared__ double Ta[NB][NB + 1], Tb[NB][NB + 1];
    const int64_t c0 = int64_t(blockIdx.x) * NB;              // block column (c0 < k0)
    const int ty = threadIdx.x / 16, tx = threadIdx.x % 16;
    double acc[4][4] = {};
    for (int64_t t0 = c0; t0 < k0; t0 += NB) {                // t blocks j .. i-1 (all full: they lie above row k0)
        __syncthreads();
        for (int e = threadIdx.x; e < NB * NB; e += 256) {
            const int i = e / NB, t2 = e % NB;
            Ta[i][t2] = i < w ? A[(k0 + i) * n + t0 + t2] : 0.0;        // L[i][t]
            Tb[i][t2] = M[(t0 + i) * n + c0 + t2];                      // M[t][j] (zero above its diagonal)
        }
        __syncthreads();
        for (int t2 = 0; t2 < NB; ++t2) {
            double a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                a[i] = Ta[4 * ty + i][t2];
                b[i] = Tb[t2][4 * tx + i];
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fma(a[i], b[j], acc[i][j]);
        }
    }
    // S (w x 64) into Tb, M_ii into Ta, then M_ij = -M_ii S
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) Tb[4 * ty + i][4 * tx + j] = acc[i][j];
    for (int e = threadIdx.x; e < NB * NB; e += 256) {
        const int i = e / NB, t2 = e % NB;
        Ta[i][t2] = (i < w && t2 < w) ? M[(k0 + i) * n + k0 + t2] : 0.0;
    }
    __syncthreads();
    double o[4][4] = {};
    for (int t2 = 0; t2 < NB; ++t2) {
        double a[4], b[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            a[i] = Ta[4 * ty + i][t2];
            b[i] = Tb[t2][4 * tx + i];
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) o[i][j] = fma(a[i], b[j], o[i][j]);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (4 * ty + i < w) M[(k0 + 4 * ty + i) * n + c0 + 4 * tx + j] = -o[i][j];
}

// U[a][b] = fp32(M[n-1-a][n-1-b]): upper triangular, visiting order
__global__ void gq_flip(const double* __restrict__ M, int64_t n, float* __restrict__ U) {
    const int64_t idx = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (idx >= n * n) return;
    const int64_t a = idx / n, b = idx % n;
    U[idx] = b >= a ? static_cast<float>(M[(n - 1 - a) * n + (n - 1 - b)]) : 0.0f;
}

// ------------------------------------------------------------------ sweep
struct QP {
    float scale, zero;
};
// the quantizer's parameters from a group's min and max (clip = 1): same formulas as adadim_quantize
__device__ __forceinline__ QP params_of(float mn, float mx, float qmax) {
    mx = fmaxf(mx, 0.0f);
    mn = fminf(mn, 0.0f);
    const float range = mx - mn;
    float scale = range / qmax;
    if (range == 0.0f) scale = 1.0f;
    float z = rintf((-mn) / scale);
    z = fminf(fmaxf(z, 0.0f), qmax);
    return {scale, z};
}

// Wp[r][i] = W[r][perm[i]] as fp32, zero for dead channels
__global__ void gq_gather_w(const __half* __restrict__ W, int64_t out, int64_t in, const int32_t* __restrict__ perm,
                            const uint8_t* __restrict__ dead, float* __restrict__ Wp) {
    const int64_t idx = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (idx >= out * in) return;
    const int64_t r = idx / in, i = idx % in;
    const int32_t j = perm[i];
    Wp[idx] = dead[j] ? 0.0f : __half2float(W[r * in + j]);
}

// One 128-channel block [i1, i1 + nbw) for the rows of one wavefront (a workgroup is one wave, so
// nothing is shared and there is no barrier).  Lane l holds RPL rows: per-OC rows 64*block + l
// (RPL = 1), per-IC rows l + 64p of the block's row group (RPL = g/64), so that the group's minimum
// and maximum are a lane-local step plus one wave reduction.  A lane's rows live in its own strip of
// LDS; the channels are walked in sub-blocks of 16 held in registers: the sub-block's own updates
// stay in registers, then its 16 errors are applied to the rest of the block, one LDS read and one
// write per element for 16 updates, always in channel order.  The block of U is staged in LDS and
// read with wave-uniform addresses.  Codes go out in visiting order (16 bytes per row and sub-block).
template <bool IC, int RPL>
__global__ __launch_bounds__(64) void gq_sweep(float* __restrict__ Wp, const float* __restrict__ U,
                                               const int32_t* __restrict__ perm, int64_t out, int64_t in, int64_t i1,
                                               int nbw, int g, float qmax, const float* __restrict__ st_scales,
                                               const uint8_t* __restrict__ st_zeros, float* __restrict__ scales_out,
                                               uint8_t* __restrict__ zeros_out, uint8_t* __restrict__ Qp,
                                               float* __restrict__ Ep) {
    constexpr int SB = 16, PITCH = GB + 1;
    extern __shared__ __align__(16) char smem[];
    float* Us = reinterpret_cast<float*>(smem);                         // [GB][GB]: rows / columns i1.. of U
    float* Ws = Us + GB * GB;                                           // [64 * RPL][PITCH]
    const int lane = threadIdx.x;
    for (int e4 = lane; e4 < nbw * (GB / 4); e4 += 64) {                // in % 4 == 0 is not required: guarded
        const int k = e4 / (GB / 4), c4 = (e4 % (GB / 4)) * 4;
        float4 v = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        const float* src = U + (i1 + k) * in + i1 + c4;
        if (c4 + 3 < nbw && ((reinterpret_cast<uintptr_t>(src) & 15u) == 0)) {
            v = *reinterpret_cast<const float4*>(src);
        } else {
            if (c4 + 0 < nbw) v.x = src[0];
            if (c4 + 1 < nbw) v.y = src[1];
            if (c4 + 2 < nbw) v.z = src[2];
            if (c4 + 3 < nbw) v.w = src[3];
        }
        *reinterpret_cast<float4*>(Us + k * GB + c4) = v;
    }
    __syncthreads();
    int64_t row[RPL];
    bool ok[RPL];
#pragma unroll
    for (int p = 0; p < RPL; ++p) {
        row[p] = IC ? int64_t(blockIdx.x) * g + lane + 64 * p : int64_t(blockIdx.x) * 64 + lane;
        ok[p] = row[p] < out;
        if (ok[p])
            for (int c = 0; c < nbw; ++c) Ws[(lane * RPL + p) * PITCH + c] = Wp[row[p] * in + i1 + c];
    }
    const int n_cg = IC ? 0 : static_cast<int>(in / g);
    for (int s0 = 0; s0 < nbw; s0 += SB) {
        const int sbw = nbw - s0 < SB ? nbw - s0 : SB;
        float w[RPL][SB], e[RPL][SB];
        uint32_t qpk[RPL][SB / 4];
#pragma unroll
        for (int p = 0; p < RPL; ++p) {
#pragma unroll
            for (int c = 0; c < SB; ++c) w[p][c] = (ok[p] && c < sbw) ? Ws[(lane * RPL + p) * PITCH + s0 + c] : 0.0f;
#pragma unroll
            for (int c = 0; c < SB / 4; ++c) qpk[p][c] = 0u;
        }
#pragma unroll
        for (int c = 0; c < SB; ++c) {
            if (c < sbw) {                                              // uniform
                const int64_t ig = i1 + s0 + c;                        // visiting index
                const int32_t j = perm[ig];                            // original channel (uniform)
                const float d = Us[(s0 + c) * GB + s0 + c];
                QP pr[RPL];
                if constexpr (IC) {
                    float mn = w[0][c], mx = w[0][c];
#pragma unroll
                    for (int p = 1; p < RPL; ++p) {
                        mn = fminf(mn, w[p][c]);
                        mx = fmaxf(mx, w[p][c]);
                    }
#pragma unroll
                    for (int m = 1; m < 64; m <<= 1) {
                        mn = fminf(mn, __shfl_xor(mn, m, 64));
                        mx = fmaxf(mx, __shfl_xor(mx, m, 64));
                    }
                    const QP q1 = params_of(mn, mx, qmax);
#pragma unroll
                    for (int p = 0; p < RPL; ++p) pr[p] = q1;
                    if (lane == 0) {
                        scales_out[int64_t(blockIdx.x) * in + j] = q1.scale;
                        zeros_out[int64_t(blockIdx.x) * in + j] = static_cast<uint8_t>(q1.zero);
                    }
                } else {
                    pr[0].scale = ok[0] ? st_scales[row[0] * n_cg + j / g] : 1.0f;
                    pr[0].zero = ok[0] ? static_cast<float>(st_zeros[row[0] * n_cg + j / g]) : 0.0f;
                }
#pragma unroll
                for (int p = 0; p < RPL; ++p) {
                    float q = rintf(w[p][c] / pr[p].scale) + pr[p].zero;
                    q = fminf(fmaxf(q, 0.0f), qmax);
                    const float wq = pr[p].scale * (q - pr[p].zero);
                    qpk[p][c / 4] |= static_cast<uint32_t>(q) << (8 * (c % 4));
                    e[p][c] = (w[p][c] - wq) / d;
#pragma unroll
                    for (int cc = c + 1; cc < SB; ++cc) {
                        if (cc < sbw) {
                            const float upd = e[p][c] * Us[(s0 + c) * GB + s0 + cc];
                            w[p][cc] = w[p][cc] - upd;
                        }
                    }
                }
            } else {
#pragma unroll
                for (int p = 0; p < RPL; ++p) e[p][c] = 0.0f;
            }
        }
        // the sub-block's codes and errors, in visiting order
#pragma unroll
        for (int p = 0; p < RPL; ++p) {
            if (!ok[p]) continue;
            const int64_t at = row[p] * in + i1 + s0;
            if (sbw == SB && ((at & 15) == 0)) {
                *reinterpret_cast<uint4*>(Qp + at) = make_uint4(qpk[p][0], qpk[p][1], qpk[p][2], qpk[p][3]);
            } else {
                for (int c = 0; c < sbw; ++c) Qp[at + c] = static_cast<uint8_t>(qpk[p][c / 4] >> (8 * (c % 4)));
            }
            for (int c = 0; c < sbw; ++c) Ep[at + c] = e[p][c];
        }
        // its errors applied to the rest of the block, channel order kept per element
        for (int cc = s0 + SB; cc < nbw; ++cc) {
            float u[SB];
#pragma unroll
            for (int k = 0; k < SB; ++k) u[k] = k < sbw ? Us[(s0 + k) * GB + cc] : 0.0f;
#pragma unroll
            for (int p = 0; p < RPL; ++p) {
                if (!ok[p]) continue;
                float v = Ws[(lane * RPL + p) * PITCH + cc];
#pragma unroll
                for (int k = 0; k < SB; ++k) {
                    const float upd = e[p][k] * u[k];
                    v = v - upd;
                }
                Ws[(lane * RPL + p) * PITCH + cc] = v;
            }
        }
    }
}

// codes back to the original channel order, and dW = W - scale*(code - zero) there
template <bool IC>
__global__ void gq_scatter(const uint8_t* __restrict__ Qp, const int32_t* __restrict__ perm,
                           const uint8_t* __restrict__ dead, const __half* __restrict__ W, int64_t out, int64_t in, int g,
                           const float* __restrict__ scales, const uint8_t* __restrict__ zeros,
                           uint8_t* __restrict__ codes, float* __restrict__ dW) {
    const int64_t idx = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (idx >= out * in) return;
    const int64_t r = idx / in, i = idx % in;
    const int32_t j = perm[i];
    const uint8_t q = Qp[idx];
    codes[r * in + j] = q;
    if (dW) {
        const int64_t pi = IC ? (r / g) * in + j : r * (in / g) + j / g;
        const float wq = scales[pi] * (static_cast<float>(q) - static_cast<float>(zeros[pi]));
        dW[r * in + j] = (dead[j] ? 0.0f : __half2float(W[r * in + j])) - wq;
    }
}

// channels behind the block: Wp[r][jj] -= E[r][k] * U[k][jj], k = i1 .. i2-1 in order (product, then difference)
__global__ __launch_bounds__(256) void gq_trailing(float* __restrict__ Wp, const float* __restrict__ U,
                                                   const float* __restrict__ Ep, int64_t out, int64_t in, int64_t i1,
                                                   int nbw) {
    __shared__ float Es[8][GB];
    const int64_t jj = i1 + nbw + int64_t(blockIdx.x) * 256 + threadIdx.x;
    const int64_t r0 = int64_t(blockIdx.y) * 8;
    for (int e = threadIdx.x; e < 8 * nbw; e += 256) {
        const int rr = e / nbw, k = e % nbw;
        Es[rr][k] = r0 + rr < out ? Ep[(r0 + rr) * in + i1 + k] : 0.0f;
    }
    __syncthreads();
    if (jj >= in) return;
    float v[8];
#pragma unroll
    for (int rr = 0; rr < 8; ++rr) v[rr] = r0 + rr < out ? Wp[(r0 + rr) * in + jj] : 0.0f;
    for (int k = 0; k < nbw; ++k) {
        const float u = U[(i1 + k) * in + jj];
#pragma unroll
        for (int rr = 0; rr < 8; ++rr) {
            const float upd = Es[rr][k] * u;
            v[rr] = v[rr] - upd;
        }
    }
#pragma unroll
    for (int rr = 0; rr < 8; ++rr)
        if (r0 + rr < out) Wp[(r0 + rr) * in + jj] = v[rr];
}

}  // namespace

int launch_gptq_prepare(adadim_ctx* ctx, const float* H, int64_t n, float percdamp, int act_order, int32_t* perm,
                        uint8_t* dead, float* U) {
    const size_t mat = size_t(n) * size_t(n) * sizeof(double);
    double* A = static_cast<double*>(adadim_workspace(ctx, WS_GPTQ_A, mat));
    double* M = static_cast<double*>(adadim_workspace(ctx, WS_GPTQ_M, mat));
    double* dvec = static_cast<double*>(adadim_workspace(ctx, WS_GPTQ_D, size_t(n + 1) * sizeof(double)));
    if (!A || !M || !dvec) return ADADIM_EHIP;
    double* damp = dvec + n;
    const unsigned nb1 = static_cast<unsigned>((n + 255) / 256), nb2 = static_cast<unsigned>((n * n + 255) / 256);
    ProfScope prof(ctx, "gptq_prepare");
    hipLaunchKernelGGL(gq_diag, dim3(nb1), dim3(256), 0, ctx->stream, H, n, dvec, dead);
    hipLaunchKernelGGL(gq_damp, dim3(1), dim3(256), 0, ctx->stream, dvec, n, static_cast<double>(percdamp), damp);
    hipLaunchKernelGGL(gq_rank, dim3(nb1), dim3(256), 0, ctx->stream, dvec, n, act_order, perm);
    hipLaunchKernelGGL(gq_gather, dim3(nb2), dim3(256), 0, ctx->stream, H, n, perm, dvec, damp, A);
    ADADIM_LAUNCH_CHECK(ctx, "gptq prepare");
    for (int64_t k0 = 0; k0 < n; k0 += NB) {
        const int w = static_cast<int>(n - k0 < NB ? n - k0 : NB);
        hipLaunchKernelGGL(chol_diag, dim3(1), dim3(256), 0, ctx->stream, A, n, k0, w);
        const int64_t rest = n - k0 - w;
        if (rest > 0) {
            hipLaunchKernelGGL(chol_trsm, dim3(static_cast<unsigned>((rest + 63) / 64)), dim3(64), 0, ctx->stream, A, n, k0, w);
            const int64_t t = (rest + NB - 1) / NB;
            hipLaunchKernelGGL(chol_syrk, dim3(static_cast<unsigned>(t * (t + 1) / 2)), dim3(256), 0, ctx->stream, A, n, k0,
                               w, k0 + w);
        }
    }
    ADADIM_LAUNCH_CHECK(ctx, "gptq cholesky");
    for (int64_t k0 = 0; k0 < n; k0 += NB) {
        const int w = static_cast<int>(n - k0 < NB ? n - k0 : NB);
        hipLaunchKernelGGL(trinv_diag, dim3(1), dim3(64), 0, ctx->stream, A, M, n, k0, w);
        if (k0 > 0)
            hipLaunchKernelGGL(trinv_row, dim3(static_cast<unsigned>(k0 / NB)), dim3(256), 0, ctx->stream, A, M, n, k0, w);
    }
    hipLaunchKernelGGL(gq_flip, dim3(nb2), dim3(256), 0, ctx->stream, M, n, U);
    ADADIM_LAUNCH_CHECK(ctx, "gptq inverse");
    return ADADIM_OK;
}

int launch_gptq_quantize(adadim_ctx* ctx, const __half* W, int64_t out, int64_t in, int dim, int bits, int g,
                         const float* U, const int32_t* perm, const uint8_t* dead, const float* st_scales,
                         const uint8_t* st_zeros, uint8_t* codes, float* scales_out, uint8_t* zeros_out, float* dW) {
    const size_t mat = size_t(out) * size_t(in) * sizeof(float);
    float* Wp = static_cast<float*>(adadim_workspace(ctx, WS_GPTQ_W, mat));
    float* Ep = static_cast<float*>(adadim_workspace(ctx, WS_GPTQ_E, mat));
    uint8_t* Qp = static_cast<uint8_t*>(adadim_workspace(ctx, WS_GPTQ_Q, size_t(out) * size_t(in)));
    if (!Wp || !Ep || !Qp) return ADADIM_EHIP;
    const float qmax = static_cast<float>((1 << bits) - 1);
    const bool ic = dim == ADADIM_DIM_IC;
    const int rpl = ic ? g / 64 : 1;                                   // rows per lane
    const unsigned blocks = static_cast<unsigned>(ic ? out / g : (out + 63) / 64);
    const size_t smem = (size_t(GB) * GB + size_t(64) * rpl * (GB + 1)) * sizeof(float);
    static bool attr_set = false;
    if (!attr_set) {
        ADADIM_HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(gq_sweep<true, 2>),
                                                hipFuncAttributeMaxDynamicSharedMemorySize, 144 * 1024));
        ADADIM_HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(gq_sweep<true, 1>),
                                                hipFuncAttributeMaxDynamicSharedMemorySize, 144 * 1024));
        ADADIM_HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(gq_sweep<false, 1>),
                                                hipFuncAttributeMaxDynamicSharedMemorySize, 144 * 1024));
        attr_set = true;
    }
    const unsigned eb = static_cast<unsigned>((out * in + 255) / 256);
    {
        ProfScope prof(ctx, "gptq_gather");
        hipLaunchKernelGGL(gq_gather_w, dim3(eb), dim3(256), 0, ctx->stream, W, out, in, perm, dead, Wp);
    }
    for (int64_t i1 = 0; i1 < in; i1 += GB) {
        const int nbw = static_cast<int>(in - i1 < GB ? in - i1 : GB);
        {
            ProfScope prof(ctx, "gptq_sweep");
#define GQ_GO(IC_, RPL_)                                                                                          \
    hipLaunchKernelGGL((gq_sweep<IC_, RPL_>), dim3(blocks), dim3(64), smem, ctx->stream, Wp, U, perm, out, in, i1, \
                       nbw, g, qmax, st_scales, st_zeros, scales_out, zeros_out, Qp, Ep)
            if (!ic) GQ_GO(false, 1);
            else if (rpl == 1) GQ_GO(true, 1);
            else GQ_GO(true, 2);
#undef GQ_GO
        }
        const int64_t rest = in - i1 - nbw;
        if (rest > 0) {
            ProfScope prof(ctx, "gptq_trailing");
            dim3 grid(static_cast<unsigned>((rest + 255) / 256), static_cast<unsigned>((out + 7) / 8));
            hipLaunchKernelGGL(gq_trailing, grid, dim3(256), 0, ctx->stream, Wp, U, Ep, out, in, i1, nbw);
        }
    }
    {
        ProfScope prof(ctx, "gptq_scatter");
        if (ic)
            hipLaunchKernelGGL(gq_scatter<true>, dim3(eb), dim3(256), 0, ctx->stream, Qp, perm, dead, W, out, in, g,
                               scales_out, zeros_out, codes, dW);
        else
            hipLaunchKernelGGL(gq_scatter<false>, dim3(eb), dim3(256), 0, ctx->stream, Qp, perm, dead, W, out, in, g,
                               st_scales, st_zeros, codes, dW);
    }
    ADADIM_LAUNCH_CHECK(ctx, "gptq sweep");
    return ADADIM_OK;
}
