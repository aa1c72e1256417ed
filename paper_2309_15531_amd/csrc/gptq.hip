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
#include "scale_format.h"

#include <algorithm>
#include <type_traits>

namespace {

constexpr int NB = 64;        // panel width of the factorization
constexpr int NBO = 512;      // its outer panel: trailing updates are applied 512 columns at a time
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

// The same ranks in two steps that use the whole chip: block (x, y) counts, for its 256 channels j,
// the channels of the y-th kilo-entry of the diagonal that come before j (staged in LDS) and adds the
// count to rank[j] (integer atomics: any order gives the same sum); then perm[rank[j]] = j.
__global__ void gq_zero_i32(int32_t* __restrict__ p, int64_t n) {
    const int64_t i = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}
__global__ __launch_bounds__(256) void gq_rank_count(const double* __restrict__ d, int64_t n, int32_t* __restrict__ rank) {
    __shared__ double s[1024];
    const int64_t j = int64_t(blockIdx.x) * 256 + threadIdx.x, k0 = int64_t(blockIdx.y) * 1024;
    for (int e = threadIdx.x; e < 1024; e += 256) s[e] = k0 + e < n ? d[k0 + e] : -1.0;   // diagonal entries are > 0
    __syncthreads();
    if (j >= n) return;
    const double dj = d[j];
    const int m = static_cast<int>(n - k0 < 1024 ? n - k0 : 1024);
    int c0 = 0, c1 = 0, c2 = 0, c3 = 0;                       // four counters: the adds do not wait for each other
    int e = 0;
    for (; e + 4 <= m; e += 4) {
        c0 += (s[e] > dj || (s[e] == dj && k0 + e < j)) ? 1 : 0;
        c1 += (s[e + 1] > dj || (s[e + 1] == dj && k0 + e + 1 < j)) ? 1 : 0;
        c2 += (s[e + 2] > dj || (s[e + 2] == dj && k0 + e + 2 < j)) ? 1 : 0;
        c3 += (s[e + 3] > dj || (s[e + 3] == dj && k0 + e + 3 < j)) ? 1 : 0;
    }
    for (; e < m; ++e) c0 += (s[e] > dj || (s[e] == dj && k0 + e < j)) ? 1 : 0;
    atomicAdd(rank + j, (c0 + c1) + (c2 + c3));
}
__global__ void gq_rank_place(const int32_t* __restrict__ rank, int64_t n, int32_t* __restrict__ perm) {
    const int64_t j = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (j < n) perm[rank[j]] = static_cast<int32_t>(j);
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

// ------------------------------------------------------------------ fp64 tiles on the matrix cores
// v_mfma_f64_16x16x4_f64: lane l supplies A[l % 16][l / 16] and B[l / 16][l % 16]; register r of its
// result is D[4 r + l / 16][l % 16].  The vector and the matrix pipe have the same fp64 peak on this
// chip; the matrix form needs a quarter of the LDS reads per flop and no issue slots for the products.
typedef double double4_t __attribute__((ext_vector_type(4)));
constexpr int GT = 64, GK = 32;                  // tile edge, contraction chunk
// (128 x 128 tiles were measured too: one workgroup per compute unit instead of four, and the
// products ran a third slower; the matrix pipe wants the other workgroups' waves to fill its gaps.)

// acc += A B (acc -= A B with NEG_A) for one TS x TS tile (TS = 64 or 128) and k in [k_lo, k_hi), 256 threads: 2 x 2 waves,
// each TS/2 x TS/2 = MT x MT matrix-core tiles of 16 x 16.
//   A(i, k) = Ap[i * lda + k], rows i < m_valid;
//   B(k, j) = B_KC ? Bp[j * ldb + k] : Bp[k * ldb + j], columns j < n_valid;
// everything outside the valid ranges reads as zero.  As, Bs: [GK][TS + 4] doubles each.
template <int TS, bool B_KC, bool NEG_A = false>
__device__ __forceinline__ void dgemm_tile(const double* __restrict__ Ap, int64_t lda, int m_valid,
                                           const double* __restrict__ Bp, int64_t ldb, int n_valid, int64_t k_lo,
                                           int64_t k_hi, double (*As)[TS + 4], double (*Bs)[TS + 4],
                                           double4_t (&acc)[TS / 32][TS / 32]) {
    constexpr int MT = TS / 32, E = TS / 16;              // matrix-core tiles per wave side; elements per thread and operand
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6, wm = wave >> 1, wn = wave & 1;
    // Loads: 16 consecutive lanes read 16 consecutive doubles (one 128-byte line).  For an operand
    // that is contiguous along k they are the chunk's 16 k of one row (rows t/16 + 16 e); for the
    // row-major B they are 16 columns of one k row (k row t/16, columns t%16 + 16 e).
    const int l16 = t & 15, h16 = t >> 4;
    constexpr int KK = GK / 16;                           // 16-wide pieces of a chunk
    double ra[KK][E], rb[KK][E];
    // the next chunk's operands travel from memory to registers while the matrix cores work on this one
    auto fetch = [&](int64_t k0) {
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
            const int64_t k = k0 + 16 * kk + l16;
#pragma unroll
            for (int e = 0; e < E; ++e) {
                const int row = h16 + 16 * e;
                ra[kk][e] = (row < m_valid && k < k_hi) ? Ap[row * lda + k] : 0.0;
            }
            if constexpr (B_KC) {
#pragma unroll
                for (int e = 0; e < E; ++e) {
                    const int row = h16 + 16 * e;
                    rb[kk][e] = (row < n_valid && k < k_hi) ? Bp[row * ldb + k] : 0.0;
                }
            } else {
                const int64_t kr = k0 + 16 * kk + h16;
#pragma unroll
                for (int e = 0; e < E; ++e) {
                    const int col = l16 + 16 * e;
                    rb[kk][e] = (kr < k_hi && col < n_valid) ? Bp[kr * ldb + col] : 0.0;
                }
            }
        }
    };
    if (k_lo < k_hi) fetch(k_lo);
    for (int64_t k0 = k_lo; k0 < k_hi; k0 += GK) {
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
#pragma unroll
            for (int e = 0; e < E; ++e) As[16 * kk + l16][h16 + 16 * e] = ra[kk][e];
            if constexpr (B_KC) {
#pragma unroll
                for (int e = 0; e < E; ++e) Bs[16 * kk + l16][h16 + 16 * e] = rb[kk][e];
            } else {
#pragma unroll
                for (int e = 0; e < E; ++e) Bs[16 * kk + h16][l16 + 16 * e] = rb[kk][e];
            }
        }
        __syncthreads();
        if (k0 + GK < k_hi) fetch(k0 + GK);
#pragma unroll
        for (int ks = 0; ks < GK; ks += 4) {
            double a[MT], b[MT];
#pragma unroll
            for (int u = 0; u < MT; ++u) {
                a[u] = As[ks + (lane >> 4)][wm * (TS / 2) + u * 16 + (lane & 15)];
                if constexpr (NEG_A) a[u] = -a[u];
                b[u] = Bs[ks + (lane >> 4)][wn * (TS / 2) + u * 16 + (lane & 15)];
            }
#pragma unroll
            for (int u = 0; u < MT; ++u)
#pragma unroll
                for (int v = 0; v < MT; ++v) acc[u][v] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[u], b[v], acc[u][v], 0, 0, 0);
        }
    }
}

// visits the tile's elements this lane holds: f(row in tile, column in tile, value)
template <int TS, typename F>
__device__ __forceinline__ void dgemm_each(const double4_t (&acc)[TS / 32][TS / 32], F f) {
    constexpr int MT = TS / 32;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, wm = wave >> 1, wn = wave & 1;
#pragma unroll
    for (int u = 0; u < MT; ++u)
#pragma unroll
        for (int v = 0; v < MT; ++v)
#pragma unroll
            for (int r = 0; r < 4; ++r)
                f(wm * (TS / 2) + u * 16 + 4 * r + (lane >> 4), wn * (TS / 2) + v * 16 + (lane & 15), acc[u][v][r]);
}

// fills the lane's elements of a tile: acc = f(row in tile, column in tile)
template <int TS, typename F>
__device__ __forceinline__ void dgemm_fill(double4_t (&acc)[TS / 32][TS / 32], F f) {
    constexpr int MT = TS / 32;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, wm = wave >> 1, wn = wave & 1;
#pragma unroll
    for (int u = 0; u < MT; ++u)
#pragma unroll
        for (int v = 0; v < MT; ++v)
#pragma unroll
            for (int r = 0; r < 4; ++r)
                acc[u][v][r] = f(wm * (TS / 2) + u * 16 + 4 * r + (lane >> 4), wn * (TS / 2) + v * 16 + (lane & 15));
}

// ------------------------------------------------------------------ Cholesky, lower, in place
// Diagonal block A[k0.., k0..] of width w <= NB = 64, factored and inverted by one workgroup of four
// waves, blocked by 16.  The whole factorization waits for this kernel, so what counts is the length
// of its dependency chain, not its flops:
//  * Cholesky, four panels of 16 columns.  Wave 0 holds the panel with lane r = row r (16 registers):
//    column c is final once its pivot is (broadcast by a lane read; reciprocal square root plus two
//    Newton steps), the later columns of the panel receive l_rc l_jc with l_jc read from lane j.  No
//    LDS and no barrier inside a panel, at most 15 updates per column.  The columns behind the panel
//    get the panel's rank-16 update from the fp64 matrix cores, the (at most six) 16 x 16 tiles dealt
//    to the four waves.
//  * inv(L) by doubling: the four 16 x 16 diagonal blocks at once, one per wave (lane j solves for
//    column j, L's entries by lane reads), then the level-16 and level-32 off-diagonal blocks as
//    -inv(B) C inv(A), two matrix-core products each.
// inv(L) goes to the diagonal block of M: it turns the panel's triangular solve into a product and is
// the first level of the triangular inverse.
// the value `v` has in lane `src_lane` (wave-uniform), in every lane
__device__ __forceinline__ double lane_read(double v, int src_lane) {
    const int lo = __builtin_amdgcn_readlane(__double2loint(v), src_lane);
    const int hi = __builtin_amdgcn_readlane(__double2hiint(v), src_lane);
    return __hiloint2double(hi, lo);
}
// LDS writes of this wave before, its LDS reads after: a wave's LDS accesses are served in order
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// LDS of the diagonal block's factorization: 41 KB.  inv(L) grows in the upper triangle of the block that holds L
// (transposed; its diagonal is rd), so that the workgroup fits beside three of the trailing update's workgroups on
// a compute unit: one that needed more than a freed slot's share of LDS would wait for that launch to drain.
struct DiagLds {
    static constexpr int LD = NB + 1;
    double t[NB][LD];                                         // the block, then L on and below the diagonal, inv(L)^T above
    double tt[NB / 2][NB / 2 + 1];                            // C inv(A) of the inverse's levels
    double rd[NB];                                            // reciprocals of the diagonal of L = diagonal of inv(L)
};
__device__ __forceinline__ void diag_factor(double* __restrict__ A, double* __restrict__ M, int64_t n, int64_t k0, int w,
                                            DiagLds& lds) {
    constexpr int P = 16;
    auto& t = lds.t;
    auto& tt = lds.tt;
    auto& rd = lds.rd;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, h16 = lane >> 4;
    // one workgroup that the whole factorization waits for: ahead of the trailing update that may share its SIMDs
    __builtin_amdgcn_s_setprio(3);
    for (int e = tid; e < NB * NB; e += 256) {
        const int r = e / NB, c = e % NB;
        t[r][c] = (r < w && c < w) ? A[(k0 + r) * n + k0 + c] : (r == c ? 1.0 : 0.0);   // identity padding
    }
    __syncthreads();
    // element (r, c) of inv(L) once its block is there
    auto mval = [&](int r, int c) {
        const double up = t[c < r ? c : r][c < r ? r : c], dg = lds.rd[r];
        return r > c ? up : (r == c ? dg : 0.0);
    };
    // the pivot's reciprocal square root: the same in every lane
    auto rsqrt_of = [](double piv) {
        double inv = __builtin_amdgcn_rsq(piv);
        inv = inv * fma(-0.5 * piv * inv, inv, 1.5);
        return inv * fma(-0.5 * piv * inv, inv, 1.5);
    };
    for (int p = 0; p < NB / P; ++p) {
        if (wave == 0) {
            double x[P];
#pragma unroll
            for (int j = 0; j < P; ++j) x[j] = t[lane][P * p + j];
#pragma unroll
            for (int c = 0; c < P; ++c) {
                const int gc = P * p + c;
                const double piv = lane_read(x[c], gc), inv = rsqrt_of(piv);
                const double l = lane == gc ? piv * inv : (lane > gc ? x[c] * inv : 0.0);
                x[c] = l;
                if (lane == gc) rd[gc] = inv;
#pragma unroll
                for (int j = c + 1; j < P; ++j) x[j] = fma(-l, lane_read(l, P * p + j), x[j]);
            }
#pragma unroll
            for (int j = 0; j < P; ++j) t[lane][P * p + j] = x[j];
        }
        __syncthreads();
        int idx = 0;
        for (int ti = p + 1; ti < NB / P; ++ti)
            for (int tj = p + 1; tj <= ti; ++tj, ++idx) {
                if ((idx & 3) != wave) continue;              // whole waves
                double4_t acc;
#pragma unroll
                for (int r = 0; r < 4; ++r) acc[r] = t[P * ti + 4 * r + h16][P * tj + l16];
#pragma unroll
                for (int kk = 0; kk < P; kk += 4)
                    acc = __builtin_amdgcn_mfma_f64_16x16x4f64(-t[P * ti + l16][P * p + kk + h16], t[P * tj + l16][P * p + kk + h16],
                                                               acc, 0, 0, 0);
#pragma unroll
                for (int r = 0; r < 4; ++r) t[P * ti + 4 * r + h16][P * tj + l16] = acc[r];
            }
        __syncthreads();
    }
    // diagonal blocks of inv(L): wave b's lanes 0..15 hold rows and solve for columns of block b (the other
    // lanes repeat them)
    {
        const int b = P * wave;
        double xr[P], a[P];
#pragma unroll
        for (int k = 0; k < P; ++k) {
            xr[k] = t[b + l16][b + k];
            a[k] = k == l16 ? 1.0 : 0.0;
        }
#pragma unroll
        for (int k = 0; k < P; ++k) {
            const double yk = a[k] * rd[b + k];
            a[k] = yk;
#pragma unroll
            for (int r = k + 1; r < P; ++r) a[r] = fma(-lane_read(xr[k], r), yk, a[r]);
        }
        if (lane < P) {
#pragma unroll
            for (int r = 0; r < P; ++r)
                if (r > lane) t[b + lane][b + r] = a[r];      // the diagonal entry is rd
        }
    }
    __syncthreads();
    // level 16: blocks (1, 0) and (3, 2), one wave each
    if (wave < 2) {
        const int ra = 2 * P * wave, rb = ra + P;            // first rows of inv(A)'s and inv(B)'s blocks
        double4_t acc = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
        for (int kk = 0; kk < P; kk += 4)
            acc = __builtin_amdgcn_mfma_f64_16x16x4f64(t[rb + l16][ra + kk + h16], mval(ra + kk + h16, ra + l16), acc, 0, 0, 0);
#pragma unroll
        for (int r = 0; r < 4; ++r) tt[P * wave + 4 * r + h16][l16] = acc[r];
        wave_lds_sync();
        acc = double4_t{0.0, 0.0, 0.0, 0.0};
#pragma unroll
        for (int kk = 0; kk < P; kk += 4)
            acc = __builtin_amdgcn_mfma_f64_16x16x4f64(-mval(rb + l16, rb + kk + h16), tt[P * wave + kk + h16][l16], acc, 0, 0, 0);
#pragma unroll
        for (int r = 0; r < 4; ++r) t[ra + l16][rb + 4 * r + h16] = acc[r];
    }
    __syncthreads();
    // level 32: the 32 x 32 block below the diagonal, one 16 x 16 tile per wave
    {
        const int ti = wave >> 1, tj = wave & 1;
        double4_t acc = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
        for (int kk = 0; kk < 2 * P; kk += 4)
            acc = __builtin_amdgcn_mfma_f64_16x16x4f64(t[2 * P + P * ti + l16][kk + h16], mval(kk + h16, P * tj + l16), acc, 0, 0, 0);
#pragma unroll
        for (int r = 0; r < 4; ++r) tt[P * ti + 4 * r + h16][P * tj + l16] = acc[r];
        __syncthreads();
        acc = double4_t{0.0, 0.0, 0.0, 0.0};
#pragma unroll
        for (int kk = 0; kk < 2 * P; kk += 4)
            acc = __builtin_amdgcn_mfma_f64_16x16x4f64(-mval(2 * P + P * ti + l16, 2 * P + kk + h16), tt[kk + h16][P * tj + l16], acc,
                                                       0, 0, 0);
#pragma unroll
        for (int r = 0; r < 4; ++r) t[P * tj + l16][2 * P + P * ti + 4 * r + h16] = acc[r];
    }
    __syncthreads();
    for (int e = tid; e < w * w; e += 256) {
        const int r = e / w, c = e % w;
        A[(k0 + r) * n + k0 + c] = r >= c ? t[r][c] : 0.0;
        M[(k0 + r) * n + k0 + c] = mval(r, c);
    }
}

__global__ __launch_bounds__(256) void chol_diag_inv(double* __restrict__ A, double* __restrict__ M, int64_t n, int64_t k0,
                                                     int w) {
    __shared__ DiagLds lds;
    diag_factor(A, M, n, k0, w, lds);
}

// rows below the diagonal block: L21 = A21 inv(L11)^T, 64 rows per block, in place (a block reads
// only the rows it writes, and has read them all before the first store)
__global__ __launch_bounds__(256) void chol_panel(double* __restrict__ A, const double* __restrict__ M, int64_t n,
                                                  int64_t k0, int w) {
    __shared__ double As[GK][GT + 4], Bs[GK][GT + 4];
    // a link of the chain the factorization waits for: its waves issue ahead of the bulk update's on a shared SIMD
    __builtin_amdgcn_s_setprio(3);
    const int64_t r0 = k0 + w + int64_t(blockIdx.x) * GT;
    const int m_valid = static_cast<int>(n - r0 < GT ? n - r0 : GT);
    double4_t acc[2][2] = {};
    dgemm_tile<GT, true>(A + r0 * n + k0, n, m_valid, M + k0 * n + k0, n, w, 0, w, As, Bs, acc);
    __syncthreads();
    dgemm_each<GT>(acc, [&](int i, int j, double v) {
        if (i < m_valid && j < w) A[(r0 + i) * n + k0 + j] = v;
    });
}

// trailing update: C[r][c] -= sum_t P[r][t] P[c][t] on the TS x TS tiles (blockIdx.y, blockIdx.x <= blockIdx.y)
// of the rows/columns from k1 on; P = A[.., k0..k0+w).  gridDim.x limits the columns that are updated
// (inside a 512-wide outer panel only the panel's own columns; behind it all, with w = 512).
// ct0: first tile column of this launch (the update behind an outer panel goes out in two launches).
template <int TS>
__global__ __launch_bounds__(256) void chol_syrk(double* __restrict__ A, int64_t n, int64_t k0, int w, int64_t k1, int ct0) {
    const int ct = static_cast<int>(blockIdx.x) + ct0;
    if (ct > static_cast<int>(blockIdx.y)) return;
    __shared__ double As[GK][TS + 4], Bs[GK][TS + 4];
    const int64_t r0 = k1 + int64_t(blockIdx.y) * TS, c0 = k1 + int64_t(ct) * TS;
    const int m_valid = static_cast<int>(n - r0 < TS ? n - r0 : TS), n_valid = static_cast<int>(n - c0 < TS ? n - c0 : TS);
    // the accumulators start as the tile of C (its loads travel with the first operand chunk's) and the products are
    // subtracted: no read-modify-write behind the loop
    double4_t acc[TS / 32][TS / 32];
    dgemm_fill<TS>(acc, [&](int i, int j) { return (i < m_valid && j < n_valid) ? A[(r0 + i) * n + c0 + j] : 0.0; });
    dgemm_tile<TS, true, true>(A + r0 * n + k0, n, m_valid, A + c0 * n + k0, n, n_valid, 0, w, As, Bs, acc);
    dgemm_each<TS>(acc, [&](int i, int j, double v) {
        if (i < m_valid && c0 + j <= r0 + i) A[(r0 + i) * n + c0 + j] = v;
    });
}

// The same update with 64 x 64 tiles, and the workgroup of the first tile (the diagonal block at k1, final once
// this update has reached it) goes on to factor and invert that block: the next step's chol_diag_inv without its
// launch, and under the other tiles' products.  The product's staging buffers and the factorization's LDS share
// their space.
__global__ __launch_bounds__(256) void chol_syrk_diag(double* __restrict__ A, double* __restrict__ M, int64_t n, int64_t k0, int w,
                                                      int64_t k1) {
    if (blockIdx.x > blockIdx.y) return;
    __builtin_amdgcn_s_setprio(3);                            // a link of the chain, as chol_panel
    __shared__ __align__(16) char smem[sizeof(DiagLds) > 2 * GK * (GT + 4) * sizeof(double) ? sizeof(DiagLds)
                                                                                             : 2 * GK * (GT + 4) * sizeof(double)];
    double(*As)[GT + 4] = reinterpret_cast<double(*)[GT + 4]>(smem);
    double(*Bs)[GT + 4] = As + GK;
    const int64_t r0 = k1 + int64_t(blockIdx.y) * GT, c0 = k1 + int64_t(blockIdx.x) * GT;
    const int m_valid = static_cast<int>(n - r0 < GT ? n - r0 : GT), n_valid = static_cast<int>(n - c0 < GT ? n - c0 : GT);
    double4_t acc[GT / 32][GT / 32];
    dgemm_fill<GT>(acc, [&](int i, int j) { return (i < m_valid && j < n_valid) ? A[(r0 + i) * n + c0 + j] : 0.0; });
    dgemm_tile<GT, true, true>(A + r0 * n + k0, n, m_valid, A + c0 * n + k0, n, n_valid, 0, w, As, Bs, acc);
    dgemm_each<GT>(acc, [&](int i, int j, double v) {
        if (i < m_valid && c0 + j <= r0 + i) A[(r0 + i) * n + c0 + j] = v;
    });
    if (blockIdx.x == 0 && blockIdx.y == 0) {                 // whole workgroup
        __syncthreads();                                      // the tile is in memory and the staging buffers are free
        diag_factor(A, M, n, k1, static_cast<int>(n - k1 < NB ? n - k1 : NB), *reinterpret_cast<DiagLds*>(smem));
    }
}

// ------------------------------------------------------------------ M = inv(L), lower, by doubling
// inv [[A, 0], [C, B]] = [[inv A, 0], [-inv(B) C inv(A), inv B]].  With the diagonal blocks of
// size s inverted, level s pairs them up: pair p = blockIdx.z covers rows a0 = 2 p s (A, s rows)
// and b0 = a0 + s (B, sb <= s rows at the matrix end).  Two products per level, every pair and
// every tile in parallel: T = C inv(A) (PASS 0, inv(A) lower triangular: k starts at the tile's
// first column), then M[B rows, A columns] = -inv(B) T (PASS 1, k ends with the tile's last row).
// TS x TS tiles, TS dividing s.
template <int PASS, int TS>
__global__ __launch_bounds__(256) void trinv_level(const double* __restrict__ L, double* __restrict__ M,
                                                   double* __restrict__ T, int64_t n, int64_t s) {
    const int64_t a0 = 2 * int64_t(blockIdx.z) * s, b0 = a0 + s;
    const int64_t sb = n - b0 < s ? n - b0 : s;               // > 0 for every pair in the grid
    const int64_t m0 = int64_t(blockIdx.y) * TS, n0 = int64_t(blockIdx.x) * TS;
    if (m0 >= sb) return;
    __shared__ double As[GK][TS + 4], Bs[GK][TS + 4];
    const int m_valid = static_cast<int>(sb - m0 < TS ? sb - m0 : TS);
    double* Tp = T + int64_t(blockIdx.z) * s * s;
    double4_t acc[TS / 32][TS / 32] = {};
    if constexpr (PASS == 0) {
        dgemm_tile<TS, false>(L + (b0 + m0) * n + a0, n, m_valid, M + a0 * n + a0 + n0, n, TS, n0, s, As, Bs, acc);
        dgemm_each<TS>(acc, [&](int i, int j, double v) {
            if (i < m_valid) Tp[(m0 + i) * s + n0 + j] = v;
        });
    } else {
        const int64_t k_hi = sb < m0 + TS ? sb : m0 + TS;
        dgemm_tile<TS, false>(M + (b0 + m0) * n + b0, n, m_valid, Tp + n0, s, TS, 0, k_hi, As, Bs, acc);
        dgemm_each<TS>(acc, [&](int i, int j, double v) {
            if (i < m_valid) M[(b0 + m0 + i) * n + a0 + n0 + j] = -v;
        });
    }
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
// (mfmt != 0: the scale rounded into the 16-bit group word first, as adadim_quantize_meta16 does)
__device__ __forceinline__ QP params_of(float mn, float mx, float qmax, int mfmt) {
    mx = fmaxf(mx, 0.0f);
    mn = fminf(mn, 0.0f);
    const float range = mx - mn;
    float scale = range / qmax;
    if (range == 0.0f) scale = 1.0f;
    if (mfmt) scale = round_scale(scale, mfmt);
    float z = rintf((-mn) / scale);
    z = fminf(fmaxf(z, 0.0f), qmax);
    return {scale, z};
}

// Minima of two values over the wavefront, the same in every lane (min is exact, any order gives the
// same bits).  Butterflies inside the rows of 16 lanes, then row 0 into 1 and 2 into 3, then lane 31
// into the upper half, all as v_min_f32 with a DPP operand; lane 63 holds the result.  The two chains
// are interleaved and padded so that two wait states separate a write from the DPP read of it.
// Needs every lane active.
__device__ __forceinline__ void wave_min2(float& a, float& b) {
    asm volatile(
        "s_nop 1\n\t"
        "v_min_f32_dpp %0, %0, %0 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
        "v_min_f32_dpp %1, %1, %1 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 0\n\t"
        "v_min_f32_dpp %0, %0, %0 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
        "v_min_f32_dpp %1, %1, %1 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 0\n\t"
        "v_min_f32_dpp %0, %0, %0 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
        "v_min_f32_dpp %1, %1, %1 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 0\n\t"
        "v_min_f32_dpp %0, %0, %0 row_mirror row_mask:0xf bank_mask:0xf\n\t"
        "v_min_f32_dpp %1, %1, %1 row_mirror row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 0\n\t"
        "v_min_f32_dpp %0, %0, %0 row_bcast:15 row_mask:0xa bank_mask:0xf\n\t"
        "v_min_f32_dpp %1, %1, %1 row_bcast:15 row_mask:0xa bank_mask:0xf\n\t"
        "s_nop 0\n\t"
        "v_min_f32_dpp %0, %0, %0 row_bcast:31 row_mask:0xc bank_mask:0xf\n\t"
        "v_min_f32_dpp %1, %1, %1 row_bcast:31 row_mask:0xc bank_mask:0xf\n\t"
        "s_nop 1"
        : "+v"(a), "+v"(b));
    a = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, a), 63));
    b = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, b), 63));
}

// Wp[r][i] = W[r][perm[i]] as fp32, zero for dead channels.  One row per workgroup: the row is read once, in
// order, into LDS and permuted from there (a thread per element reading W[r][perm[i]] from memory fetched a
// separate 64-byte piece for every two bytes it used).  Dynamic LDS: in halves.
__global__ __launch_bounds__(256) void gq_gather_w(const __half* __restrict__ W, int64_t out, int64_t in,
                                                   const int32_t* __restrict__ perm, const uint8_t* __restrict__ dead,
                                                   float* __restrict__ Wp) {
    extern __shared__ __align__(16) char gw_smem[];
    __half* row = reinterpret_cast<__half*>(gw_smem);
    const int64_t r = blockIdx.x;
    const __half* src = W + r * in;
    for (int64_t j = threadIdx.x; j < in; j += 256) row[j] = src[j];
    __syncthreads();
    for (int64_t i = threadIdx.x; i < in; i += 256) {
        const int32_t j = perm[i];
        Wp[r * in + i] = dead[j] ? 0.0f : __half2float(row[j]);
    }
}

// One 128-channel block [i1, i1 + nbw) for 64 * RPL rows, by a workgroup of four wavefronts.  Lane l
// of the first wave holds RPL rows: per-OC rows 64*block + l (RPL = 1), per-IC rows l + 64p of the
// block's row group (RPL = g/64), so that the group's minimum and maximum are a lane-local step
// plus one wave reduction.  The rows live in an LDS strip; the channels are walked in sub-blocks of
// 16 that the first wave holds in registers: the sub-block's own updates stay in registers, then
// its 16 errors are posted in LDS.  All four waves apply them to the next sub-block's 16 columns at
// once, so that the chain can go on; the columns behind those receive them from the other three
// waves while the first one walks the next sub-block (two error buffers, taken in turn).  One LDS
// read and one write per element for 16 updates, always in channel order (which wave applies them
// does not change a bit).  The block of U is staged in LDS and read with wave-uniform addresses.
// Codes go out in visiting order (16 bytes per row and sub-block).
template <bool IC, int RPL>
__global__ __launch_bounds__(256) void gq_sweep(float* __restrict__ Wp, const float* __restrict__ U,
                                               const int32_t* __restrict__ perm, int64_t out, int64_t in, int64_t i1,
                                               int nbw, int g, float qmax, int mfmt,
                                               const float* __restrict__ st_scales,
                                               const uint8_t* __restrict__ st_zeros, float* __restrict__ scales_out,
                                               uint8_t* __restrict__ zeros_out, uint8_t* __restrict__ Qp,
                                               float* __restrict__ Ep) {
    constexpr int SB = 16, PITCH = GB + 1;
    extern __shared__ __align__(16) char smem[];
    float* Us = reinterpret_cast<float*>(smem);                         // [GB][GB]: rows / columns i1.. of U
    float* Ws = Us + GB * GB;                                           // [64 * RPL][PITCH]
    float* Es0 = Ws + 64 * RPL * PITCH;                                 // [2][64 * RPL][SB + 1]: the errors of this sub-block and the last
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    // The block of U and the strip of W: every thread's loads are issued before the first of them is stored, so the
    // block pays one trip to memory each, not one per loop iteration (16 and 32 of them: a fifth of the kernel).
    {
        constexpr int NU = GB * (GB / 4) / 256;                         // 16-byte pieces of the block of U per thread
        float4 uv[NU];
#pragma unroll
        for (int q = 0; q < NU; ++q) {
            const int e4 = threadIdx.x + 256 * q, k = e4 / (GB / 4), c4 = (e4 % (GB / 4)) * 4;
            float4 v = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            if (k < nbw) {                                              // in % 4 == 0 is not required: guarded
                const float* src = U + (i1 + k) * in + i1 + c4;
                if (c4 + 3 < nbw && ((reinterpret_cast<uintptr_t>(src) & 15u) == 0)) {
                    v = *reinterpret_cast<const float4*>(src);
                } else {
                    if (c4 + 0 < nbw) v.x = src[0];
                    if (c4 + 1 < nbw) v.y = src[1];
                    if (c4 + 2 < nbw) v.z = src[2];
                    if (c4 + 3 < nbw) v.w = src[3];
                }
            }
            uv[q] = v;
        }
#pragma unroll
        for (int q = 0; q < NU; ++q) {
            const int e4 = threadIdx.x + 256 * q, k = e4 / (GB / 4), c4 = (e4 % (GB / 4)) * 4;
            if (k < nbw) *reinterpret_cast<float4*>(Us + k * GB + c4) = uv[q];
        }
    }
    int64_t row[RPL];
    bool ok[RPL];
#pragma unroll
    for (int p = 0; p < RPL; ++p) {
        row[p] = IC ? int64_t(blockIdx.x) * g + lane + 64 * p : int64_t(blockIdx.x) * 64 + lane;
        ok[p] = row[p] < out;
    }
    {
        // strip element (r, c): thread t takes columns t % 128 of rows t / 128 + 2 j, consecutive lanes consecutive
        // columns
        constexpr int NR = 64 * RPL / 2;
        const int c = threadIdx.x & (GB - 1), r_first = threadIdx.x >> 7;
        const int64_t strip_row0 = IC ? int64_t(blockIdx.x) * g : int64_t(blockIdx.x) * 64;
        float wv[NR];
#pragma unroll
        for (int j = 0; j < NR; ++j) {
            const int r = r_first + 2 * j;                              // strip row; per-IC rows l + 64 p sit at (l * RPL + p)
            const int64_t grow = strip_row0 + r;
            wv[j] = (c < nbw && grow < out) ? Wp[grow * in + i1 + c] : 0.0f;
        }
#pragma unroll
        for (int j = 0; j < NR; ++j) {
            const int r = r_first + 2 * j;
            const int slot = IC ? (r & 63) * RPL + (r >> 6) : r;        // row l + 64 p of a group -> strip slot l * RPL + p
            if (c < nbw) Ws[slot * PITCH + c] = wv[j];
        }
    }
    __syncthreads();
    const int n_cg = IC ? 0 : static_cast<int>(in / g);
    // errors of a sub-block applied to columns [c_lo, c_hi), every `step`-th from c_lo + first; channel order kept
    // per element (which wave applies them does not change a bit)
    auto apply = [&](const float* Esrc, int k0, int kw, int c_lo, int c_hi, int first, int step) {
        float e[RPL][SB];
#pragma unroll
        for (int p = 0; p < RPL; ++p)
#pragma unroll
            for (int k = 0; k < SB; ++k) e[p][k] = Esrc[(lane * RPL + p) * (SB + 1) + k];
        for (int cc = c_lo + first; cc < c_hi; cc += step) {
            float u[SB];
#pragma unroll
            for (int k = 0; k < SB; ++k) u[k] = k < kw ? Us[(k0 + k) * GB + cc] : 0.0f;
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
    };
    for (int s0 = 0; s0 < nbw; s0 += SB) {
        const int sbw = nbw - s0 < SB ? nbw - s0 : SB;
        float* Es = Es0 + ((s0 / SB) & 1) * (64 * RPL * (SB + 1));
        const float* Es_last = Es0 + (((s0 / SB) & 1) ^ 1) * (64 * RPL * (SB + 1));
        // the sequential part, one wave; FULL: all 16 channels exist (every sub-block but a ragged last
        // one), which takes the bounds tests and their branches out of the chain
        auto sub_block = [&](auto full_tag) {
            constexpr bool FULL = decltype(full_tag)::value;
            float w[RPL][SB], e[RPL][SB];
            uint32_t qpk[RPL][SB / 4];
#pragma unroll
            for (int p = 0; p < RPL; ++p) {
#pragma unroll
                for (int c = 0; c < SB; ++c) w[p][c] = (ok[p] && (FULL || c < sbw)) ? Ws[(lane * RPL + p) * PITCH + s0 + c] : 0.0f;
#pragma unroll
                for (int c = 0; c < SB / 4; ++c) qpk[p][c] = 0u;
            }
            // the sub-block's original channel indices and, for static groups, its parameters: fetched
            // together up front, off the channel-by-channel chain
            QP st[SB];
            if constexpr (!IC) {
                int32_t jo[SB];
#pragma unroll
                for (int c = 0; c < SB; ++c) jo[c] = (FULL || c < sbw) ? perm[i1 + s0 + c] : 0;
#pragma unroll
                for (int c = 0; c < SB; ++c) {
                    const bool have = ok[0] && (FULL || c < sbw);
                    if (mfmt) {                                            // static parameters as group words
                        const uint32_t wd = have ? reinterpret_cast<const uint16_t*>(st_scales)[row[0] * n_cg + jo[c] / g]
                                                 : (0x3C00u >> (mfmt - 1)) << mfmt;           // scale 1, zero 0
                        st[c].scale = word_scale(wd, mfmt);
                        st[c].zero = word_zero(wd, mfmt);
                    } else {
                        st[c].scale = have ? st_scales[row[0] * n_cg + jo[c] / g] : 1.0f;
                        st[c].zero = have ? static_cast<float>(st_zeros[row[0] * n_cg + jo[c] / g]) : 0.0f;
                    }
                }
            }
            float my_scale = 1.0f, my_zero = 0.0f;                          // lane c: channel c's parameters (per-IC)
            // The sub-block's 16 x 16 corner of U, all of it in registers before the chain starts (16-byte reads at
            // wave-uniform addresses, every index below a constant): read row by row where it is used, each
            // channel's chain began by waiting for its row.  The fence keeps the reads up here.
            float ub[SB][SB];
#pragma unroll
            for (int c = 0; c < SB; ++c)
#pragma unroll
                for (int q4 = 0; q4 < SB / 4; ++q4) {
                    const float4 t = *reinterpret_cast<const float4*>(Us + (s0 + c) * GB + s0 + 4 * q4);
                    ub[c][4 * q4 + 0] = t.x;
                    ub[c][4 * q4 + 1] = t.y;
                    ub[c][4 * q4 + 2] = t.z;
                    ub[c][4 * q4 + 3] = t.w;
                }
            asm volatile("" ::: "memory");
#pragma unroll
            for (int c = 0; c < SB; ++c) {
                if (FULL || c < sbw) {                                      // uniform
                    const float (&u)[SB] = ub[c];
                    const float d = u[c];
                    QP pr[RPL];
                    if constexpr (IC) {
                        float mn = w[0][c], nmx = -w[0][c];
#pragma unroll
                        for (int p = 1; p < RPL; ++p) {
                            mn = fminf(mn, w[p][c]);
                            nmx = fminf(nmx, -w[p][c]);
                        }
                        wave_min2(mn, nmx);
                        const QP q1 = params_of(mn, -nmx, qmax, mfmt);
#pragma unroll
                        for (int p = 0; p < RPL; ++p) pr[p] = q1;
                        if (lane == c) {                                    // two selects; stored after the chain
                            my_scale = q1.scale;
                            my_zero = q1.zero;
                        }
                    } else {
                        pr[0] = st[c];
                    }
#pragma unroll
                    for (int p = 0; p < RPL; ++p) {
                        float q = rintf(w[p][c] / pr[p].scale) + pr[p].zero;
                        q = fminf(fmaxf(q, 0.0f), qmax);
                        const float wq = pr[p].scale * (q - pr[p].zero);
                        qpk[p][c / 4] |= static_cast<uint32_t>(q) << (8 * (c % 4));
                        e[p][c] = (w[p][c] - wq) / d;
                        // (constant bounds with a test, not "cc = c + 1": a trip count that depends on c is
                        // unrolled too late, after the loop has been vectorized with a run-time-indexed remainder)
#pragma unroll
                        for (int cc = 0; cc < SB; ++cc) {
                            if (cc > c && (FULL || cc < sbw)) {
                                const float upd = e[p][c] * u[cc];
                                w[p][cc] = w[p][cc] - upd;
                            }
                        }
                    }
                } else {
#pragma unroll
                    for (int p = 0; p < RPL; ++p) e[p][c] = 0.0f;
                }
            }
            if constexpr (IC) {
                if (lane < sbw)
                    store_params(scales_out, zeros_out, int64_t(blockIdx.x) * in + perm[i1 + s0 + lane], my_scale, my_zero, mfmt);
            }
            // the sub-block's codes and errors, in visiting order
#pragma unroll
            for (int p = 0; p < RPL; ++p) {
                if (!ok[p]) continue;
                const int64_t at = row[p] * in + i1 + s0;
                if (FULL && ((at & 15) == 0)) {
                    *reinterpret_cast<uint4*>(Qp + at) = make_uint4(qpk[p][0], qpk[p][1], qpk[p][2], qpk[p][3]);
                } else {
                    for (int c = 0; c < sbw; ++c) Qp[at + c] = static_cast<uint8_t>(qpk[p][c / 4] >> (8 * (c % 4)));
                }
                if (FULL && ((at & 3) == 0)) {
#pragma unroll
                    for (int c = 0; c < SB; c += 4)
                        *reinterpret_cast<float4*>(Ep + at + c) = make_float4(e[p][c], e[p][c + 1], e[p][c + 2], e[p][c + 3]);
                } else {
                    for (int c = 0; c < sbw; ++c) Ep[at + c] = e[p][c];
                }
            }
#pragma unroll
            for (int p = 0; p < RPL; ++p)
#pragma unroll
                for (int k = 0; k < SB; ++k) Es[(lane * RPL + p) * (SB + 1) + k] = e[p][k];
        };
        if (wave == 0) {
            // the chain every later launch waits for: ahead of the bulk update that shares the SIMD with it
            __builtin_amdgcn_s_setprio(3);
            if (sbw == SB) sub_block(std::true_type{});
            else sub_block(std::false_type{});
            __builtin_amdgcn_s_setprio(0);
        } else if (s0 > 0 && s0 + SB < nbw) {
            // meanwhile the other three waves bring the columns behind this sub-block up to date with the
            // errors of the sub-block before it (this sub-block's own columns got them ahead of the chain)
            apply(Es_last, s0 - SB, SB, s0 + SB, nbw, wave - 1, 3);
        }
        __syncthreads();
        // the new errors go to the next sub-block's columns at once, all four waves, so that the chain can go on
        if (s0 + SB < nbw) apply(Es, s0, sbw, s0 + SB, s0 + 2 * SB < nbw ? s0 + 2 * SB : nbw, wave, 4);
        __syncthreads();
    }
}

// visited[perm[i]] = i: where in the visiting order an original channel sits
__global__ void gq_invperm(const int32_t* __restrict__ perm, int64_t in, int32_t* __restrict__ visited) {
    const int64_t i = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i < in) visited[perm[i]] = static_cast<int32_t>(i);
}

// codes back to the original channel order, and dW = W - scale*(code - zero) there.  One row per workgroup:
// its codes in visiting order are read once into LDS and looked up there; the writes (and the reads of W and the
// parameters) are consecutive.  Dynamic LDS: in bytes.
template <bool IC>
__global__ __launch_bounds__(256) void gq_scatter(const uint8_t* __restrict__ Qp, const int32_t* __restrict__ visited,
                                                  const uint8_t* __restrict__ dead, const __half* __restrict__ W, int64_t out,
                                                  int64_t in, int g, const float* __restrict__ scales,
                                                  const uint8_t* __restrict__ zeros, int mfmt, uint8_t* __restrict__ codes,
                                                  float* __restrict__ dW) {
    extern __shared__ __align__(16) char gs_smem[];
    uint8_t* qrow = reinterpret_cast<uint8_t*>(gs_smem);
    const int64_t r = blockIdx.x;
    for (int64_t i = threadIdx.x; i < in; i += 256) qrow[i] = Qp[r * in + i];
    __syncthreads();
    for (int64_t j = threadIdx.x; j < in; j += 256) {
        const int64_t idx = r * in + j;
        const uint8_t q = qrow[visited[j]];
        codes[idx] = q;
        if (dW) {
            const int64_t pi = IC ? (r / g) * in + j : r * (in / g) + j / g;
            float sc, zp;
            if (mfmt) {
                const uint32_t wd = reinterpret_cast<const uint16_t*>(scales)[pi];
                sc = word_scale(wd, mfmt);
                zp = word_zero(wd, mfmt);
            } else {
                sc = scales[pi];
                zp = static_cast<float>(zeros[pi]);
            }
            const float wq = sc * (static_cast<float>(q) - zp);
            dW[idx] = (dead[j] ? 0.0f : __half2float(W[idx])) - wq;
        }
    }
}

// channels behind the block, columns [col0, col1): Wp[r][jj] -= E[r][k] * U[k][jj], k = i1 .. i2-1 in order
// (product, then difference)
__global__ __launch_bounds__(256) void gq_trailing(float* __restrict__ Wp, const float* __restrict__ U,
                                                   const float* __restrict__ Ep, int64_t out, int64_t in, int64_t i1,
                                                   int nbw, int64_t col0, int64_t col1) {
    __shared__ __align__(16) float Es[GB][8];                 // [channel][row]: a channel's eight errors in two 16-byte reads
    const int64_t jj = col0 + int64_t(blockIdx.x) * 256 + threadIdx.x;
    const int64_t r0 = int64_t(blockIdx.y) * 8;
    for (int e = threadIdx.x; e < 8 * nbw; e += 256) {
        const int rr = e / nbw, k = e % nbw;
        Es[k][rr] = r0 + rr < out ? Ep[(r0 + rr) * in + i1 + k] : 0.0f;
    }
    __syncthreads();
    if (jj >= col1) return;
    float v[8];
#pragma unroll
    for (int rr = 0; rr < 8; ++rr) v[rr] = r0 + rr < out ? Wp[(r0 + rr) * in + jj] : 0.0f;
#pragma unroll 4
    for (int k = 0; k < nbw; ++k) {
        const float u = U[(i1 + k) * in + jj];
        const float4 ea = *reinterpret_cast<const float4*>(&Es[k][0]), eb = *reinterpret_cast<const float4*>(&Es[k][4]);
        const float e8[8] = {ea.x, ea.y, ea.z, ea.w, eb.x, eb.y, eb.z, eb.w};
#pragma unroll
        for (int rr = 0; rr < 8; ++rr) {
            const float upd = e8[rr] * u;
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
    // products C inv(A) of the inverse's doubling levels: pairs * s * s doubles at level s
    size_t t_elems = 1;
    for (int64_t s = NB; s < n; s *= 2) t_elems = std::max(t_elems, size_t((n - s + 2 * s - 1) / (2 * s)) * size_t(s) * size_t(s));
    double* T = static_cast<double*>(adadim_workspace(ctx, WS_GPTQ_T, t_elems * sizeof(double)));
    int32_t* rank = static_cast<int32_t*>(adadim_workspace(ctx, WS_GPTQ_V, size_t(n) * sizeof(int32_t)));   // free here
    if (!A || !M || !dvec || !T || !rank) return ADADIM_EHIP;
    double* damp = dvec + n;
    const unsigned nb1 = static_cast<unsigned>((n + 255) / 256), nb2 = static_cast<unsigned>((n * n + 255) / 256);
    ProfScope prof(ctx, "gptq_prepare");
    hipLaunchKernelGGL(gq_diag, dim3(nb1), dim3(256), 0, ctx->stream, H, n, dvec, dead);
    hipLaunchKernelGGL(gq_damp, dim3(1), dim3(256), 0, ctx->stream, dvec, n, static_cast<double>(percdamp), damp);
    if (act_order) {
        hipLaunchKernelGGL(gq_zero_i32, dim3(nb1), dim3(256), 0, ctx->stream, rank, n);
        hipLaunchKernelGGL(gq_rank_count, dim3(nb1, static_cast<unsigned>((n + 1023) / 1024)), dim3(256), 0, ctx->stream,
                           dvec, n, rank);
        hipLaunchKernelGGL(gq_rank_place, dim3(nb1), dim3(256), 0, ctx->stream, rank, n, perm);
    } else
        hipLaunchKernelGGL(gq_rank, dim3(nb1), dim3(256), 0, ctx->stream, dvec, n, act_order, perm);
    hipLaunchKernelGGL(gq_gather, dim3(nb2), dim3(256), 0, ctx->stream, H, n, perm, dvec, damp, A);
    ADADIM_LAUNCH_CHECK(ctx, "gptq prepare");
    // Outer panels of 512 columns: inside a panel the 64-wide steps update the panel's own columns
    // only; the columns behind it get the whole panel at once, a product with 256 contraction steps
    // per pass over the trailing matrix instead of 64.
    const bool overlap = n > 2 * NBO;
    if (overlap && !adadim_side_stream(ctx)) return ADADIM_EHIP;
    bool side_busy = false;
    bool diag_ready = false;                                  // the block at the next k0 is already factored (chol_syrk_diag)
    static_assert(GT == NB, "chol_syrk_diag's first tile is the next diagonal block");
    for (int64_t K0 = 0; K0 < n; K0 += NBO) {
        const int64_t W = n - K0 < NBO ? n - K0 : NBO;
        for (int64_t k0 = K0; k0 < K0 + W; k0 += NB) {
            const int w = static_cast<int>(n - k0 < NB ? n - k0 : NB);
            if (!diag_ready) hipLaunchKernelGGL(chol_diag_inv, dim3(1), dim3(256), 0, ctx->stream, A, M, n, k0, w);
            diag_ready = false;
            const int64_t rest = n - k0 - w;
            if (rest > 0) {
                const unsigned t = static_cast<unsigned>((rest + GT - 1) / GT);
                hipLaunchKernelGGL(chol_panel, dim3(t), dim3(256), 0, ctx->stream, A, M, n, k0, w);
                const unsigned tc = static_cast<unsigned>((K0 + W - (k0 + w) + GT - 1) / GT);
                if (tc > 0) {
                    hipLaunchKernelGGL(chol_syrk_diag, dim3(tc, t), dim3(256), 0, ctx->stream, A, M, n, k0, w, k0 + w);
                    diag_ready = true;
                }
            }
        }
        const int64_t rest = n - K0 - W;
        if (rest > 0) {
            // The panel's update of everything behind it.  The next panel's own columns first, on the main
            // stream (its first tile's workgroup factors the next diagonal block as well): the panel's 64-wide
            // steps need nothing else.  The columns behind those on the side stream, under those steps (which are
            // chains of small launches that leave the chip idle).  Every element still receives the panels'
            // updates in panel order: the side stream applies them in order, and the main stream waits for the
            // side stream's last launch before it updates columns that launch wrote.
            const unsigned t = static_cast<unsigned>((rest + GT - 1) / GT);
            const unsigned tn = static_cast<unsigned>(((rest < NBO ? rest : NBO) + GT - 1) / GT);
            if (side_busy) ADADIM_HIP_TRY(ctx, hipStreamWaitEvent(ctx->stream, ctx->side_ev[1], 0));
            side_busy = false;
            // both launches need the finished panel, and write different tile columns: the side stream starts with
            // the main stream's launch, not behind it
            if (overlap && t > tn) ADADIM_HIP_TRY(ctx, hipEventRecord(ctx->side_ev[0], ctx->stream));
            hipLaunchKernelGGL(chol_syrk_diag, dim3(overlap ? tn : t, t), dim3(256), 0, ctx->stream, A, M, n, K0,
                               static_cast<int>(W), K0 + W);
            diag_ready = true;
            if (overlap && t > tn) {
                ADADIM_HIP_TRY(ctx, hipStreamWaitEvent(ctx->side, ctx->side_ev[0], 0));
                hipLaunchKernelGGL(chol_syrk<GT>, dim3(t - tn, t), dim3(256), 0, ctx->side, A, n, K0, static_cast<int>(W),
                                   K0 + W, static_cast<int>(tn));
                ADADIM_HIP_TRY(ctx, hipEventRecord(ctx->side_ev[1], ctx->side));
                side_busy = true;
            }
        }
    }
    if (side_busy) ADADIM_HIP_TRY(ctx, hipStreamWaitEvent(ctx->stream, ctx->side_ev[1], 0));   // join
    ADADIM_LAUNCH_CHECK(ctx, "gptq cholesky");
    for (int64_t s = NB; s < n; s *= 2) {
        const unsigned pairs = static_cast<unsigned>((n - s + 2 * s - 1) / (2 * s));   // those with rows below a0 + s
        const dim3 grid(static_cast<unsigned>(s / GT), static_cast<unsigned>(s / GT), pairs);
        hipLaunchKernelGGL((trinv_level<0, GT>), grid, dim3(256), 0, ctx->stream, A, M, T, n, s);
        hipLaunchKernelGGL((trinv_level<1, GT>), grid, dim3(256), 0, ctx->stream, A, M, T, n, s);
    }
    hipLaunchKernelGGL(gq_flip, dim3(nb2), dim3(256), 0, ctx->stream, M, n, U);
    ADADIM_LAUNCH_CHECK(ctx, "gptq inverse");
    return ADADIM_OK;
}

int launch_gptq_quantize(adadim_ctx* ctx, const __half* W, int64_t out, int64_t in, int dim, int bits, int g,
                         const float* U, const int32_t* perm, const uint8_t* dead, const float* st_scales,
                         const uint8_t* st_zeros, uint8_t* codes, float* scales_out, uint8_t* zeros_out, float* dW,
                         int mfmt) {
    const size_t mat = size_t(out) * size_t(in) * sizeof(float);
    float* Wp = static_cast<float*>(adadim_workspace(ctx, WS_GPTQ_W, mat));
    float* Ep = static_cast<float*>(adadim_workspace(ctx, WS_GPTQ_E, mat));
    uint8_t* Qp = static_cast<uint8_t*>(adadim_workspace(ctx, WS_GPTQ_Q, size_t(out) * size_t(in)));
    int32_t* visited = static_cast<int32_t*>(adadim_workspace(ctx, WS_GPTQ_V, size_t(in) * sizeof(int32_t)));
    if (!Wp || !Ep || !Qp || !visited) return ADADIM_EHIP;
    const float qmax = static_cast<float>((1 << bits) - 1);
    const bool ic = dim == ADADIM_DIM_IC;
    const int rpl = ic ? g / 64 : 1;                                   // rows per lane
    const unsigned blocks = static_cast<unsigned>(ic ? out / g : (out + 63) / 64);
    const size_t smem = (size_t(GB) * GB + size_t(64) * rpl * (GB + 1) + size_t(2) * 64 * rpl * 17) * sizeof(float);
    static PerDeviceOnce once;
    ADADIM_HIP_TRY(ctx, once.run([] {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(gq_sweep<true, 2>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 152 * 1024);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(gq_sweep<true, 1>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, 152 * 1024);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(gq_sweep<false, 1>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, 152 * 1024);
        // a row of W in LDS: up to 46340 halves
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(gq_gather_w),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024);
        return e;
    }));
    {
        ProfScope prof(ctx, "gptq_gather");
        hipLaunchKernelGGL(gq_gather_w, dim3(static_cast<unsigned>(out)), dim3(256), static_cast<size_t>(in) * 2, ctx->stream, W, out,
                           in, perm, dead, Wp);
    }
    // A block's errors reach the channels behind it in two launches: the next block's 128 channels at
    // once, on the main stream, so that the next sweep can start; the rest on a side stream, under
    // that sweep, which keeps only a few compute units busy.  Every element still receives the
    // blocks' errors in block order: the side stream applies them in order, and the main stream
    // waits for the side stream's last launch before it adds the following block's errors to the
    // channels that launch wrote.  With per-kernel timing on, everything runs on the main stream.
    const bool overlap = !ctx->prof.enabled && in > 2 * GB;
    if (overlap && !adadim_side_stream(ctx)) return ADADIM_EHIP;
    bool side_busy = false;
    for (int64_t i1 = 0; i1 < in; i1 += GB) {
        const int nbw = static_cast<int>(in - i1 < GB ? in - i1 : GB);
        {
            ProfScope prof(ctx, "gptq_sweep");
#define GQ_GO(IC_, RPL_)                                                                                          \
    hipLaunchKernelGGL((gq_sweep<IC_, RPL_>), dim3(blocks), dim3(256), smem, ctx->stream, Wp, U, perm, out, in, i1, \
                       nbw, g, qmax, mfmt, st_scales, st_zeros, scales_out, zeros_out, Qp, Ep)
            if (!ic) GQ_GO(false, 1);
            else if (rpl == 1) GQ_GO(true, 1);
            else GQ_GO(true, 2);
#undef GQ_GO
        }
        const int64_t behind = i1 + nbw;                        // first channel behind the block
        if (behind >= in) break;
        const int64_t next_end = behind + GB < in ? behind + GB : in;
        const unsigned rows8 = static_cast<unsigned>((out + 7) / 8);
        if (!overlap) {
            ProfScope prof(ctx, "gptq_trailing");
            hipLaunchKernelGGL(gq_trailing, dim3(static_cast<unsigned>((in - behind + 255) / 256), rows8), dim3(256), 0,
                               ctx->stream, Wp, U, Ep, out, in, i1, nbw, behind, in);
            continue;
        }
        if (side_busy) ADADIM_HIP_TRY(ctx, hipStreamWaitEvent(ctx->stream, ctx->side_ev[1], 0));
        hipLaunchKernelGGL(gq_trailing, dim3(static_cast<unsigned>((next_end - behind + 255) / 256), rows8), dim3(256), 0,
                           ctx->stream, Wp, U, Ep, out, in, i1, nbw, behind, next_end);
        // the side stream starts behind this short launch, not beside it: the next sweep waits for it
        ADADIM_HIP_TRY(ctx, hipEventRecord(ctx->side_ev[0], ctx->stream));
        if (next_end < in) {
            ADADIM_HIP_TRY(ctx, hipStreamWaitEvent(ctx->side, ctx->side_ev[0], 0));
            hipLaunchKernelGGL(gq_trailing, dim3(static_cast<unsigned>((in - next_end + 255) / 256), rows8), dim3(256), 0,
                               ctx->side, Wp, U, Ep, out, in, i1, nbw, next_end, in);
            ADADIM_HIP_TRY(ctx, hipEventRecord(ctx->side_ev[1], ctx->side));
            side_busy = true;
        }
    }
    if (side_busy) ADADIM_HIP_TRY(ctx, hipStreamWaitEvent(ctx->stream, ctx->side_ev[1], 0));   // join
    {
        ProfScope prof(ctx, "gptq_scatter");
        hipLaunchKernelGGL(gq_invperm, dim3(static_cast<unsigned>((in + 255) / 256)), dim3(256), 0, ctx->stream, perm, in,
                           visited);
        if (ic)
            hipLaunchKernelGGL(gq_scatter<true>, dim3(static_cast<unsigned>(out)), dim3(256), static_cast<size_t>(in), ctx->stream, Qp, visited, dead, W, out, in, g,
                               scales_out, zeros_out, mfmt, codes, dW);
        else
            hipLaunchKernelGGL(gq_scatter<false>, dim3(static_cast<unsigned>(out)), dim3(256), static_cast<size_t>(in), ctx->stream, Qp, visited, dead, W, out, in, g,
                               st_scales, st_zeros, mfmt, codes, dW);
    }
    ADADIM_LAUNCH_CHECK(ctx, "gptq sweep");
    return ADADIM_OK;
}
