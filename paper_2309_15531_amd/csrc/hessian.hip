// H (+)= X^T X on the matrix cores, and the preparation of H for scoring.
//
// H is the Gram matrix that turns the reconstruction error of Eq. 1 (Sec. 3.3)
// into a quadratic form in dW.  It is a symmetric rank-k update whose
// contraction runs over the tokens, the slow axis of X, so both operands are
// transposed on their way into LDS.  Only tiles on or above the diagonal are
// computed.  As many tiles as fill whole rounds of the chip run over all tokens
// and store their part of H themselves, both halves; for the others the token
// range is split over workgroups to fill the last round, each (tile, split)
// writes an fp32 partial tile, and a second kernel adds the partials in a
// fixed order, mirrors the result and stores or accumulates H.
// No atomics: the result is bit-reproducible and exactly symmetric.
#include "common.h"

#include <algorithm>
#include <cmath>
#include <cstring>
#include <vector>
#include "mfma_tile.h"
#include "gram_dma.h"

namespace {

using namespace mfma;

template <int BT>
__global__ __launch_bounds__(THREADS) void gram_tiles(const __half* __restrict__ X, int64_t tokens, int64_t in,
                                                      int64_t ldx, int nb, int64_t t_per_split,
                                                      float* __restrict__ part) {
    constexpr int WM = BT / 2, TM = WM / 32;
    extern __shared__ __align__(16) char smem[];
    constexpr int TILE_BYTES = BT * ROW_BYTES;
    auto sA = [&](int b) { return smem + b * (2 * TILE_BYTES); };
    auto sB = [&](int b) { return smem + b * (2 * TILE_BYTES) + TILE_BYTES; };

    int I, J;
    decode_tile(blockIdx.x, nb, I, J);
    const int64_t t_begin = int64_t(blockIdx.y) * t_per_split;
    const int64_t t_end = min(tokens, t_begin + t_per_split);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    floatx16 acc[TM][TM];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    TransposeStage<BT> ga, gb;
    const int64_t rowA = int64_t(I) * BT, rowB = int64_t(J) * BT;
    if (t_begin < t_end) {
        ga.load(X, ldx, rowA, in, t_begin, t_end, tid);
        gb.load(X, ldx, rowB, in, t_begin, t_end, tid);
        ga.store(sA(0), tid);
        gb.store(sB(0), tid);
    }
    __syncthreads();
    int buf = 0;
    for (int64_t k0 = t_begin; k0 < t_end; k0 += KT) {
        const bool more = k0 + KT < t_end;
        if (more) {
            ga.load(X, ldx, rowA, in, k0 + KT, t_end, tid);
            gb.load(X, ldx, rowB, in, k0 + KT, t_end, tid);
        }
        mma_stage<TM, TM>(sA(buf), sB(buf), wm * WM, wn * WM, lane, acc);
        if (more) {
            ga.store(sA(buf ^ 1), tid);
            gb.store(sB(buf ^ 1), tid);
        }
        __syncthreads();
        buf ^= 1;
    }

    float* dst = part + (int64_t(blockIdx.y) * gridDim.x + blockIdx.x) * (int64_t(BT) * BT);
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = wm * WM + 32 * i + acc_row(r, lane);
                const int col = wn * WM + 32 * j + (lane & 31);
                dst[row * BT + col] = acc[i][j][r];
            }
}

// Adds the split partials of one 32x32 sub-block, writes it to H and, off the
// diagonal, its mirror image.  grid = tiles * (sub-blocks per tile side)^2.
// REGMAJOR: the partial tiles are in the register order of the DMA tile kernel (float4 number
// ((i*4 + j)*4 + q)*256 + thread holds accumulator registers 4q..4q+3 of that thread's 32x32 block
// (i, j)), which for thread (tx, ty) here is one 16-byte load: rows 4*ty..4*ty+3 of column tx.
//
// PREP (accumulate == 0 only): the same pass also writes what adadim_hessian_prepare derives from H, so
// that H is not read back and two launches fall away: hmeta (from the diagonal blocks) and the scaled
// fp16 Hs in the scoring layout, Hs[n,k] = H[n,k]/(d_n d_k) for k < n and 0 elsewhere.  The block
// needs d for its 32 rows and 32 columns: each is a function of a diagonal entry of H, which the
// block adds up itself from the partial diagonal tiles, in the same order as the block that owns
// that entry, hence to the same bits.

// index of the diagonal tile (I, I) in decode_tile's order
__host__ __device__ inline int diag_tile_index(int I, int nb) {
    const int s = I >> 2;
    int base = 0;
    for (int t = 0; t < s; ++t) {
        const int rows = min(4, nb - 4 * t);
        base += rows * (rows + 1) / 2 + rows * max(0, nb - 4 * t - 4);
    }
    const int c = I - 4 * s;
    return base + c * (c + 1) / 2 + c;
}

// d = 2^(round(log2(h)/2) - 6) (1 if h <= 0): a power of two near sqrt(h) / 64.  Any power of two serves (the
// scaling is undone exactly); this one splits fp16's 30 binades between the two scoring operands so that neither
// leaves them for any fp16 input: Hs = H / (d d) stays below 2^13, and dW' = dW d stays finite up to
// |dW| sqrt(h) = 4e6, which weights of ordinary size do not reach even on activations at fp16's largest value
// in every token.  The exponent is clamped so that d, 1/d and d*d stay normal fp32 numbers.
constexpr int SCORE_SHIFT = 6;
__device__ __forceinline__ float jacobi_scale(float h) {
    float d = 1.0f;
    if (h > 0.0f && h < 3.0e38f) {
        int e = static_cast<int>(rintf(0.5f * log2f(h))) - SCORE_SHIFT;
        e = max(-30, min(30, e));
        d = ldexpf(1.0f, e);
    }
    return d;
}

template <int BT, bool REGMAJOR = false, bool PREP = false>
__global__ __launch_bounds__(256) void gram_reduce(const float* __restrict__ part, GramPlan plan, int nb, int64_t in,
                                                   float* __restrict__ H, int accumulate, __half* __restrict__ Hs,
                                                   float* __restrict__ hmeta) {
    constexpr int SB = BT / 32;
    __shared__ float s[32][33];
    __shared__ float s_rd[2][32];                             // PREP: 1/d of the block's rows and columns
    // the grid holds the tiles with partials (n_whole .. n_tiles - 1) and, behind them when PREP, the diagonal tiles
    // among the whole ones (the first ones in diagonal order: diag_tile_index grows with the tile's row)
    const int n_tiles = plan.n_tiles, n_whole = plan.n_whole;
    const int slot = blockIdx.x / (SB * SB), sub = blockIdx.x % (SB * SB);
    const int tile = slot < n_tiles - n_whole ? n_whole + slot : diag_tile_index(slot - (n_tiles - n_whole), nb);
    int I, J;
    decode_tile(tile, nb, I, J);
    const int sr = sub / SB, sc = sub % SB;
    const int64_t R0 = int64_t(I) * BT + sr * 32, C0 = int64_t(J) * BT + sc * 32;
    if (R0 > C0 || R0 >= in || C0 >= in) return;  // below the diagonal or outside H
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    // The first n_whole tiles are in H already, both halves (the tile kernel ran them over all tokens and stored
    // them itself): nothing to add up, only the prepared form to derive, from H (here for the diagonal tiles among
    // them, which also yield hmeta).  The others have the plan's partial tiles, added in the order of their tokens.
    const bool whole = tile < n_whole;
    if (whole && (!PREP || I != J)) return;                   // prepared form of whole off-diagonal tiles: gram_prep_whole
    // A tile's partials are two runs of slots with a constant stride each: the full pieces (one per split, a
    // split apart) and the pieces of the rest (next to each other).
    constexpr int64_t TILE = int64_t(BT) * BT;
    struct Runs { const float* a; int na; int64_t sa; const float* b; int nb; };
    auto runs_of = [&](int tile_r) {
        const int n = gram_plan_parts(plan, tile_r);
        Runs r;
        r.a = part + int64_t(tile_r) * TILE;
        r.na = plan.n_full;
        r.sa = int64_t(gram_plan_rest(plan)) * TILE;
        r.nb = n - plan.n_full;
        r.b = r.nb > 0 ? part + int64_t(gram_plan_slot(plan, tile_r, plan.n_full)) * TILE : part;
        return r;
    };
    const Runs mine = whole ? Runs{part, 0, 0, part, 0} : runs_of(tile - n_whole);
    if (whole) {
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
            const int r = ty * 4 + rr;
            s[r][tx] = (R0 + r < in && C0 + tx < in) ? H[(R0 + r) * in + C0 + tx] : 0.0f;
        }
    } else if constexpr (REGMAJOR) {
        static_assert(!REGMAJOR || BT == 256, "register-major partials come from the 256-wide DMA kernel");
        const int wave = (sr >> 2) * 2 + (sc >> 2);
        const int64_t idx = (((sr & 3) * 4 + (sc & 3)) * 4 + (ty >> 1)) * 256 + wave * 64 + (ty & 1) * 32 + tx;
        float4 v = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        for (int sp = 0; sp < mine.na; ++sp) {
            const float4 p = *reinterpret_cast<const float4*>(mine.a + sp * mine.sa + idx * 4);
            v.x += p.x; v.y += p.y; v.z += p.z; v.w += p.w;
        }
        for (int sp = 0; sp < mine.nb; ++sp) {
            const float4 p = *reinterpret_cast<const float4*>(mine.b + sp * TILE + idx * 4);
            v.x += p.x; v.y += p.y; v.z += p.z; v.w += p.w;
        }
        s[ty * 4 + 0][tx] = v.x;
        s[ty * 4 + 1][tx] = v.y;
        s[ty * 4 + 2][tx] = v.z;
        s[ty * 4 + 3][tx] = v.w;
    } else {
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
            const int r = ty * 4 + rr;
            float v = 0.0f;
            const int64_t at = (sr * 32 + r) * BT + sc * 32 + tx;
            for (int sp = 0; sp < mine.na; ++sp) v += mine.a[sp * mine.sa + at];
            for (int sp = 0; sp < mine.nb; ++sp) v += mine.b[sp * TILE + at];
            s[r][tx] = v;
        }
    }
    const bool diag = R0 == C0;
    if constexpr (PREP) {
        if (threadIdx.x < 64) {
            const int which = threadIdx.x >> 5, a = threadIdx.x & 31;   // 0: the block's rows, 1: its columns
            const int T = which ? J : I, sb = which ? sc : sr;
            const int64_t j = int64_t(T) * BT + sb * 32 + a;
            float h = 0.0f;
            if (j < in) {
                int64_t off;
                if constexpr (REGMAJOR) {
                    const int ty2 = a >> 2, w2 = 3 * (sb >> 2);
                    off = ((((sb & 3) * 5) * 4 + (ty2 >> 1)) * 256 + w2 * 64 + (ty2 & 1) * 32 + a) * 4 + (a & 3);
                } else {
                    off = int64_t(sb * 32 + a) * BT + sb * 32 + a;
                }
                const int dtile = diag_tile_index(T, nb);
                if (dtile < n_whole) {
                    h = H[j * in + j];
                } else {
                    const Runs dg = runs_of(dtile - n_whole);
                    for (int sp = 0; sp < dg.na; ++sp) h += dg.a[sp * dg.sa + off];
                    for (int sp = 0; sp < dg.nb; ++sp) h += dg.b[sp * TILE + off];
                }
            }
            const float d = jacobi_scale(h);
            s_rd[which][a] = 1.0f / d;                        // exact: a power of two
            if (diag && which == 0 && j < in) {
                hmeta[j] = d;
                hmeta[in + j] = h;
            }
        }
    }
    __syncthreads();
    if constexpr (PREP) {
        // 16-byte stores: a row of the block is 32 fp16 = four pieces.  Threads 0..127 write the mirrored
        // block Hs[n = C0 + nl][k = R0 + kq ..+7] = H[k][n] / (d_n d_k), threads 128..255 the zeros above
        // the diagonal, Hs[n = R0 + nl][k = C0 + kq ..+7].  in % 8 == 0: a piece is inside or outside whole.
        const int t = threadIdx.x & 127, nl = t >> 2, kq = (t & 3) * 8;
        if (threadIdx.x < 128) {
            const int64_t n = C0 + nl, k = R0 + kq;
            if (n < in && k < in) {
                uint4 o;
                __half2* h = reinterpret_cast<__half2*>(&o);
#pragma unroll
                for (int e = 0; e < 8; e += 2) {
                    const float v0 = k + e < n ? s[kq + e][nl] * s_rd[1][nl] * s_rd[0][kq + e] : 0.0f;
                    const float v1 = k + e + 1 < n ? s[kq + e + 1][nl] * s_rd[1][nl] * s_rd[0][kq + e + 1] : 0.0f;
                    h[e / 2] = __floats2half2_rn(v0, v1);
                }
                *reinterpret_cast<uint4*>(Hs + score_index(n, k, in, in)) = o;
            }
        } else if (!diag) {
            const int64_t n = R0 + nl, k = C0 + kq;
            if (n < in && k < in) *reinterpret_cast<uint4*>(Hs + score_index(n, k, in, in)) = make_uint4(0, 0, 0, 0);
        }
    }
    if (whole) return;                                        // H holds the tile already
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) {
        const int r = ty * 4 + rr;
        // upper block: element (r, tx); on a diagonal block take the upper triangle for both halves
        if (R0 + r < in && C0 + tx < in) {
            const float v = (diag && r > tx) ? s[tx][r] : s[r][tx];
            float* p = H + (R0 + r) * in + C0 + tx;
            *p = accumulate ? *p + v : v;
        }
        // mirrored block: element (r, tx) of the transpose
        if (!diag && C0 + r < in && R0 + tx < in) {
            const float v = s[tx][r];
            float* p = H + (C0 + r) * in + R0 + tx;
            *p = accumulate ? *p + v : v;
        }
    }
}

// Prepared form of the off-diagonal tiles that the tile kernel stored whole (256 x 256): Hs[n, k] = H[k, n] / (d_n d_k) for the tile's rows k and columns n, and zeros in the mirrored
// place.  A block takes 32 rows of the tile: it reads 32 x 1 KB of H, turns them through LDS and writes the 16 KB
// that these 32 k and the tile's 256 n occupy in the scoring layout in one piece, then 8 x 2 KB of zeros.  d comes
// from hmeta, which gram_reduce has written by then.
__global__ __launch_bounds__(256) void gram_prep_whole(const float* __restrict__ H, int nb, int64_t in, const float* __restrict__ hmeta,
                                                       __half* __restrict__ Hs) {
    constexpr int BT = 256;
    __shared__ float s[BT][33];
    __shared__ float s_rk[32];
    int I, J;
    decode_tile(blockIdx.x >> 3, nb, I, J);
    if (I == J) return;
    const int strip = blockIdx.x & 7, t = threadIdx.x;
    const int64_t R0 = int64_t(I) * BT + strip * 32, C0 = int64_t(J) * BT;
    // (a ragged last tile: rows and columns past the end read as zero and are not stored; in % 8 == 0)
    if (t < 32) s_rk[t] = R0 + t < in ? 1.0f / hmeta[R0 + t] : 1.0f;   // exact: powers of two
    const float rn = C0 + t < in ? 1.0f / hmeta[C0 + t] : 1.0f;
    {
        const int c4 = (t & 63) * 4, r_first = t >> 6;
        float4 v[8];
#pragma unroll
        for (int q = 0; q < 8; ++q)
            v[q] = (R0 + r_first + 4 * q < in && C0 + c4 < in)
                       ? *reinterpret_cast<const float4*>(H + (R0 + r_first + 4 * q) * in + C0 + c4)
                       : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const int r = r_first + 4 * q;
            s[c4][r] = v[q].x; s[c4 + 1][r] = v[q].y; s[c4 + 2][r] = v[q].z; s[c4 + 3][r] = v[q].w;
        }
    }
    __syncthreads();
    // thread t = column n of the tile: its 32 k are 64 contiguous bytes, the block's 256 n x 64 bytes one 16 KB piece
    {
        uint4 o[4];
        __half2* h = reinterpret_cast<__half2*>(o);
#pragma unroll
        for (int e = 0; e < 32; e += 2)
            h[e / 2] = __floats2half2_rn(s[t][e] * rn * s_rk[e], s[t][e + 1] * rn * s_rk[e + 1]);
        if (C0 + t < in) {
            uint4* dst = reinterpret_cast<uint4*>(Hs + score_index(C0 + t, R0, in, in));
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (R0 + 8 * q < in) dst[q] = o[q];
        }
    }
    // zeros above the diagonal: rows n = R0 .. R0 + 31, the tile's 8 column blocks of 32 k, 64 bytes per row and block
    {
        const int kb = t >> 5, nl = t & 31;
        if (R0 + nl < in && C0 + 32 * kb < in) {
            uint4* dst = reinterpret_cast<uint4*>(Hs + score_index(R0 + nl, C0 + 32 * kb, in, in));
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (C0 + 32 * kb + 8 * q < in) dst[q] = make_uint4(0, 0, 0, 0);
        }
    }
}

__global__ void zero_f32(float* p, int64_t n) {
    const int64_t i = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0.0f;
}

// hmeta[0,j] = d_j = 2^round(log2(H_jj)/2) (1 if H_jj <= 0), hmeta[1,j] = H_jj.
__global__ void hprep_meta(const float* __restrict__ H, int64_t in, float* __restrict__ hmeta) {
    const int64_t j = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (j >= in) return;
    const float h = H[j * in + j];
    const float d = jacobi_scale(h);
    hmeta[j] = d;
    hmeta[in + j] = h;
}

// Hs[n,k] = fp16(H[n,k] / (d_n d_k)) for k < n, else 0, stored in the scoring layout.  8 elements per thread.
__global__ __launch_bounds__(256) void hprep_scale(const float* __restrict__ H, int64_t in,
                                                   const float* __restrict__ hmeta, __half* __restrict__ Hs) {
    const int64_t chunks_per_row = in / 8;
    const int64_t c = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (c * 8 >= score_elems(in, in)) return;
    // Threads walk the OUTPUT in memory order, so that stores are contiguous in either layout:
    // blocked (in % 32 == 0): 16-byte piece c is (row tile, k block, row in tile, quarter).
    int64_t n, k0;
    if (score_blocked(in)) {
        const int64_t piece = c >> 10;                       // (row tile, k block): 256 rows x 4 quarters each
        n = (piece / (in >> 5)) * 256 + ((c >> 2) & 255);
        k0 = (piece % (in >> 5)) * 32 + (c & 3) * 8;
        if (n >= in) return;                                 // padding rows of the last tile
    } else {
        n = c / chunks_per_row;
        k0 = (c % chunks_per_row) * 8;
    }
    uint4 o = make_uint4(0, 0, 0, 0);
    if (k0 < n) {
        const float rn = 1.0f / hmeta[n];  // exact: powers of two
        const float4 a = *reinterpret_cast<const float4*>(H + n * in + k0);
        const float4 b = *reinterpret_cast<const float4*>(H + n * in + k0 + 4);
        const float4 da = *reinterpret_cast<const float4*>(hmeta + k0);
        const float4 db = *reinterpret_cast<const float4*>(hmeta + k0 + 4);
        float v[8] = {a.x * rn / da.x, a.y * rn / da.y, a.z * rn / da.z, a.w * rn / da.w,
                      b.x * rn / db.x, b.y * rn / db.y, b.z * rn / db.z, b.w * rn / db.w};
#pragma unroll
        for (int e = 0; e < 8; ++e)
            if (k0 + e >= n) v[e] = 0.0f;
        __half2* h = reinterpret_cast<__half2*>(&o);
#pragma unroll
        for (int e = 0; e < 4; ++e) h[e] = __floats2half2_rn(v[2 * e], v[2 * e + 1]);
    }
    *reinterpret_cast<uint4*>(Hs + c * 8) = o;
}

template <int BT>
int run_gram(adadim_ctx* ctx, const __half* X, int64_t tokens, int64_t in, int64_t ldx, float* H, int accumulate,
             __half* Hs, float* hmeta) {
    const int nb = static_cast<int>((in + BT - 1) / BT);
    const int n_tiles = nb * (nb + 1) / 2;
    // The 128-wide kernel takes a grid of (tile, token split): about ceil(workgroups / 256) rounds of stages/n_split
    // stages each, while every split adds one partial tile per tile to write and to read back.  Take the split
    // count with the lowest estimate (unit: the time of one stage; a partial costs about a fifth of that per split
    // in traffic).  The 256-wide kernel's launch is planned by simulation (gram_plan.h); plans are kept per context.
    GramPlan plan;
    const GramOrder* order = nullptr;
    if constexpr (BT == 256) {
        int hit = -1;
        for (int k = 0; k < ctx->gram_split_n; ++k)
            if (ctx->gram_split[k].plan.tokens == tokens && ctx->gram_split[k].plan.n_tiles == n_tiles &&
                ctx->gram_split[k].whole_ok == (accumulate == 0))
                hit = k;
        if (hit < 0) {
            hit = ctx->gram_split_next;                             // the oldest entry makes room
            ctx->gram_split[hit].plan = gram_plan_choose(tokens, n_tiles, accumulate == 0);
            gram_plan_order(ctx->gram_split[hit].plan, ctx->gram_split[hit].order);
            ctx->gram_split[hit].whole_ok = accumulate == 0;
            ctx->gram_split_next = (hit + 1) % 8;
            if (ctx->gram_split_n < 8) ++ctx->gram_split_n;
        }
        plan = ctx->gram_split[hit].plan;
        order = &ctx->gram_split[hit].order;
    } else {
        const int64_t stages = (tokens + KT - 1) / KT;
        int n_split = 1;
        double best_cost = 0.0;
        for (int n = 1; n <= 32 && n <= stages; ++n) {
            const int64_t per = (stages + n - 1) / n;
            const int64_t rounds = (int64_t(n_tiles) * n + 255) / 256;
            const double cost = double(rounds) * double(per) + 0.19 * double(n) * double(n_tiles) * (BT * BT / 65536.0);
            if (n == 1 || cost < best_cost) {
                best_cost = cost;
                n_split = n;
            }
        }
        const int64_t t_per_split = ((stages + n_split - 1) / n_split) * KT;
        plan = {n_tiles, 0, static_cast<int>(tokens / t_per_split), 0, 1, tokens, t_per_split, KT};
    }
    const int n_whole = plan.n_whole, n_rest = n_tiles - n_whole;
    const size_t part_bytes = std::max<size_t>(256, size_t(gram_plan_slots(plan)) * BT * BT * sizeof(float));
    float* part = static_cast<float*>(adadim_workspace(ctx, WS_HESS_PART, part_bytes));
    if (!part) return ADADIM_EHIP;

    if constexpr (BT == 256) {
        // zero-filled source for rows past the end of the token range: the DMA of a surplus stage
        // reads up to 32 token rows of pitch ldx from it
        const size_t zero_bytes = size_t(32) * size_t(ldx) * 2 + 512;
        void* zero16 = adadim_workspace(ctx, WS_ZERO, zero_bytes);
        if (!zero16) return ADADIM_EHIP;
        static PerDeviceOnce once;
        ADADIM_HIP_TRY(ctx, once.run([] {
            return hipFuncSetAttribute(reinterpret_cast<const void*>(dma::gram_tiles_dma<2, 2>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, dma::SMEM_BYTES);
        }));
        if (ctx->zero_ready_bytes != ctx->ws_bytes[WS_ZERO]) {
            const int64_t n = static_cast<int64_t>(ctx->ws_bytes[WS_ZERO] / 4);
            hipLaunchKernelGGL(zero_f32, dim3(static_cast<unsigned>((n + 255) / 256)), dim3(256), 0, ctx->stream,
                               static_cast<float*>(zero16), n);
            ADADIM_LAUNCH_CHECK(ctx, "zero_f32");
            ctx->zero_ready_bytes = ctx->ws_bytes[WS_ZERO];
        }
        {
            ProfScope prof(ctx, "gram_tiles");
            // 32 workgroups per XCD walking their own items, or one workgroup per item where there is no order
            const unsigned grid = 8u * static_cast<unsigned>(order->n ? 32 : gram_plan_per_xcd(plan));
            hipLaunchKernelGGL((dma::gram_tiles_dma<2, 2>), dim3(grid), dim3(256), dma::SMEM_BYTES, ctx->stream, X, in,
                               ldx, nb, plan, *order, zero16, part, H);
        }
        ADADIM_LAUNCH_CHECK(ctx, "gram_tiles");
    } else {
        constexpr int smem = 4 * BT * ROW_BYTES;
        static PerDeviceOnce once;
        ADADIM_HIP_TRY(ctx, once.run([] {
            return hipFuncSetAttribute(reinterpret_cast<const void*>(gram_tiles<BT>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, smem);
        }));
        {
            ProfScope prof(ctx, "gram_tiles");
            const int n_split = plan.n_full + (gram_plan_has_rem(plan) ? 1 : 0);   // partial [split][tile]: the plan's slots
            hipLaunchKernelGGL(gram_tiles<BT>, dim3(n_tiles, n_split), dim3(THREADS), smem, ctx->stream, X, tokens,
                               in, ldx, nb, plan.t_per_split, part);
        }
        ADADIM_LAUNCH_CHECK(ctx, "gram_tiles");
    }
    constexpr int SB = BT / 32;
    int whole_diag = 0;                                       // diagonal tiles among the whole ones
    while (Hs && whole_diag < nb && diag_tile_index(whole_diag, nb) < n_whole) ++whole_diag;
    const unsigned reduce_tiles = static_cast<unsigned>(n_rest + whole_diag);
    if (reduce_tiles > 0) {
        ProfScope prof(ctx, "gram_reduce");
        if (Hs)
            hipLaunchKernelGGL((gram_reduce<BT, BT == 256, true>), dim3(SB * SB * reduce_tiles), dim3(256), 0, ctx->stream,
                               part, plan, nb, in, H, 0, Hs, hmeta);
        else
            hipLaunchKernelGGL((gram_reduce<BT, BT == 256, false>), dim3(SB * SB * reduce_tiles), dim3(256), 0, ctx->stream,
                               part, plan, nb, in, H, accumulate, Hs, hmeta);
    }
    ADADIM_LAUNCH_CHECK(ctx, "gram_reduce");
    if (Hs && n_whole > 0) {
        {
            ProfScope prof(ctx, "gram_prep_whole");
            hipLaunchKernelGGL(gram_prep_whole, dim3(8u * static_cast<unsigned>(n_whole)), dim3(256), 0, ctx->stream, H, nb, in, hmeta,
                               Hs);
        }
        ADADIM_LAUNCH_CHECK(ctx, "gram_prep_whole");
    }
    return ADADIM_OK;
}

}  // namespace

int launch_hessian(adadim_ctx* ctx, const __half* X, int64_t tokens, int64_t in, int64_t ldx, float* H,
                   int accumulate) {
    if (tokens == 0) {
        if (!accumulate) {
            const int64_t n = in * in;
            {
                ProfScope prof(ctx, "zero_f32");
                hipLaunchKernelGGL(zero_f32, dim3(static_cast<unsigned>((n + 255) / 256)), dim3(256), 0, ctx->stream,
                                   H, n);
            }
            ADADIM_LAUNCH_CHECK(ctx, "zero_f32");
        }
        return ADADIM_OK;
    }
    if (in <= 1024) return run_gram<128>(ctx, X, tokens, in, ldx, H, accumulate, nullptr, nullptr);
    return run_gram<256>(ctx, X, tokens, in, ldx, H, accumulate, nullptr, nullptr);
}

// H = X^T X together with its prepared form (see gram_reduce, PREP)
int launch_hessian_prepared(adadim_ctx* ctx, const __half* X, int64_t tokens, int64_t in, int64_t ldx, float* H,
                            __half* Hs, float* hmeta) {
    if (tokens == 0) {
        const int rc = launch_hessian(ctx, X, tokens, in, ldx, H, 0);
        return rc != ADADIM_OK ? rc : launch_hessian_prepare(ctx, H, in, Hs, hmeta);
    }
    if (in <= 1024) return run_gram<128>(ctx, X, tokens, in, ldx, H, 0, Hs, hmeta);
    return run_gram<256>(ctx, X, tokens, in, ldx, H, 0, Hs, hmeta);
}

// Measurement aid: one launch of the 256-wide tile kernel built with time stamps around every piece.
extern "C" int adadim_probe_gram_timeline(adadim_ctx* ctx, const void* X, int64_t tokens, int64_t in, int64_t ldx,
                                          int dispatcher, float* records, int cap, int* n_records, int* plan_out) {
    if (!ctx) return ADADIM_ENULL;
    if (!X || !records || !n_records || !plan_out)
        return adadim_fail(ctx, ADADIM_ENULL, "adadim_probe_gram_timeline: NULL argument");
    if (tokens <= 0 || tokens > (int64_t(1) << 24) || in <= 1024 || in > (int64_t(1) << 16) || ldx < in ||
        (dispatcher != 0 && dispatcher != 1))
        return adadim_fail(ctx, ADADIM_EINVAL, "adadim_probe_gram_timeline: need 0 < tokens <= 2^24, 1024 < in <= 65536 "
                                               "(the 256-wide kernel), ldx >= in, dispatcher 0 or 1");
    if ((in % 8) != 0 || (ldx % 8) != 0 || !aligned16(X))
        return adadim_fail(ctx, ADADIM_EALIGN, "adadim_probe_gram_timeline: in and ldx multiples of 8, X 16-byte aligned");
    if (ctx->capturing)
        return adadim_fail(ctx, ADADIM_EINVAL, "adadim_probe_gram_timeline: not while a graph is being recorded");
    constexpr int BT = 256;
    const int nb = static_cast<int>((in + BT - 1) / BT), n_tiles = nb * (nb + 1) / 2;
    const GramPlan plan = gram_plan_choose(tokens, n_tiles, false);   // no whole tiles: they carry no time stamps
    GramOrder order;
    gram_plan_order(plan, order);
    if (dispatcher) order.n = 0;
    const int slots = gram_plan_slots(plan);
    *n_records = slots;
    plan_out[0] = plan.n_tiles; plan_out[1] = plan.n_full; plan_out[2] = static_cast<int>(plan.t_per_split / GRAM_STAGE);
    plan_out[3] = plan.n_cut; plan_out[4] = plan.m; plan_out[5] = static_cast<int>(plan.t_sub / GRAM_STAGE);
    plan_out[6] = order.n ? 1 : 0; plan_out[7] = gram_plan_per_xcd(plan);
    if (cap < slots)
        return adadim_fail(ctx, ADADIM_EINVAL, "adadim_probe_gram_timeline: %d records needed, room for %d", slots, cap);
    float* part = static_cast<float*>(adadim_workspace(ctx, WS_HESS_PART, size_t(slots) * BT * BT * sizeof(float)));
    void* zero16 = adadim_workspace(ctx, WS_ZERO, size_t(32) * size_t(ldx) * 2 + 512);
    if (!part || !zero16) return ADADIM_EHIP;
    if (ctx->zero_ready_bytes != ctx->ws_bytes[WS_ZERO]) {
        const int64_t n = static_cast<int64_t>(ctx->ws_bytes[WS_ZERO] / 4);
        hipLaunchKernelGGL(zero_f32, dim3(static_cast<unsigned>((n + 255) / 256)), dim3(256), 0, ctx->stream,
                           static_cast<float*>(zero16), n);
        ADADIM_LAUNCH_CHECK(ctx, "zero_f32");
        ctx->zero_ready_bytes = ctx->ws_bytes[WS_ZERO];
    }
    static PerDeviceOnce once;
    ADADIM_HIP_TRY(ctx, once.run([] {
        return hipFuncSetAttribute(reinterpret_cast<const void*>(dma::gram_tiles_dma<2, 2, 8>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, dma::SMEM_BYTES);
    }));
    const unsigned grid = 8u * static_cast<unsigned>(order.n ? 32 : gram_plan_per_xcd(plan));
    for (int rep = 0; rep < 3; ++rep) {                       // the last launch is the one read back
        hipLaunchKernelGGL((dma::gram_tiles_dma<2, 2, 8>), dim3(grid), dim3(256), dma::SMEM_BYTES, ctx->stream,
                           static_cast<const __half*>(X), in, ldx, nb, plan, order, zero16, part,
                           static_cast<float*>(nullptr));
        ADADIM_LAUNCH_CHECK(ctx, "gram_tiles (time stamps)");
    }
    ADADIM_HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    // a piece leaves its stamps in the first 16 bytes of its partial tile and 4 KB further on
    std::vector<float> head(size_t(slots) * 4), phase(size_t(slots) * 4);
    const size_t pitch = size_t(BT) * BT * sizeof(float);
    ADADIM_HIP_TRY(ctx, hipMemcpy2D(head.data(), 16, part, pitch, 16, slots, hipMemcpyDeviceToHost));
    ADADIM_HIP_TRY(ctx, hipMemcpy2D(phase.data(), 16, part + 1024, pitch, 16, slots, hipMemcpyDeviceToHost));
    uint32_t t0 = 0;
    for (int i = 0; i < slots; ++i) {
        uint32_t st;
        std::memcpy(&st, &head[size_t(i) * 4 + 2], 4);
        if (i == 0 || static_cast<int32_t>(st - t0) < 0) t0 = st;
    }
    const int n_big = gram_plan_big(plan), n_small = gram_plan_small(plan), n_sub = gram_plan_sub(plan);
    auto xcd_of = [](int n, int i) {                          // the XCD whose share of an n-item list holds item i
        int x = 0;
        while (x < 7 && gram_plan_share_begin(n, x + 1) <= i) ++x;
        return x;
    };
    for (int i = 0; i < slots; ++i) {
        uint32_t st, en;
        std::memcpy(&st, &head[size_t(i) * 4 + 2], 4);
        std::memcpy(&en, &head[size_t(i) * 4 + 3], 4);
        const int cls = i < n_big ? 0 : i < n_big + n_small ? 1 : 2;
        const int xcd = cls == 0 ? xcd_of(n_big, i) : cls == 1 ? xcd_of(n_small, i - n_big) : xcd_of(n_sub, i - n_big - n_small);
        float* r = records + size_t(i) * 8;
        r[0] = static_cast<float>(cls);
        r[1] = static_cast<float>(xcd);
        r[2] = static_cast<float>(st - t0) / 100.0f;            // 100 MHz ticks -> us
        r[3] = static_cast<float>(en - t0) / 100.0f;
        r[4] = head[size_t(i) * 4];                            // shader cycles
        r[5] = phase[size_t(i) * 4] / 100.0f;                  // prologue
        r[6] = phase[size_t(i) * 4 + 1] / 100.0f;              // main loop
        r[7] = 0.0f;
    }
    (void)n_sub;
    return ADADIM_OK;
}

int launch_hessian_prepare(adadim_ctx* ctx, const float* H, int64_t in, __half* Hs, float* hmeta) {
    {
        ProfScope prof(ctx, "hprep_meta");
        hipLaunchKernelGGL(hprep_meta, dim3(static_cast<unsigned>((in + 255) / 256)), dim3(256), 0, ctx->stream, H,
                           in, hmeta);
    }
    ADADIM_LAUNCH_CHECK(ctx, "hprep_meta");
    const int64_t chunks = score_elems(in, in) / 8;
    {
        ProfScope prof(ctx, "hprep_scale");
        hipLaunchKernelGGL(hprep_scale, dim3(static_cast<unsigned>((chunks + 255) / 256)), dim3(256), 0, ctx->stream,
                           H, in, hmeta, Hs);
    }
    ADADIM_LAUNCH_CHECK(ctx, "hprep_scale");
    return ADADIM_OK;
}
