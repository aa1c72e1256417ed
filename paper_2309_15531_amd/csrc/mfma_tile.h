// Shared pieces of the two matrix-core kernels (Gram matrix and error GEMM):
// LDS tile layout, global->LDS staging with and without a transpose, and the
// per-stage MFMA sweep.  gfx950 only: v_mfma_f32_32x32x16_f16, 64-wide waves.
//
// LDS tile layout.  A tile holds ROWS rows (the M or N index) of KT = 64 halfs
// (the contraction index), 128 bytes per row, no padding.  The row is cut into
// eight 16-byte chunks and chunk c of row r is stored at chunk slot
// c ^ ((r ^ (r >> 3)) & 7).  With that swizzle both access patterns are free of
// bank conflicts: a fragment read (32 consecutive rows, one chunk) and a staging
// write (rows 8 apart, one chunk) each touch all eight slots evenly.
//
// MFMA operand mapping (32x32x16, f16 in, f32 out).  Lane l supplies row
// (l & 31) of A and column (l & 31) of B, each with the 8 contraction elements
// of chunk-half (l >> 5); the contraction pairs element e of A's lane group
// with element e of B's same lane group, so any consistent assignment of the
// contraction index to (chunk, element) is correct.  Output register r of lane
// l is D[8*(r/4) + 4*(l>>5) + (r&3)][l & 31].
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>

#include <cstdint>

namespace mfma {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int KT = 64;            // contraction elements per LDS stage
constexpr int ROW_BYTES = 128;    // KT halfs
constexpr int THREADS = 256;      // 4 wavefronts per workgroup

__device__ __forceinline__ int lds_off(int row, int chunk) {
    return row * ROW_BYTES + (((chunk ^ row ^ (row >> 3)) & 7) << 4);
}

__device__ __forceinline__ int acc_row(int r, int lane) { return 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3); }

// Operand whose contraction index is contiguous in memory: element (row, k) at
// base[row*ld + k].  Rows >= n_rows and k >= k_end read as zero.
template <int ROWS>
struct DirectStage {
    static constexpr int N = ROWS * 8 / THREADS;
    static_assert(ROWS * 8 % THREADS == 0, "tile rows");
    uint4 r[N];

    __device__ __forceinline__ void load(const __half* __restrict__ base, int64_t ld, int64_t row0,
                                         int64_t n_rows, int64_t k0, int64_t k_end, int tid) {
#pragma unroll
        for (int p = 0; p < N; ++p) {
            const int idx = tid + THREADS * p;
            const int64_t row = row0 + (idx >> 3);
            const int64_t k = k0 + ((idx & 7) << 3);
            uint4 v = make_uint4(0, 0, 0, 0);
            if (row < n_rows && k < k_end) v = *reinterpret_cast<const uint4*>(base + row * ld + k);
            r[p] = v;
        }
    }
    __device__ __forceinline__ void store(char* lds, int tid) const {
#pragma unroll
        for (int p = 0; p < N; ++p) {
            const int idx = tid + THREADS * p;
            *reinterpret_cast<uint4*>(lds + lds_off(idx >> 3, idx & 7)) = r[p];
        }
    }
};

// Operand whose contraction index is the slow axis in memory: element (row, k)
// at base[k*ld + row] (the Gram matrix reads X[t, i] with k = t, row = i).
// Each thread loads an 8(k) x 8(row) block with eight 16-byte loads, transposes
// it in registers and writes eight 16-byte LDS chunks.
template <int ROWS>
struct TransposeStage {
    static constexpr int IB = ROWS / 8;                       // row blocks per tile
    static constexpr int BLOCKS = IB * (KT / 8);              // 8x8 blocks per tile
    static constexpr int N = (BLOCKS + THREADS - 1) / THREADS;
    uint4 r[N][8];

    __device__ __forceinline__ void load(const __half* __restrict__ base, int64_t ld, int64_t row0,
                                         int64_t n_rows, int64_t k0, int64_t k_end, int tid) {
#pragma unroll
        for (int p = 0; p < N; ++p) {
            const int b = tid + THREADS * p;
            const int ib = b % IB, tb = b / IB;
            const int64_t row = row0 + ib * 8;
            const bool row_ok = (BLOCKS % THREADS == 0 || b < BLOCKS) && row < n_rows;
#pragma unroll
            for (int rr = 0; rr < 8; ++rr) {
                const int64_t k = k0 + tb * 8 + rr;
                uint4 v = make_uint4(0, 0, 0, 0);
                if (row_ok && k < k_end) v = *reinterpret_cast<const uint4*>(base + k * ld + row);
                r[p][rr] = v;
            }
        }
    }
    __device__ __forceinline__ void store(char* lds, int tid) const {
#pragma unroll
        for (int p = 0; p < N; ++p) {
            const int b = tid + THREADS * p;
            if (BLOCKS % THREADS != 0 && b >= BLOCKS) continue;
            const int ib = b % IB, tb = b / IB;
            const uint32_t* in = reinterpret_cast<const uint32_t*>(&r[p][0]);  // in[rr*4 + d]
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                const int d = c >> 1;
                uint32_t o[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const uint32_t lo = in[(2 * q) * 4 + d], hi = in[(2 * q + 1) * 4 + d];
                    o[q] = (c & 1) ? ((lo >> 16) | (hi & 0xffff0000u)) : ((lo & 0xffffu) | (hi << 16));
                }
                *reinterpret_cast<uint4*>(lds + lds_off(ib * 8 + c, tb)) = make_uint4(o[0], o[1], o[2], o[3]);
            }
        }
    }
};

// Order of the upper-triangular tiles (I <= J) of an nb x nb tile grid: strips of four tile
// rows, each strip walked column by column.  Any 32 consecutive tiles then touch about 4 row
// panels and 8 column panels, so the workgroups that run together on one XCD share most of
// their operand panels in its L2 (a row-major walk would touch 17 panels for 16 tiles).
__device__ __forceinline__ void decode_tile(int idx, int nb, int& I, int& J) {
    int s = 0;
    for (;;) {
        const int rows = min(4, nb - 4 * s);                      // tile rows in this strip
        const int head = rows * (rows + 1) / 2;                   // its triangular first columns
        const int size = head + rows * max(0, nb - 4 * s - 4);    // then full columns of `rows` tiles
        if (idx < size) {
            if (idx < head) {
                int c = 0;
                while (idx >= c + 1) {                            // column c of the head holds c + 1 tiles
                    idx -= c + 1;
                    ++c;
                }
                J = 4 * s + c;
                I = 4 * s + idx;
            } else {
                const int q = idx - head;
                J = 4 * s + 4 + q / rows;
                I = 4 * s + q % rows;
            }
            return;
        }
        idx -= size;
        ++s;
    }
}

// One LDS stage of MFMAs for a wave tile of TM x TN 32x32 blocks whose first
// rows in the A and B tiles are a_row0 and b_row0.
template <int TM, int TN>
__device__ __forceinline__ void mma_stage(const char* ldsA, const char* ldsB, int a_row0, int b_row0, int lane,
                                          floatx16 (&acc)[TM][TN]) {
    const int lr = lane & 31, lh = lane >> 5;
#pragma unroll
    for (int ks = 0; ks < KT / 16; ++ks) {
        const int ch = 2 * ks + lh;
        half8 a[TM], b[TN];
#pragma unroll
        for (int i = 0; i < TM; ++i) a[i] = *reinterpret_cast<const half8*>(ldsA + lds_off(a_row0 + 32 * i + lr, ch));
#pragma unroll
        for (int j = 0; j < TN; ++j) b[j] = *reinterpret_cast<const half8*>(ldsB + lds_off(b_row0 + 32 * j + lr, ch));
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
}

}  // namespace mfma
