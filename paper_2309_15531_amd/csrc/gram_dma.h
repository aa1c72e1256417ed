// Gram-matrix tile kernel with LDS-DMA staging (gfx950).  Included by hessian.hip.
#pragma once

#include "gram_plan.h"
#include "mfma_tile.h"

#include <type_traits>

namespace {

using namespace mfma;

// ---------------------------------------------------------------------------
// 256x256 tiles with LDS-DMA staging.  X is copied global -> LDS without
// passing through registers (global_load_lds_dwordx4, 1 KB per wavefront
// instruction = two token rows of 256 columns) into a ring of four 32-token
// stages, and the MFMA fragments are fetched with the transposing LDS read
// (ds_read_b64_tr_b16), which turns the token-major tile into the
// contraction-contiguous operand layout on the fly.
//
// LDS stage layout: operand A (row panel I) then operand B (column panel J),
// each [32 tokens][256 columns] fp16, 512 bytes per token row.  The 16-byte
// chunk c of token row r is stored at chunk slot c ^ ((r & 3) << 2): the four
// token rows that one transposing read touches then fall into different
// 64-byte bank groups.  The permutation is applied on the global side (the
// LDS side of a DMA transfer is always lane-linear).
//
// ds_read_b64_tr_b16: within each block of 16 lanes, lane i receives the four
// 16-bit elements {i, 16+i, 32+i, 48+i} of the 64 elements the block's lanes
// address (lane L contributing elements 4L..4L+3).  Lane L therefore points at
// token row L/4, columns 4*(L%4)..+3 of a 4-token x 16-column patch and lane i
// ends up with column i of the patch for the four tokens.
//
// Pipeline per 32-token stage s (two 16-token MFMA sweeps, fragments double
// buffered in registers):  sweep 0 with the reads of sweep 1 spread between its
// MFMAs | a quarter of sweep 1 | wait for stage s+1's DMA, barrier | rest of
// sweep 1 with, spread between its MFMAs, the DMA of stage s+3 (into the buffer
// stage s-1 used) and the reads of stage s+1's first fragments.  Instruction
// order is pinned with sched_barrier: a burst of DMA or LDS instructions
// stalls the wave's in-order issue and starves the matrix pipe.
namespace dma {

constexpr int BT = 256, KT = 32, NST = 4;
static_assert(KT == GRAM_STAGE, "the plan counts in stages of this kernel");
constexpr int ROWB = BT * 2;
constexpr int OP_BYTES = KT * ROWB;
constexpr int STAGE_BYTES = 2 * OP_BYTES;
constexpr int SMEM_BYTES = NST * STAGE_BYTES;

typedef short short4v __attribute__((ext_vector_type(4)));
typedef short short8v __attribute__((ext_vector_type(8)));

__device__ __forceinline__ void g2l16(const void* g, uint32_t lds) {
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds), "v"(g) : "memory", "m0");
}

// Same transfer with a scalar base address plus a per-lane unsigned 32-bit byte offset.
__device__ __forceinline__ void g2l16_s(const void* sbase, uint32_t voff, uint32_t lds) {
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds), "v"(voff), "s"(sbase)
                 : "memory", "m0");
}

__device__ __forceinline__ half8 tr_read8(uint32_t addr) {
    typedef short4v __attribute__((address_space(3))) * lds_ptr;
    const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(reinterpret_cast<lds_ptr>(uintptr_t(addr)));
    const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(reinterpret_cast<lds_ptr>(uintptr_t(addr + 4 * ROWB)));
    const short8v v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(half8, v);
}

__device__ __forceinline__ short4v tr_read4(uint32_t addr) {
    typedef short4v __attribute__((address_space(3))) * lds_ptr;
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16(reinterpret_cast<lds_ptr>(uintptr_t(addr)));
}

// Fragments of one 16-token sweep, held as the two 4-token halves each
// transposing read delivers.
template <int TM, int TN>
struct Frags {
    short4v lo[TM + TN];
    short4v hi[TM + TN];
    __device__ __forceinline__ half8 get(int k) const {
        const short8v v = __builtin_shufflevector(lo[k], hi[k], 0, 1, 2, 3, 4, 5, 6, 7);
        return __builtin_bit_cast(half8, v);
    }
};

template <int WGM, int WGN, int DBG = 0>
__global__ __launch_bounds__(64 * WGM * WGN) void gram_tiles_dma(const __half* __restrict__ X, int64_t in,
                                                                 int64_t ldx, int nb, GramPlan plan,
                                                                 GramOrder order, const void* zero16,
                                                                 float* __restrict__ part, float* __restrict__ H) {
    constexpr int NW = WGM * WGN;
    constexpr int WM = BT / WGM, WN = BT / WGN, TM = WM / 32, TN = WN / 32;
    constexpr int LOADS = 32 / NW;  // 1-KB transfers per wavefront per stage
    static_assert(32 % NW == 0, "wavefront count");
    extern __shared__ __align__(16) char smem[];
    const uint32_t lds0 = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(smem));

    // Work items of this workgroup (see gram_plan.h): whole tiles over all tokens, stored straight into H, both
    // halves, and pieces of a tile's token range, each written as an fp32 partial tile that gram_reduce adds up.
    // Workgroups are handed to the eight XCDs round-robin by launch index, and each XCD has its own L2.  With an
    // order the launch has 32 workgroups per XCD and workgroup c walks its own places of the XCD's lists; without,
    // every place has a workgroup of its own.
    const int xcd = static_cast<int>(blockIdx.x % 8), unit = static_cast<int>(blockIdx.x / 8);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WGN, wn = wave % WGN;
    const int i_begin = order.n ? (unit < 32 ? order.first[unit] : 0) : unit;
    const int i_end = order.n ? (unit < 32 ? order.first[unit + 1] : 0) : unit + 1;
#pragma unroll 1
    for (int i_place = i_begin; i_place < i_end; ++i_place) {
        GramItem it;
        if (!gram_plan_item(plan, xcd, order.n ? int(order.pos[i_place]) : i_place, it)) continue;
        const bool whole = it.slot < 0;                          // the same for the whole workgroup
        int I, J;
        decode_tile(it.tile, nb, I, J);
        const int64_t t_begin = it.t_begin, t_end = it.t_end;
        const int t_len = static_cast<int>(t_end - t_begin);
        const int n_st = t_len > 0 ? (t_len + KT - 1) / KT : 1;  // an empty range still runs one all-zero stage

        long long dbg_c0 = 0, dbg_w0 = 0;
        if constexpr (DBG & 8) {
            dbg_c0 = clock64();
            dbg_w0 = wall_clock64();
        }

        // ---- DMA descriptors: transfer j of this wavefront moves token rows 2*rp, 2*rp+1 of operand op.
        // The token range is cut so that the FIRST stage takes the ragged remainder (r0 rows, the
        // rest of its rows read a page of zeros through per-lane predicates, outside the main loop)
        // and every later stage is a full 32 tokens.  Those are fetched with a scalar base that
        // advances once per stage plus a constant per-lane offset: one VALU op per transfer.
        // Stages past the end are still issued, from a zero-filled buffer (`zero16`, at least
        // 32*ldx*2 + 512 bytes), so that the vmcnt bookkeeping stays uniform.  Lanes whose columns fall outside H
        // re-read column block 0 of the panel:
        // their products only reach rows/columns of the tile that are never stored.
        const int r0 = t_len - KT * (n_st - 1);   // rows of stage 0: 1..32 (0 for an empty range)
        const int rl = lane >> 5, p = lane & 31;
        uint32_t goff[LOADS];   // byte offset of this lane's 16 bytes from the stage's first token row
        uint32_t gdst[LOADS];
#pragma unroll
        for (int j = 0; j < LOADS; ++j) {
            const int q = wave + NW * j;
            const int op = q >> 4, rp = q & 15;
            const int row = 2 * rp + rl;
            const int c = p ^ ((row & 3) << 2);
            int64_t col = int64_t(op ? J : I) * BT + 8 * c;
            if (col >= in) col = int64_t(op ? J : I) * BT;
            goff[j] = static_cast<uint32_t>((int64_t(row) * ldx + col) * 2);
            gdst[j] = lds0 + op * OP_BYTES + rp * 1024;
            // stage 0, predicated
            const void* g = row < r0 ? static_cast<const void*>(X + (t_begin + row) * ldx + col) : zero16;
            g2l16(g, gdst[j]);
        }
        const char* sbase = reinterpret_cast<const char*>(X + (t_begin + r0) * ldx);  // next stage to issue
        const int64_t stage_bytes = int64_t(KT) * ldx * 2;
        int issued = 1;  // stages whose DMA has been started
        const char* cur_base = sbase;
        auto stage_begin = [&]() {   // wave-uniform base of the stage about to be issued
            const uintptr_t b = reinterpret_cast<uintptr_t>(issued < n_st ? sbase : static_cast<const char*>(zero16));
            const uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(b));
            const uint32_t hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(b >> 32));
            cur_base = reinterpret_cast<const char*>((uintptr_t(hi) << 32) | lo);
        };
        // buf = ring slot of the stage being issued (issued & 3), a compile-time constant in the main loop
        auto issue_one = [&](int j, int buf) { g2l16_s(cur_base, goff[j], gdst[j] + buf * STAGE_BYTES); };
        auto stage_issued = [&]() {
            ++issued;
            sbase += stage_bytes;
        };
        auto issue_stage = [&](int buf) {
            stage_begin();
#pragma unroll
            for (int j = 0; j < LOADS; ++j) issue_one(j, buf);
            stage_issued();
        };

        // ---- fragment addresses (stage-relative, first sweep); index k < TM: A block k, else B block k-TM
        const int f = ((lane & 15) >> 2) << 2;
        const int lrow = 8 * (lane >> 5) + ((lane & 15) >> 2);
        const int mlow = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
        uint32_t f_off[TM + TN];
#pragma unroll
        for (int i = 0; i < TM; ++i)
            f_off[i] = lds0 + lrow * ROWB + ((((wm * WM) / 8 + 4 * i + (mlow >> 3)) ^ f) << 4) + (mlow & 7) * 2;
#pragma unroll
        for (int j = 0; j < TN; ++j)
            f_off[TM + j] =
                lds0 + OP_BYTES + lrow * ROWB + ((((wn * WN) / 8 + 4 * j + (mlow >> 3)) ^ f) << 4) + (mlow & 7) * 2;

        // one transposing read: half h (0: tokens +0..3, 1: tokens +4..7) of fragment k
        // `buf` is the ring slot (a compile-time constant in the main loop, so that the whole offset
        // folds into the instruction's immediate; slots 2 and 3 lie beyond its 64 KB reach and use a
        // second base register)
        uint32_t f_off_hi[TM + TN];
#pragma unroll
        for (int k = 0; k < TM + TN; ++k) {
            f_off_hi[k] = f_off[k] + 2 * STAGE_BYTES;
            asm("" : "+v"(f_off_hi[k]));  // keep it in a register: the sum does not fit an immediate
        }
        auto read_half = [&](Frags<TM, TN>& F, int buf, int sweep_id, int k, int h) {
            const uint32_t off = (buf & 1) * STAGE_BYTES + sweep_id * 16 * ROWB + h * 4 * ROWB;
            const uint32_t base = (buf & 2) ? f_off_hi[k] : f_off[k];
            if (h == 0) F.lo[k] = tr_read4(base + off);
            else F.hi[k] = tr_read4(base + off);
        };
        auto read_frags = [&](Frags<TM, TN>& F, int buf, int sweep_id) {
#pragma unroll
            for (int k = 0; k < TM + TN; ++k) {
                read_half(F, buf, sweep_id, k, 0);
                read_half(F, buf, sweep_id, k, 1);
            }
        };

        floatx16 acc[TM][TN];
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

        constexpr int NMMA = TM * TN;            // MFMAs per sweep
        constexpr int NRD = 2 * (TM + TN);       // transposing reads per sweep
        auto mma = [&](const Frags<TM, TN>& F, int m) {
            const int i = m / TN, j = m % TN;
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(F.get(i), F.get(TM + j), acc[i][j], 0, 0, 0);
        };

        Frags<TM, TN> F0, F1;
        issue_stage(1);
        issue_stage(2);
        // stage 0 landed (two later stages may still be in flight)
        if constexpr (LOADS == 8) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
        else asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        read_frags(F0, 0, 0);
        // MFMAs issued before the mid-stage barrier, so that the matrix pipe has work while waves meet
        constexpr int PRE = NMMA / 4;
        // One stage with ring slot B known at compile time.
        auto stage_body = [&](auto buf_tag) {
            constexpr int B = decltype(buf_tag)::value;
            // sweep 0: MFMAs on F0, the reads of sweep 1 spread between them
#pragma unroll
            for (int m = 0; m < NMMA; ++m) {
                if constexpr (!(DBG & 4)) {
#pragma unroll
                    for (int r = m * NRD / NMMA; r < (m + 1) * NRD / NMMA; ++r) read_half(F1, B, 1, r >> 1, r & 1);
                }
                mma(F0, m);
                __builtin_amdgcn_sched_barrier(0);
            }
            // sweep 1: a few MFMAs, then the stage hand-over, then the rest with DMA and prefetch in between
#pragma unroll
            for (int m = 0; m < PRE; ++m) mma(F1, m);
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (!(DBG & 1)) {
                if constexpr (LOADS == 8) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
                else asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
                __builtin_amdgcn_s_barrier();
            }
            __builtin_amdgcn_sched_barrier(0);
            stage_begin();
#pragma unroll
            for (int m = PRE; m < NMMA; ++m) {
                constexpr int REST = NMMA - PRE;
                const int q = m - PRE;
                if constexpr (!(DBG & 4)) {
#pragma unroll
                    for (int r = q * NRD / REST; r < (q + 1) * NRD / REST; ++r)
                        read_half(F0, (B + 1) & 3, 0, r >> 1, r & 1);
                }
                if constexpr (!(DBG & 2)) {
#pragma unroll
                    for (int j = q * LOADS / REST; j < (q + 1) * LOADS / REST; ++j) issue_one(j, (B + 3) & 3);
                }
                mma(F1, m);
                __builtin_amdgcn_sched_barrier(0);
            }
            stage_issued();  // stage s+3 is on its way into the slot stage s-1 used
        };
        // Four stages per trip so that ring slots are constants; the up to three surplus stages at
        // the end multiply zeros.
        long long dbg_w1 = 0, dbg_w2 = 0;
        if constexpr (DBG & 8) dbg_w1 = wall_clock64();
        for (int s = 0; s < n_st; s += 4) {
            stage_body(std::integral_constant<int, 0>{});
            stage_body(std::integral_constant<int, 1>{});
            stage_body(std::integral_constant<int, 2>{});
            stage_body(std::integral_constant<int, 3>{});
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // no DMA may outlive the workgroup
        if constexpr (DBG & 8) dbg_w2 = wall_clock64();

        // The partial tile is stored in register order: float4 number ((i*TN + j)*4 + q)*256 + thread
        // holds accumulator registers 4q..4q+3 of block (i, j), so every store instruction writes one
        // contiguous kilobyte per wave; gram_reduce reads it back in the same order.
        static_assert(WGM == 2 && WGN == 2, "register-order partials assume 2 x 2 waves of 4 x 4 blocks");
        if (whole) {
            // Straight into H, one row of four 32x32 blocks per pass: the blocks go to a private LDS patch with
            // constant offsets (the only code that names accumulator registers), then a rolled loop stores each
            // block row by row (lanes 0..31 take 32 consecutive columns of one row: 128-byte pieces), its mirror
            // image below the diagonal from the turned patch, and a block on the diagonal with its lower half taken
            // from its upper half, so H is exactly symmetric.  Blocks below the diagonal of a diagonal tile are
            // their mirror images' business.
            __builtin_amdgcn_s_barrier();                    // every wave has read its last fragments: the ring is free
            float* sp = reinterpret_cast<float*>(smem) + wave * (TN * 32 * 33);
            const int half = lane >> 5, l32 = lane & 31;
            const int64_t Rw = int64_t(I) * BT + wm * WM, Cw = int64_t(J) * BT + wn * WN;
#pragma unroll
            for (int i = 0; i < TM; ++i) {
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r) sp[j * (32 * 33) + acc_row(r, lane) * 33 + l32] = acc[i][j][r];
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                const int64_t R0 = Rw + 32 * i;
#pragma unroll 1
                for (int j = 0; j < TN; ++j) {
                    const int64_t C0 = Cw + 32 * j;
                    if (R0 > C0 || R0 >= in || C0 >= in) continue;   // wave-uniform
                    const float* sb = sp + j * (32 * 33);
                    const bool dg = R0 == C0;
#pragma unroll 1
                    for (int pz = 0; pz < 16; ++pz) {
                        const int row = 2 * pz + half;
                        const float up = sb[row * 33 + l32], tr = sb[l32 * 33 + row];
                        const bool ok_u = R0 + row < in && C0 + l32 < in;
                        if (ok_u) H[(R0 + row) * in + C0 + l32] = (dg && l32 < row) ? tr : up;
                        if (!dg && C0 + row < in && R0 + l32 < in) H[(C0 + row) * in + R0 + l32] = tr;
                    }
                }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            }
        } else {
            float4* dst = reinterpret_cast<float4*>(part + int64_t(it.slot) * (int64_t(BT) * BT));
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        dst[((i * TN + j) * 4 + q) * 256 + tid] =
                            make_float4(acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
            if constexpr (DBG & 8) {
                if (tid == 0) {
                    dst[0].x = static_cast<float>(clock64() - dbg_c0);
                    dst[0].y = static_cast<float>(wall_clock64() - dbg_w0);
                    dst[0].z = __uint_as_float(static_cast<uint32_t>(dbg_w0));            // start, 100 MHz ticks
                    dst[0].w = __uint_as_float(static_cast<uint32_t>(wall_clock64()));   // end
                    dst[256].x = static_cast<float>(dbg_w1 - dbg_w0);                    // prologue ticks
                    dst[256].y = static_cast<float>(dbg_w2 - dbg_w1);                    // main loop ticks
                }
            }
        }
        // the next item's DMA reuses the ring (and the patches of the whole-tile stores): every wave must be past
        // its last LDS access, and this item's stores retired before the next one counts its DMA transfers in vmcnt
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
    }
}

}  // namespace dma

}  // namespace
