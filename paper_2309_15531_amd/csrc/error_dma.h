// Error-GEMM tile kernel with LDS-DMA staging (gfx950).  Included by layer_error.hip.
//
// Computes, for one 256x256 tile (row block mb of dW', column block nb of E)
// and one chunk of the contraction range, the partial row sums
//     part[slot, o] = sum_{n in block nb} ( sum_{k in chunk} dW'[o,k] Hs[n,k] ) * dW'[o,n]
// where Hs is the scaled strictly-lower triangle of H (zero for k >= n), so the
// contraction of column block nb stops at its diagonal block.  Row sums are
// linear in the contraction range, so chunks simply add up; cutting the long
// contractions of the right-hand column blocks into chunks is what balances the
// triangular work over the compute units.
//
// The MFMA's M index runs over the columns n of E (rows of Hs) and its N index
// over the rows o (rows of dW'): each lane then owns one output row o per
// 32-wide block and four consecutive n per accumulator quad, so the epilogue's
// dW'[o,n] factors are 8-byte loads and the sum over n stays inside the lane.
//
// Both operands are contraction-contiguous per row, so a DMA transfer
// (global_load_lds_dwordx4, 1 KB per wavefront instruction) brings 16 rows x
// 32 k and the MFMA fragments are plain 16-byte LDS reads.  In the scoring
// layout (common.h: 256-row tiles blocked by 32 along k when `in` is a multiple
// of 32) those 16 x 64 bytes are one contiguous kilobyte, i.e. eight whole
// 128-byte lines, and a tile's stages follow each other in memory;
// with row-major operands they would be sixteen half lines and the L2 request
// rate, not the matrix cores, would set the pace.  Stage layout:
// operand 0 (256 rows of Hs) then operand 1 (256 rows of dW'), each [256 rows][64 bytes];
// the 16-byte chunk c of row r sits at chunk slot c ^ ((r >> 2) & 3), which
// makes the fragment reads (32 consecutive rows, one chunk) conflict-free.  The
// permutation is applied on the global side of the transfer.
//
// The software pipeline is the one of the Gram kernel: a ring of four 32-k
// stages, two 16-k MFMA sweeps per stage with register double buffering, one
// barrier per stage, DMA and LDS reads interleaved with the MFMAs in a pinned
// order, the ragged remainder of the contraction range taken by the first
// stage through per-lane predicates.
//
// Epilogue inside the main loop.  The row sums need E[o,n] * dW'[o,n] for the n
// of the column block.  When the workgroup's contraction range ends with the
// block's own 256 k (the diagonal block of Hs: always, unless the contraction is
// cut into chunks), those dW' values pass through the ring as operand 1 of the
// last eight stages: stage i of the eight brings dW'[o, 32i .. 32i+31].  Hs is
// strictly lower triangular, so the accumulators of columns 32i .. 32i+31 are
// final once that stage's products are in (later stages add exact zeros).  The
// waves that own those columns therefore copy the stage's dW' entries from the
// ring into registers while the stage is computed and fold them into the row
// sums during the next stage, between its MFMAs.  No separate fetch of the
// 128 KB dW' tile, no pass over the accumulators after the loop: on 4096-wide
// layers, where a workgroup computes for 6 to 100 us, that fetch and pass were
// 8 to 10 us of every workgroup.  Workgroups whose range does not hold the
// diagonal block, row-major operands and ragged widths take the separate
// epilogue further down.
#pragma once

#include "common.h"
#include "mfma_tile.h"

#include <type_traits>

namespace {

using namespace mfma;

namespace edma {

constexpr int BT = 256, KT = 32, NST = 4;
constexpr int ROWB = KT * 2;               // 64 bytes per tile row per stage
constexpr int OP_BYTES = BT * ROWB;        // 16384
constexpr int STAGE_BYTES = 2 * OP_BYTES;
constexpr int SMEM_BYTES = NST * STAGE_BYTES;
constexpr int NW = 4, WM = 128, WN = 128, TM = 4, TN = 4, LOADS = 8;

__device__ __forceinline__ void g2l16(const void* g, uint32_t lds) {
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds), "v"(g) : "memory", "m0");
}
__device__ __forceinline__ void g2l16_s(const void* sbase, uint32_t voff, uint32_t lds) {
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds), "v"(voff), "s"(sbase)
                 : "memory", "m0");
}
__device__ __forceinline__ half8 lds_read8(uint32_t addr) {
    typedef half8 __attribute__((address_space(3))) * lds_ptr;
    return *reinterpret_cast<lds_ptr>(uintptr_t(addr));
}

typedef uint32_t uint2v __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint2 lds_read_u2(uint32_t addr) {
    typedef uint2v __attribute__((address_space(3))) * lds_ptr;
    const uint2v v = *reinterpret_cast<lds_ptr>(uintptr_t(addr));
    return make_uint2(v.x, v.y);
}

struct Frags {
    half8 v[TM + TN];
};

// fma(half HI of a packed fp16 pair, b, c): the conversion rides on the instruction (v_fma_mix_f32)
typedef _Float16 f16x2v __attribute__((ext_vector_type(2)));
template <int HI>
__device__ __forceinline__ float fma_h(uint32_t pair, float b, float c) {
    return __builtin_fmaf(static_cast<float>(__builtin_bit_cast(f16x2v, pair)[HI]), b, c);
}

// Candidates scored by one launch: their (column-scaled fp16) dW matrices share H.
constexpr int MAX_BATCH = 8;
struct Batch {
    const __half* A[MAX_BATCH];
    int n;
};

// Column block nb contracts over k < kend(nb) = min(in, (nb+1)*256), cut into
// chunks of kc_len (a multiple of 256).  Slots enumerate (chunk, nb): chunk
// ascending, nb descending over the column blocks that reach the chunk.
// One work item: position `seq` in the list of XCD `xcd` (see below).  Returns 0 after computing the item, 1 for a
// padding position inside the list, 2 when the list of that XCD is exhausted (so is every later position).
// rec: index of the item's timeline record (DBG 8).
template <int DBG>
__device__ __forceinline__ int error_item(const Batch& batch, const __half* __restrict__ Hs, int64_t out, int64_t in,
                                          int MB, int NB, int kc_len, int n_slots, const void* zero16,
                                          const float* __restrict__ hmeta_diag, float* __restrict__ part, int xcd, int seq,
                                          int64_t rec, char* smem) {
    __shared__ float s_rows[2][BT];   // [wm][output row within the tile]
    __shared__ __align__(16) float s_hd[2][BT];   // in-loop epilogue: column scales d and diag(H) of the block's columns ...
    __shared__ __align__(16) float s_hq[BT];      // ... and H_nn / d_n^2 / 2 (0 when this workgroup does not add the diagonal term)
    const uint32_t lds0 = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(smem));

    // Workgroups go to the eight XCDs round-robin by launch index, and a compute unit holds one
    // workgroup, so 32 consecutive workgroups of an XCD run together and share its L2.  They are
    // made a unit of 4 slots x 8 row blocks: per pipeline stage the unit then fetches 4 Hs tiles
    // and 8 dW' tiles instead of the 33 tiles that 32 row blocks of one slot would need (the dW'
    // tiles, re-read for every column block, are what would otherwise saturate the memory
    // fabric).  Slots are listed chunk by chunk, column blocks descending inside a chunk, so the
    // slots of a unit cover the same contraction range; units are dealt to the XCDs in serpentine
    // order (0..7, 7..0, ...), which evens out the totals, slot group by slot group, so that
    // neighbouring XCDs work on the same Hs tiles at the same time.
    const int n_pairs = batch.n * MB;                        // (candidate, row block) pairs
    const int n_rs = (n_pairs + 7) / 8, n_sg = (n_slots + 3) / 4;
    const int round = seq / 32, within = seq % 32;
    const int unit = round * 8 + ((round & 1) ? 7 - xcd : xcd);
    if (unit >= n_sg * n_rs) return 2;
    // (workgroup-uniform values: kept in scalar registers, where there is room)
    const int slot = __builtin_amdgcn_readfirstlane((unit / n_rs) * 4 + (within & 3));
    const int pair = __builtin_amdgcn_readfirstlane((unit % n_rs) * 8 + (within >> 2));
    if (slot >= n_slots || pair >= n_pairs) return 1;
    const int cand = __builtin_amdgcn_readfirstlane(pair / MB), mb = __builtin_amdgcn_readfirstlane(pair % MB);
    const __half* __restrict__ A = batch.A[cand];
    const int kb = kc_len / BT;
    int chunk = 0, rem = slot;
    for (;;) {
        const int cnt = NB - chunk * kb;                     // column blocks that reach this chunk
        if (rem < cnt) break;
        rem -= cnt;
        ++chunk;
    }
    const int nb = NB - 1 - rem;
    const int64_t kend = (DBG & 1) ? in : min(in, int64_t(nb + 1) * BT);   // DBG 1: dense timing probe
    const int64_t k_begin = int64_t(chunk) * kc_len;
    const int k_len = static_cast<int>(min(kend, k_begin + kc_len) - k_begin);   // > 0, multiple of 8
    const int n_st = (k_len + KT - 1) / KT;
    const int r0 = k_len - KT * (n_st - 1);                                       // k of stage 0: 8..32
    const int64_t row0 = int64_t(mb) * BT, col0 = int64_t(nb) * BT;

    // DBG 8: four 100 MHz timestamps per workgroup (entry, main loop begin and end, exit) behind the
    // partial sums, for the timeline probe
    long long dbg_t[4] = {0, 0, 0, 0};
    if constexpr (DBG & 8) dbg_t[0] = wall_clock64();
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;

    // ---- DMA descriptors.  Transfer j of this wavefront moves rows 16*rq .. 16*rq+15 of operand op
    // (q = wave + 4j: op = q >> 4, rq = q & 15; operand 0 = Hs rows of column block nb, operand 1 =
    // dW' rows of row block mb); lane l takes row l >> 2, chunk slot l & 3.  Rows past the end of a
    // matrix re-read the block's first row: they only feed entries of E that the epilogue skips.
    const int lr = lane >> 2, p = lane & 3;
    const bool blocked = score_blocked(in);
    // in-loop epilogue (see the head of the file): the contraction range ends with the column block's own 256 k
    const bool fused = !(DBG & 1) && blocked && (in % BT) == 0 && k_begin <= col0 && col0 < k_begin + kc_len;
    const bool add_diag = hmeta_diag != nullptr && chunk == 0;
    if (fused && add_diag && wave == 0) {
        // column scales and diag(H) of the block's 256 columns, 1 KB each, straight into LDS; issued before the
        // first stage so that the wait for that stage covers them
        g2l16(hmeta_diag + col0 + 4 * lane, static_cast<uint32_t>(reinterpret_cast<uintptr_t>(&s_hd[0][0])));
        g2l16(hmeta_diag + in + col0 + 4 * lane, static_cast<uint32_t>(reinterpret_cast<uintptr_t>(&s_hd[1][0])));
    }
    uint32_t goff[LOADS], gdst[LOADS];
#pragma unroll
    for (int j = 0; j < LOADS; ++j) {
        const int q = wave + NW * j;
        const int op = q >> 4, rq = q & 15;
        const int row = 16 * rq + lr;
        const int c = p ^ ((row >> 2) & 3);
        const int64_t blk0 = op ? row0 : col0, lim = op ? out : in;
        int64_t grow = blk0 + row;
        if (grow >= lim) grow = blk0;
        const __half* base = op ? A : Hs;
        // offset of this lane's 16 bytes from the first row of the block, within one stage
        goff[j] = static_cast<uint32_t>(((grow - blk0) * (blocked ? 32 : in) + 8 * c) * 2);
        gdst[j] = lds0 + op * OP_BYTES + rq * 1024;
        // stage 0, predicated on the ragged length
        const void* g = 8 * c < r0 ? static_cast<const void*>(base + score_index(grow, k_begin + 8 * c, lim, in))
                                   : zero16;
        g2l16(g, gdst[j]);
    }
    // scalar bases of the two operands for the next stage to issue (first row of the block, first k
    // of the stage) and their advance per stage
    const char* baseA = reinterpret_cast<const char*>(Hs + score_index(col0, k_begin + r0, in, in));    // operand 0
    const char* baseB = reinterpret_cast<const char*>(A + score_index(row0, k_begin + r0, out, in));    // operand 1
    const int64_t stepA = blocked ? BT * ROWB : KT * 2, stepB = stepA;   // blocked: the next 16 KB piece
    int issued = 1;
    const char* curA = baseA;
    const char* curB = baseB;
    uint32_t cur_mask = 0;
    auto uniform_ptr = [](const char* ptr) {
        const uintptr_t b = reinterpret_cast<uintptr_t>(ptr);
        const uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(b));
        const uint32_t hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(b >> 32));
        return reinterpret_cast<const char*>((uintptr_t(hi) << 32) | lo);
    };
    auto stage_begin = [&]() {
        const bool real = issued < n_st;   // stages past the end read the 16 zero bytes
        curA = uniform_ptr(real ? baseA : static_cast<const char*>(zero16));
        curB = uniform_ptr(real ? baseB : static_cast<const char*>(zero16));
        cur_mask = real ? 0xffffffffu : 0u;
    };
    auto issue_one = [&](int j, int buf) {
        g2l16_s(j < LOADS / 2 ? curA : curB, goff[j] & cur_mask, gdst[j] + buf * STAGE_BYTES);
    };
    auto stage_issued = [&]() {
        ++issued;
        baseA += stepA;
        baseB += stepB;
    };
    auto issue_stage = [&](int buf) {
        stage_begin();
#pragma unroll
        for (int j = 0; j < LOADS; ++j) issue_one(j, buf);
        stage_issued();
    };

    // ---- fragment addresses: lane l reads row (l & 31) of a 32-row block, chunk 2*sweep + (l >> 5)
    const int fr = lane & 31, fh = lane >> 5;
    uint32_t f_off[2][TM + TN], f_off_hi[2][TM + TN];   // [sweep][fragment]
#pragma unroll
    for (int sw = 0; sw < 2; ++sw) {
#pragma unroll
        for (int k = 0; k < TM + TN; ++k) {
            const int row = (k < TM ? wm * WM + 32 * k : wn * WN + 32 * (k - TM)) + fr;
            const int c = (2 * sw + fh) ^ ((row >> 2) & 3);
            f_off[sw][k] = lds0 + (k < TM ? 0 : OP_BYTES) + row * ROWB + c * 16;
            f_off_hi[sw][k] = f_off[sw][k] + 2 * STAGE_BYTES;
            asm("" : "+v"(f_off_hi[sw][k]));
        }
    }
    auto read_one = [&](Frags& F, int buf, int sw, int k) {
        const uint32_t base = (buf & 2) ? f_off_hi[sw][k] : f_off[sw][k];
        F.v[k] = lds_read8(base + (buf & 1) * STAGE_BYTES);
    };
    auto read_frags = [&](Frags& F, int buf, int sw) {
#pragma unroll
        for (int k = 0; k < TM + TN; ++k) read_one(F, buf, sw, k);
    };

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    constexpr int NMMA = TM * TN, NRD = TM + TN;
    auto mma = [&](const Frags& F, int m) {
        const int i = m / TN, j = m % TN;
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(F.v[i], F.v[TM + j], acc[i][j], 0, 0, 0);
    };

    Frags F0, F1;
    issue_stage(1);
    issue_stage(2);
    asm volatile("s_waitcnt vmcnt(16)" ::: "memory");   // stage 0 landed
    __builtin_amdgcn_s_barrier();
    read_frags(F0, 0, 0);
    if (fused) {
        // H_nn / d_n^2 / 2 for the block's columns (d = 2^e: the bit pattern of 1/d is 0x7F000000 minus that of d);
        // read again only in the last eight stages, many barriers from here
        float hq = 0.0f;
        if (add_diag) {
            const float r = __uint_as_float(0x7F000000u - __float_as_uint(s_hd[0][tid]));
            hq = 0.5f * s_hd[1][tid] * r * r;
        }
        s_hq[tid] = hq;
    }
    constexpr int PRE = NMMA / 4;
    // in-loop epilogue state: the dW' entries of one 32-column sub-block (copied during the second sweep of its
    // stage, used during the first sweep of the next) and the row sums
    uint2 cap[TN * 4];
    float sum[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) sum[j] = 0.0f;
    // this lane's 8 bytes in row ol = wn*128 + 32 j + (lane & 31) of an operand-1 stage tile: j adds 32 rows, the
    // chunk swizzle (ol >> 2) & 3 does not depend on j
    const uint32_t cap_base = lds0 + OP_BYTES + (wn * WN + (lane & 31)) * ROWB + (lane >> 5) * 8;
    const int cap_swz = ((lane & 31) >> 2) & 3;
    // copy: item m = (j = m / 4, g = m % 4) of the sub-block whose stage sits in ring slot B
    auto capture = [&](auto buf_tag, int m) {
        constexpr int B = decltype(buf_tag)::value;
        const int j = m >> 2, g = m & 3;
        cap[m] = lds_read_u2(cap_base + B * STAGE_BYTES + j * 32 * ROWB + ((g ^ cap_swz) << 4));
    };
    // fold, at MFMA slot m of a first sweep: sum[j] += (E + hq * dW') * dW' for the four n of one item (j, g) of
    // sub-block IP (accumulator block row i = IP % 4).  That sweep's MFMAs for row i sit at slots 4 i .. 4 i + 3 and
    // add exact zeros to the finished accumulators; the items of column j are taken at slots 4 (i + 1 + j) + g
    // (mod 16), so that no item reads an accumulator block whose MFMA has just been issued.
    auto fold = [&](auto ip_tag, int m, const float4 (&hq4)[4]) {
        constexpr int IP = decltype(ip_tag)::value, i = IP & 3;
        const int t = (m - 4 * (i + 1)) & 15, j = t >> 2, g = t & 3;
        const uint2 raw = cap[t];
        // the four accumulator entries are fetched here and nowhere earlier (the empty asm pins the copy out of the
        // accumulator registers to this place; hoisted to the head of the sweep they would cost 64 registers)
        float e0 = acc[i][j][4 * g + 0], e1 = acc[i][j][4 * g + 1], e2 = acc[i][j][4 * g + 2], e3 = acc[i][j][4 * g + 3];
        asm volatile("" : "+v"(e0), "+v"(e1), "+v"(e2), "+v"(e3));
        sum[j] = fma_h<0>(raw.x, fma_h<0>(raw.x, hq4[g].x, e0), sum[j]);
        sum[j] = fma_h<1>(raw.x, fma_h<1>(raw.x, hq4[g].y, e1), sum[j]);
        sum[j] = fma_h<0>(raw.y, fma_h<0>(raw.y, hq4[g].z, e2), sum[j]);
        sum[j] = fma_h<1>(raw.y, fma_h<1>(raw.y, hq4[g].w, e3), sum[j]);
    };
    auto load_hq = [&](auto ip_tag, float4 (&hq4)[4]) {
        constexpr int IP = decltype(ip_tag)::value;
#pragma unroll
        for (int g = 0; g < 4; ++g)
            hq4[g] = *reinterpret_cast<const float4*>(&s_hq[(IP >> 2) * WM + 32 * (IP & 3) + 8 * g + 4 * (lane >> 5)]);
    };
    // One stage in ring slot B.  IP < 0: a plain stage.  IP = 0..7: stage IP of the diagonal block with the in-loop
    // epilogue: the waves that own sub-block IP - 1 (wm == (IP - 1) / 4) fold the entries copied a stage ago into
    // the row sums, one item per MFMA of the first sweep; the waves that own sub-block IP copy its dW' entries from
    // this stage's operand-1 tile, one item per MFMA of the second sweep (the tile stays in its ring slot until
    // the next stage's barrier).  The branches hold no MFMA: the accumulators are only read inside them.
    auto stage_body = [&](auto buf_tag, auto ip_tag) {
        constexpr int B = decltype(buf_tag)::value, IP = decltype(ip_tag)::value;
        constexpr int IPF = IP >= 1 ? IP - 1 : 0;
        static_assert(NMMA == TN * 4, "one epilogue item per MFMA of a sweep");
        float4 hq4[4] = {};
        const bool do_fold = IP >= 1 && wm == IPF / 4, do_cap = IP >= 0 && wm == (IP >= 0 ? IP : 0) / 4;
        if constexpr (IP >= 1) {
            if (do_fold) load_hq(std::integral_constant<int, IPF>{}, hq4);
        }
#pragma unroll
        for (int m = 0; m < NMMA; ++m) {
#pragma unroll
            for (int r = m * NRD / NMMA; r < (m + 1) * NRD / NMMA; ++r) read_one(F1, B, 1, r);
            if constexpr (IP >= 1) {
                if (do_fold) fold(std::integral_constant<int, IPF>{}, m, hq4);
            }
            mma(F0, m);
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int m = 0; m < PRE; ++m) {
            if constexpr (IP >= 0) {
                if (do_cap) capture(buf_tag, m);
            }
            mma(F1, m);
        }
        __builtin_amdgcn_sched_barrier(0);
        asm volatile("s_waitcnt vmcnt(8)" ::: "memory");   // next stage landed
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        stage_begin();
#pragma unroll
        for (int m = PRE; m < NMMA; ++m) {
            constexpr int REST = NMMA - PRE;
            const int q = m - PRE;
#pragma unroll
            for (int r = q * NRD / REST; r < (q + 1) * NRD / REST; ++r) read_one(F0, (B + 1) & 3, 0, r);
#pragma unroll
            for (int j = q * LOADS / REST; j < (q + 1) * LOADS / REST; ++j) issue_one(j, (B + 3) & 3);
            if constexpr (IP >= 0) {
                if (do_cap) capture(buf_tag, m);
            }
            mma(F1, m);
            __builtin_amdgcn_sched_barrier(0);
        }
        stage_issued();
    };
    if constexpr (DBG & 8) dbg_t[1] = wall_clock64();
    // four stages per trip (constant ring slots); surplus stages multiply zeros.  With the in-loop epilogue the
    // range is a whole number of 256-k blocks (n_st a multiple of 8, no surplus stages) and its last eight stages
    // are the diagonal block.
    constexpr std::integral_constant<int, -1> plain{};
    const int n_main = fused ? n_st - 8 : n_st;
    for (int s = 0; s < n_main; s += 4) {
        stage_body(std::integral_constant<int, 0>{}, plain);
        stage_body(std::integral_constant<int, 1>{}, plain);
        stage_body(std::integral_constant<int, 2>{}, plain);
        stage_body(std::integral_constant<int, 3>{}, plain);
    }
    if (fused) {
        stage_body(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
        stage_body(std::integral_constant<int, 1>{}, std::integral_constant<int, 1>{});
        stage_body(std::integral_constant<int, 2>{}, std::integral_constant<int, 2>{});
        stage_body(std::integral_constant<int, 3>{}, std::integral_constant<int, 3>{});
        stage_body(std::integral_constant<int, 0>{}, std::integral_constant<int, 4>{});
        stage_body(std::integral_constant<int, 1>{}, std::integral_constant<int, 5>{});
        stage_body(std::integral_constant<int, 2>{}, std::integral_constant<int, 6>{});
        stage_body(std::integral_constant<int, 3>{}, std::integral_constant<int, 7>{});
        if (wm == 1) {
            float4 hq4[4];
            load_hq(std::integral_constant<int, 7>{}, hq4);
#pragma unroll
            for (int m = 0; m < NMMA; ++m) fold(std::integral_constant<int, 7>{}, m, hq4);
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // no DMA may outlive the workgroup
    if constexpr (DBG & 8) dbg_t[2] = wall_clock64();

    // ---- epilogue: acc[i][j][r] = E[o, n] with o = row0 + wn*WN + 32j + (lane & 31) and
    // n = col0 + wm*WM + 32i + 8*(r/4) + 4*(lane >> 5) + (r & 3).  Multiply by dW'[o, n] (four
    // consecutive n per 8-byte read) and add up over n inside the lane.  In the scoring layout the
    // 256 x 256 tile of dW' is eight consecutive 16 KB pieces: it is copied into the ring (free by
    // now) with the transfers of operand 1, one piece per operand slot, and read back with the
    // fragment pattern; a lane's direct 8-byte loads would touch a different 64-byte row each.
    // With hmeta_diag (column scales d then diag H, as adadim_hessian_prepare writes them) the
    // workgroup of a column block's first chunk also adds half the diagonal term,
    // dW'[o,n]^2 H_nn / d_n^2 / 2: the final reduction doubles the row sums.
    if (blocked && !fused) {
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();                        // every wave is done with the ring
        const char* ebase = reinterpret_cast<const char*>(A + score_index(row0, col0, out, in));
        const int n_piece = static_cast<int>(min(int64_t(8), (in - col0) >> 5));
#pragma unroll
        for (int blk = 0; blk < 8; ++blk) {
            if (blk < n_piece) {                             // uniform
                const char* sb = uniform_ptr(ebase + blk * OP_BYTES);
#pragma unroll
                for (int j = LOADS / 2; j < LOADS; ++j) g2l16_s(sb, goff[j], gdst[j] + (blk - 1) * OP_BYTES);
            }
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
    }
    // Rows past `out` need no test on the LDS path: they hold a valid row's data and their sums
    // are never stored.  Columns past `in` are skipped (their accumulators are not zero).
    auto reduce = [&](auto from_lds) {
        constexpr bool LDS = decltype(from_lds)::value;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int64_t n0 = col0 + wm * WM + 32 * i + 8 * g + 4 * (lane >> 5);
                if (n0 >= in) continue;   // in % 8 == 0: the four columns are inside together
                float hq[4] = {0.0f, 0.0f, 0.0f, 0.0f};
                if (add_diag) {
                    const float4 d4 = *reinterpret_cast<const float4*>(hmeta_diag + n0);
                    const float4 h4 = *reinterpret_cast<const float4*>(hmeta_diag + in + n0);
                    // d = 2^e: the bit pattern of 1/d is 0x7F000000 minus that of d
                    const float r0 = __uint_as_float(0x7F000000u - __float_as_uint(d4.x));
                    const float r1 = __uint_as_float(0x7F000000u - __float_as_uint(d4.y));
                    const float r2 = __uint_as_float(0x7F000000u - __float_as_uint(d4.z));
                    const float r3 = __uint_as_float(0x7F000000u - __float_as_uint(d4.w));
                    hq[0] = 0.5f * h4.x * r0 * r0;
                    hq[1] = 0.5f * h4.y * r1 * r1;
                    hq[2] = 0.5f * h4.z * r2 * r2;
                    hq[3] = 0.5f * h4.w * r3 * r3;
                }
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const int ol = wn * WN + 32 * j + (lane & 31);
                    uint2 raw = make_uint2(0u, 0u);
                    if constexpr (LDS) {
                        raw = lds_read_u2(lds0 + (wm * 4 + i) * OP_BYTES + ol * ROWB + ((g ^ ((ol >> 2) & 3)) << 4) +
                                          (lane >> 5) * 8);
                    } else {
                        if (row0 + ol < out) raw = *reinterpret_cast<const uint2*>(A + score_index(row0 + ol, n0, out, in));
                    }
                    const float2 a = __half22float2(*reinterpret_cast<const __half2*>(&raw.x));
                    const float2 b = __half22float2(*reinterpret_cast<const __half2*>(&raw.y));
                    sum[j] += (acc[i][j][4 * g + 0] + hq[0] * a.x) * a.x;
                    sum[j] += (acc[i][j][4 * g + 1] + hq[1] * a.y) * a.y;
                    sum[j] += (acc[i][j][4 * g + 2] + hq[2] * b.x) * b.x;
                    sum[j] += (acc[i][j][4 * g + 3] + hq[3] * b.y) * b.y;
                }
            }
        }
    };
    if (!fused) {
        if (blocked) reduce(std::true_type{});
        else reduce(std::false_type{});
    }
    float v[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) v[j] = sum[j] + __shfl_xor(sum[j], 32, 64);
    if (lane < 32) {
#pragma unroll
        for (int j = 0; j < TN; ++j) s_rows[wm][wn * WN + 32 * j + lane] = v[j];
    }
    __syncthreads();
    if (tid < BT && row0 + tid < out)
        part[(int64_t(cand) * n_slots + slot) * out + row0 + tid] = s_rows[0][tid] + s_rows[1][tid];
    if constexpr (DBG & 8) {
        if (tid == 0) {
            dbg_t[3] = wall_clock64();
            uint32_t* d = reinterpret_cast<uint32_t*>(part + int64_t(batch.n) * n_slots * out) + rec * 8;
#pragma unroll
            for (int q = 0; q < 4; ++q) d[q] = static_cast<uint32_t>(dbg_t[q]);
            d[4] = static_cast<uint32_t>(n_st);
            d[5] = static_cast<uint32_t>(slot);
            // where it ran: XCC id (hardware register 20) in bits 16..19 above the SE / SH / CU fields of HW_ID (register 4)
            const uint32_t hw = __builtin_amdgcn_s_getreg((4 << 0) | (0 << 6) | (31 << 11));
            const uint32_t xcc = __builtin_amdgcn_s_getreg((20 << 0) | (0 << 6) | (3 << 11));
            d[6] = (xcc << 16) | (hw & 0xff00u);
            d[7] = 1u;
        }
    }
    return 0;
}

// The launch: one workgroup per list position, XCD = launch index % 8 (workgroups go to the eight XCDs round-robin
// by launch index).  (Tried and not kept: persistent workgroups, one per compute unit, taking positions from
// per-XCD counters.  Between two workgroups of a launch the hardware leaves a compute unit idle for 6 to 8 us on
// average, and a persistent workgroup goes on within 3 us; but the time a compute unit is busy with the same
// items then grows by about as much as the gaps shrink, 778 -> 832 us per compute unit on the 4096 x 11008
// layer: the matrix cores run against the chip's power limit, and idle time between workgroups is time at a
// higher clock afterwards.  Whole launches moved by -2 % to +9 %.)
template <int DBG = 0>
__global__ __launch_bounds__(256) void error_tiles_dma(Batch batch, const __half* __restrict__ Hs, int64_t out,
                                                       int64_t in, int MB, int NB, int kc_len, int n_slots,
                                                       const void* zero16, const float* __restrict__ hmeta_diag,
                                                       float* __restrict__ part) {
    extern __shared__ __align__(16) char smem[];
    (void)error_item<DBG>(batch, Hs, out, in, MB, NB, kc_len, n_slots, zero16, hmeta_diag, part,
                          static_cast<int>(blockIdx.x % 8), static_cast<int>(blockIdx.x / 8), int64_t(blockIdx.x), smem);
}

}  // namespace edma

}  // namespace
