// Launch plan of the 256-wide Gram kernel (H = X^T X, Eq. 1's quadratic form): which workgroup runs which tile
// over which token range, and where its partial tile goes.
//
// The kernel runs one workgroup per compute unit, 32 per XCD.  A plan cuts the work into four lists:
//   whole   the first n_whole tiles (decode order), each over all tokens, stored straight into H;
//   big     every other tile, n_full pieces of t_per_split tokens each (split-major);
//   small   the rest of the token range (shorter than a full piece) of the tiles n_cut .. n_rest-1;
//   sub     that rest for the tiles 0 .. n_cut-1, cut once more into m pieces of t_sub tokens (tile-major):
//           short items that level the last round.
// XCD x takes the x-th contiguous eighth of each list, so the workgroups resident on one XCD stream the same
// token range over different tiles and share their row and column panels in its L2.  Every piece but a whole
// tile writes one fp32 partial tile into its slot; the reduction adds a tile's slots up in a fixed order.
//
// A plan with sub pieces also fixes who runs what (GramOrder): the launch has 32 workgroups per XCD and each walks
// its own list of items, the list that "every item, long ones first, to the unit that is free first" gives in a
// simulation on the host.  Leaving that to the hardware's dispatcher (one workgroup per item, in list order)
// costs such a plan its last round: it was seen to keep short items waiting for particular units while others
// stood idle (12 of 14 started at once on 15 free units, the other two a hundred microseconds later).  Plans
// without sub pieces, and launches with more items per XCD than the order table holds, run one workgroup per
// item.
//
// Plain C++, so that the same text compiles into the kernels (through hipcc), into the host code that chooses a
// plan, and into tests/host/gram_plan_check.cpp, which walks every item of many plans and checks that the pieces
// cover each tile's token range exactly once and that no two share a slot.
#pragma once

#include <algorithm>
#include <cstdint>

#if defined(__HIPCC__)
#include <hip/hip_runtime.h>
#define GRAM_PLAN_FN __host__ __device__ __forceinline__
#else
#define GRAM_PLAN_FN inline
#endif

constexpr int GRAM_STAGE = 32;     // tokens per pipeline stage of the tile kernel

struct GramPlan {
    int n_tiles;            // upper-triangular 256x256 tiles of H
    int n_whole;            // tiles taken whole
    int n_full;             // full-length pieces of each other tile
    int n_cut;              // tiles (the first of the others) whose rest is cut into m pieces; 0 when there is no rest
    int m;                  // pieces per cut rest (>= 1)
    int64_t tokens;
    int64_t t_per_split;    // tokens per full-length piece, a multiple of GRAM_STAGE
    int64_t t_sub;          // tokens per piece of a cut rest, a multiple of GRAM_STAGE
};

struct GramItem {
    int tile;               // index in decode order
    int slot;               // partial tile to write; -1: a whole tile, stored into H
    int64_t t_begin, t_end; // token range (may be empty for a surplus piece of a cut rest: its partial is all zero)
};

constexpr int GRAM_ORDER_MAX = 1000;
struct GramOrder {
    uint16_t n;                     // entries of pos (= gram_plan_per_xcd); 0: no order, one workgroup per item
    uint16_t first[33];             // unit c of an XCD runs the places pos[first[c]] .. pos[first[c + 1] - 1], in turn
    uint16_t pos[GRAM_ORDER_MAX];   // places in the XCD's lists (gram_plan_item's q)
};

GRAM_PLAN_FN int gram_plan_rest(const GramPlan& p) { return p.n_tiles - p.n_whole; }
GRAM_PLAN_FN bool gram_plan_has_rem(const GramPlan& p) { return p.tokens > int64_t(p.n_full) * p.t_per_split; }
GRAM_PLAN_FN int gram_plan_big(const GramPlan& p) { return gram_plan_rest(p) * p.n_full; }
GRAM_PLAN_FN int gram_plan_small(const GramPlan& p) { return gram_plan_has_rem(p) ? gram_plan_rest(p) - p.n_cut : 0; }
GRAM_PLAN_FN int gram_plan_sub(const GramPlan& p) { return gram_plan_has_rem(p) ? p.n_cut * p.m : 0; }
GRAM_PLAN_FN int gram_plan_slots(const GramPlan& p) { return gram_plan_big(p) + gram_plan_small(p) + gram_plan_sub(p); }

// workgroups per XCD of each list, and of the launch
GRAM_PLAN_FN int gram_plan_per_xcd(const GramPlan& p) {
    return (p.n_whole + 7) / 8 + (gram_plan_big(p) + 7) / 8 + (gram_plan_small(p) + 7) / 8 + (gram_plan_sub(p) + 7) / 8;
}

// XCD x's share of a list of n items begins at item x * ceil(n / 8): contiguous eighths, the last one (or ones)
// short.  (Shares that differ by one item at most were measured on the 5120-wide input, 27 x 7 + 21 tiles against
// 26 or 27 each: no faster.  A short XCD leaves its part of the chip's power to the others.)
GRAM_PLAN_FN int gram_plan_share_begin(int n, int xcd) {
    const int b = xcd * ((n + 7) / 8);
    return b < n ? b : n;
}

// Item of workgroup q (0 .. gram_plan_per_xcd - 1) on XCD xcd; false if that place of the launch is empty.
GRAM_PLAN_FN bool gram_plan_item(const GramPlan& p, int xcd, int q, GramItem& it) {
    const int n_rest = gram_plan_rest(p), total_big = gram_plan_big(p), n_small = gram_plan_small(p),
              n_sub = gram_plan_sub(p);
    const int per_whole = (p.n_whole + 7) / 8, per_big = (total_big + 7) / 8, per_small = (n_small + 7) / 8,
              per_sub = (n_sub + 7) / 8;
    if (q < per_whole) {
        it.tile = gram_plan_share_begin(p.n_whole, xcd) + q;
        it.slot = -1;
        it.t_begin = 0;
        it.t_end = p.tokens;
        return it.tile < gram_plan_share_begin(p.n_whole, xcd + 1);
    }
    q -= per_whole;
    if (q < per_big) {
        const int i = gram_plan_share_begin(total_big, xcd) + q;
        if (i >= gram_plan_share_begin(total_big, xcd + 1)) return false;
        const int split = i / n_rest;
        it.tile = p.n_whole + (i - split * n_rest);
        it.slot = i;
        it.t_begin = int64_t(split) * p.t_per_split;
        it.t_end = it.t_begin + p.t_per_split;
        return true;
    }
    q -= per_big;
    const int64_t rem_begin = int64_t(p.n_full) * p.t_per_split;
    if (q < per_small) {
        const int s = gram_plan_share_begin(n_small, xcd) + q;
        if (s >= gram_plan_share_begin(n_small, xcd + 1)) return false;
        it.tile = p.n_whole + p.n_cut + s;
        it.slot = total_big + s;
        it.t_begin = rem_begin;
        it.t_end = p.tokens;
        return true;
    }
    q -= per_small;
    if (q >= per_sub) return false;
    const int u = gram_plan_share_begin(n_sub, xcd) + q;
    if (u >= gram_plan_share_begin(n_sub, xcd + 1)) return false;
    const int t = u / p.m, j = u - t * p.m;
    it.tile = p.n_whole + t;
    it.slot = total_big + n_small + u;
    it.t_begin = std::min<int64_t>(p.tokens, rem_begin + int64_t(j) * p.t_sub);
    it.t_end = j == p.m - 1 ? p.tokens : std::min<int64_t>(p.tokens, it.t_begin + p.t_sub);
    return true;
}

// Partial tiles of the tile with index tile_r among the tiles that are not whole: how many, and the k-th one's slot.
GRAM_PLAN_FN int gram_plan_parts(const GramPlan& p, int tile_r) {
    return p.n_full + (gram_plan_has_rem(p) ? (tile_r < p.n_cut ? p.m : 1) : 0);
}
GRAM_PLAN_FN int gram_plan_slot(const GramPlan& p, int tile_r, int k) {
    if (k < p.n_full) return k * gram_plan_rest(p) + tile_r;
    const int total_big = gram_plan_big(p);
    if (tile_r < p.n_cut) return total_big + gram_plan_small(p) + tile_r * p.m + (k - p.n_full);
    return total_big + tile_r - p.n_cut;
}

// ---- choosing a plan (host) ----
//
// By simulating one XCD's 32 units: each list's eighth, long items first, every item to the unit that is free
// first.  Unit of time: one 32-token stage; an item costs about 12 stages of prologue and epilogue
// on top of its stages, a partial tile about 0.2 stage of reduction traffic behind the tile kernel, a whole tile
// 0.15 (its prepared form is made from H).  Equal pieces alone leave the last round partly empty (17 tiles per
// XCD in three pieces each: 51 items and a short rest on 32 units, 0.90 of the even share); cutting the rest of a
// few tiles into short pieces fills it (0.98).
namespace gram_plan_detail {

struct Slots32 {
    double t[32];
    int place(double dur) {                                   // onto the unit that is free first
        int m = 0;
        for (int k = 1; k < 32; ++k)
            if (t[k] < t[m]) m = k;
        t[m] += dur;
        return m;
    }
    double span() const {
        double s = 0.0;
        for (int k = 0; k < 32; ++k) s = std::max(s, t[k]);
        return s;
    }
};

constexpr double ITEM_OVERHEAD = 12.0, PARTIAL_COST = 0.20, WHOLE_COST = 0.15;

}  // namespace gram_plan_detail

// Estimated cost (stages) of a plan; the simulation behind gram_plan_choose.  `after_whole`: the 32 units' times once
// the whole tiles are placed, if the caller has them.
inline double gram_plan_cost(const GramPlan& p, double* span_out = nullptr,
                             const gram_plan_detail::Slots32* after_whole = nullptr) {
    using namespace gram_plan_detail;
    const int64_t stages = (p.tokens + GRAM_STAGE - 1) / GRAM_STAGE;
    const int64_t per = p.t_per_split / GRAM_STAGE, rem = stages - int64_t(p.n_full) * per;
    Slots32 s = {};
    if (after_whole) s = *after_whole;
    else
        for (int i = 0; i < (p.n_whole + 7) / 8; ++i) s.place(double(stages) + ITEM_OVERHEAD);
    for (int i = 0; i < (gram_plan_big(p) + 7) / 8; ++i) s.place(double(per) + ITEM_OVERHEAD);
    for (int i = 0; i < (gram_plan_small(p) + 7) / 8; ++i) s.place(double(rem) + ITEM_OVERHEAD);
    for (int i = 0; i < (gram_plan_sub(p) + 7) / 8; ++i) s.place(double(p.t_sub / GRAM_STAGE) + ITEM_OVERHEAD);
    const double span = s.span();
    if (span_out) *span_out = span;
    return span + PARTIAL_COST * double(gram_plan_slots(p)) + WHOLE_COST * double(p.n_whole);
}

// The fixed order of a plan: the same simulation, remembering which unit took which place.
inline void gram_plan_order(const GramPlan& p, GramOrder& o) {
    using namespace gram_plan_detail;
    o = GramOrder{};
    const int per = gram_plan_per_xcd(p);
    // plans without short pieces run as well with one workgroup per item (measured), and that way adapts to units
    // of unequal speed
    if (p.n_cut == 0 || !gram_plan_has_rem(p) || per > GRAM_ORDER_MAX) return;
    const int64_t stages = (p.tokens + GRAM_STAGE - 1) / GRAM_STAGE;
    const int64_t len_big = p.t_per_split / GRAM_STAGE, len_small = stages - int64_t(p.n_full) * len_big;
    const int n0 = (p.n_whole + 7) / 8, n1 = n0 + (gram_plan_big(p) + 7) / 8, n2 = n1 + (gram_plan_small(p) + 7) / 8;
    static_assert(GRAM_ORDER_MAX < 65536, "places are stored in 16 bits");
    uint8_t unit[GRAM_ORDER_MAX];
    Slots32 s = {};
    for (int q = 0; q < per; ++q) {
        const int64_t len = q < n0 ? stages : q < n1 ? len_big : q < n2 ? len_small : p.t_sub / GRAM_STAGE;
        unit[q] = static_cast<uint8_t>(s.place(double(len) + ITEM_OVERHEAD));
    }
    int k = 0;
    for (int c = 0; c < 32; ++c) {
        o.first[c] = static_cast<uint16_t>(k);
        for (int q = 0; q < per; ++q)
            if (unit[q] == c) o.pos[k++] = static_cast<uint16_t>(q);
    }
    o.first[32] = static_cast<uint16_t>(k);
    o.n = static_cast<uint16_t>(per);
}

// whole_ok: whole tiles need a plain store (not an accumulating call).
inline GramPlan gram_plan_choose(int64_t tokens, int n_tiles, bool whole_ok) {
    using namespace gram_plan_detail;
    const int64_t stages = (tokens + GRAM_STAGE - 1) / GRAM_STAGE;
    GramPlan best = {n_tiles, 0, 1, 0, 1, tokens, stages * GRAM_STAGE, GRAM_STAGE};
    best.n_full = static_cast<int>(tokens / best.t_per_split);
    double best_cost = gram_plan_cost(best);
    Slots32 after_whole = {};
    auto consider = [&](const GramPlan& c) {
        const double cost = gram_plan_cost(c, nullptr, &after_whole);
        if (cost < best_cost) {
            best_cost = cost;
            best = c;
        }
    };
    // candidates with full pieces of `per` stages: the plain one, and the rest of 8, 16 or 24 tiles cut further
    auto with_per = [&](int nw, int64_t per) {
        if (per <= 0 || per > stages) return;
        GramPlan c = {n_tiles, nw, 0, 0, 1, tokens, per * GRAM_STAGE, GRAM_STAGE};
        c.n_full = static_cast<int>(tokens / c.t_per_split);
        const int n_rest = n_tiles - nw;
        if (int64_t(n_rest) * (c.n_full + 1) > 8 * 512) return;          // keeps the launch and the partials modest
        if (c.n_full > 1 && int64_t(n_rest) * c.n_full > 8 * 128) return; // more than four rounds of short pieces
        consider(c);
        const int64_t rem = stages - int64_t(c.n_full) * per;
        // no cut can end before the busiest unit's full pieces do
        const double floor_cost = after_whole.span() > 0.0 ? 0.0 : double(per) + ITEM_OVERHEAD + PARTIAL_COST * n_rest * (c.n_full + 1);
        if (rem < 32 || floor_cost >= best_cost) return;
        for (int cut = 8; cut <= 24 && cut <= n_rest; cut += 8)
            for (int m = 2; m <= 8; ++m) {
                const int64_t sub = ((rem + m - 1) / m + 3) / 4 * 4;     // whole trips of the kernel's four-stage loop
                if (sub * (m - 1) >= rem) continue;                       // the last piece would be empty
                c.n_cut = cut;
                c.m = m;
                c.t_sub = sub * GRAM_STAGE;
                consider(c);
            }
    };
    const int top = whole_ok ? (n_tiles / 256) * 256 : 0;
    for (int nw = top; nw >= 0 && nw >= top - 512; nw -= 256) {
        after_whole = Slots32{};
        for (int i = 0; i < (nw + 7) / 8; ++i) after_whole.place(double(stages) + ITEM_OVERHEAD);
        if (nw == n_tiles) {
            GramPlan c = {n_tiles, nw, 1, 0, 1, tokens, stages * GRAM_STAGE, GRAM_STAGE};
            c.n_full = static_cast<int>(tokens / c.t_per_split);
            consider(c);
            continue;
        }
        for (int nf = 1; nf <= 32 && nf <= stages; ++nf) {
            // piece lengths that give nf full pieces: stages/(nf+1) < per <= stages/nf, in steps of four stages
            // (about 1/24 of the range where that is coarser, refined around the best one), and the even division
            const int64_t lo = stages / (nf + 1) + 1, hi = stages / nf;
            if (lo > hi) continue;
            if (nf > 1 && int64_t(n_tiles - nw) * nf > 8 * 128) break;
            const int64_t step = std::max<int64_t>(4, ((hi - lo) / 24 + 3) / 4 * 4);
            const GramPlan before = best;
            for (int64_t per = (lo + 3) / 4 * 4; per <= hi; per += step) with_per(nw, per);
            with_per(nw, hi);
            if (step > 4 && best.n_whole == nw && (before.n_whole != nw || before.t_per_split != best.t_per_split)) {
                const int64_t mid = best.t_per_split / GRAM_STAGE;     // this nf took the lead: look around its best
                for (int64_t per = std::max(lo, mid - step + 4); per <= std::min(hi, mid + step - 4); per += 4)
                    with_per(nw, per);
            }
        }
    }
    return best;
}
