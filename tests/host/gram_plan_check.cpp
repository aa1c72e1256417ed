// Host-side check of the Gram kernel's launch plans (csrc/gram_plan.h, the text the kernels compile): for many
// (token count, tile count) pairs, choose a plan as the library does, walk every workgroup of the launch through
// gram_plan_item, and check that
//   * every tile is either taken whole exactly once, or its pieces cover [0, tokens) exactly once, in order;
//   * every piece but the first of its token range starts on a stage boundary (the kernel puts a ragged length
//     into the piece's first stage) and full pieces have the plan's length;
//   * no two pieces share a partial slot, every slot is below gram_plan_slots, and the slots the reduction reads
//     for a tile (gram_plan_parts / gram_plan_slot) are exactly the ones its pieces wrote, in token order;
//   * the fixed order of a plan with short pieces (gram_plan_order) names every place of an XCD's lists once.
// With arguments "tokens in" it prints the plan chosen for that shape and its simulated balance.
#include "../../paper_2309_15531_amd/csrc/gram_plan.h"

#include <chrono>
#include <cstdio>
#include <cstdlib>
#include <map>
#include <vector>

static long check(const GramPlan& p) {
    long bad = 0;
    struct Piece { int64_t b, e; int slot; };
    std::vector<std::vector<Piece>> pieces(p.n_tiles);
    std::vector<int> whole(p.n_tiles, 0);
    std::map<int, int> slot_use;
    const int per = gram_plan_per_xcd(p);
    for (int xcd = 0; xcd < 8; ++xcd)
        for (int q = 0; q < per; ++q) {
            GramItem it;
            if (!gram_plan_item(p, xcd, q, it)) continue;
            if (it.tile < 0 || it.tile >= p.n_tiles) { ++bad; continue; }
            if (it.slot < 0) {
                if (it.tile >= p.n_whole || it.t_begin != 0 || it.t_end != p.tokens) ++bad;
                ++whole[it.tile];
            } else {
                if (it.tile < p.n_whole || it.slot >= gram_plan_slots(p)) ++bad;
                if (it.t_begin > it.t_end || it.t_end > p.tokens) ++bad;
                if (it.t_begin < it.t_end && it.t_begin % GRAM_STAGE != 0) ++bad;   // an empty piece reads nothing
                ++slot_use[it.slot];
                pieces[it.tile].push_back({it.t_begin, it.t_end, it.slot});
            }
        }
    for (auto& kv : slot_use) bad += kv.second != 1;
    for (int t = 0; t < p.n_tiles; ++t) {
        if (t < p.n_whole) {
            bad += whole[t] != 1 || !pieces[t].empty();
            continue;
        }
        bad += whole[t] != 0;
        // the reduction's view of the tile: slots in order k = 0 ..; they must be the pieces in token order
        const int tile_r = t - p.n_whole, n = gram_plan_parts(p, tile_r);
        if (n != static_cast<int>(pieces[t].size())) { ++bad; continue; }
        int64_t at = 0;
        for (int k = 0; k < n; ++k) {
            const int slot = gram_plan_slot(p, tile_r, k);
            const Piece* hit = nullptr;
            for (auto& pc : pieces[t]) if (pc.slot == slot) hit = &pc;
            if (!hit) { ++bad; continue; }
            if (hit->b != at) ++bad;
            at = hit->e;
        }
        bad += at != p.tokens;
    }
    // the fixed order, where the plan has one: every place of an XCD's lists exactly once, units in ascending runs
    GramOrder o;
    gram_plan_order(p, o);
    if (o.n) {
        bad += o.n != per || o.first[0] != 0 || o.first[32] != o.n;
        std::vector<int> seen(per, 0);
        for (int c = 0; c < 32; ++c) {
            bad += o.first[c] > o.first[c + 1];
            for (int k = o.first[c]; k < o.first[c + 1] && k < GRAM_ORDER_MAX; ++k) {
                if (o.pos[k] >= per) { ++bad; continue; }
                ++seen[o.pos[k]];
            }
        }
        for (int q = 0; q < per; ++q) bad += seen[q] != 1;
    }
    return bad;
}

int main(int argc, char** argv) {
    if (argc == 3) {
        const int64_t tokens = atoll(argv[1]), in = atoll(argv[2]);
        const int nb = static_cast<int>((in + 255) / 256), n_tiles = nb * (nb + 1) / 2;
        for (int whole_ok = 1; whole_ok >= 0; --whole_ok) {
            const auto t0 = std::chrono::steady_clock::now();
            const GramPlan p = gram_plan_choose(tokens, n_tiles, whole_ok != 0);
            const double ms = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count();
            double span = 0.0;
            gram_plan_cost(p, &span);
            const double even = double(n_tiles) * double((tokens + GRAM_STAGE - 1) / GRAM_STAGE) / 256.0;
            printf("tokens %lld in %lld tiles %d whole_ok %d: n_whole %d n_full %d per %lld n_cut %d m %d sub %lld slots %d "
                   "span %.0f even share %.0f (%.3f) chosen in %.2f ms, %ld mistakes\n",
                   (long long)tokens, (long long)in, n_tiles, whole_ok, p.n_whole, p.n_full,
                   (long long)(p.t_per_split / GRAM_STAGE), p.n_cut, p.m, (long long)(p.t_sub / GRAM_STAGE),
                   gram_plan_slots(p), span, even, even / span, ms, check(p));
        }
        return 0;
    }
    long bad = 0, plans = 0;
    const int64_t token_counts[] = {1, 31, 32, 33, 70, 200, 511, 1024, 4097, 16384, 65536, 65530, 131072, 100003};
    const int widths[] = {1280, 1536, 2048, 4096, 5120, 6008, 6144, 8192, 11008, 13824, 28672};
    for (int64_t tokens : token_counts)
        for (int in : widths) {
            const int nb = (in + 255) / 256, n_tiles = nb * (nb + 1) / 2;
            for (int whole_ok = 0; whole_ok < 2; ++whole_ok) {
                const GramPlan p = gram_plan_choose(tokens, n_tiles, whole_ok != 0);
                const long b = check(p);
                if (b) printf("tokens %lld in %d whole_ok %d: %ld mistakes\n", (long long)tokens, in, whole_ok, b);
                bad += b;
                ++plans;
            }
        }
    // plans nobody would choose, to reach the corners of the item arithmetic
    for (int n_tiles : {1, 3, 15, 136, 300})
        for (int n_whole : {0, 256})
            for (int n_full : {0, 1, 3})
                for (int n_cut : {0, 1, 8, 13})
                    for (int m : {1, 2, 7})
                        for (int64_t tokens : {int64_t(33), int64_t(1000), int64_t(4096)}) {
                            if (n_whole > n_tiles || n_cut > n_tiles - n_whole) continue;
                            const int64_t stages = (tokens + GRAM_STAGE - 1) / GRAM_STAGE;
                            const int64_t per = n_full ? std::max<int64_t>(1, stages / (n_full + 1) + 1) : stages + 1;
                            if (n_full && int64_t(n_full) * per * GRAM_STAGE > tokens) continue;
                            GramPlan p = {n_tiles, n_whole, n_full, n_cut, m, tokens, per * GRAM_STAGE, GRAM_STAGE};
                            const int64_t rem = stages - n_full * per;
                            p.t_sub = std::max<int64_t>(1, (rem + m - 1) / m) * GRAM_STAGE;
                            if (!gram_plan_has_rem(p)) p.n_cut = 0;
                            const long b = check(p);
                            if (b) printf("hand plan tiles %d whole %d full %d cut %d m %d tokens %lld: %ld mistakes\n", n_tiles,
                                          n_whole, n_full, n_cut, m, (long long)tokens, b);
                            bad += b;
                            ++plans;
                        }
    printf("%ld plans, %ld mistakes\n", plans, bad);
    return bad != 0;
}
