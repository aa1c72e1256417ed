// Host-side check of csrc/fastdiv.h: fastdiv(w, s, RN(1/s)) == RN(w/s) (bit for bit, up to the sign of zero).
// usage: fastdiv_check <log2 of the number of scale significands per weight significand, <= 23> [threads]
// With 23 the check is exhaustive over all (11-bit weight significand, 24-bit scale significand) pairs.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <thread>
#include <vector>
#include <atomic>

#include "../../paper_2309_15531_amd/csrc/fastdiv.h"

static float from_bits(uint32_t b) { float f; std::memcpy(&f, &b, 4); return f; }
static uint32_t bits_of(float f) { uint32_t b; std::memcpy(&b, &f, 4); return b; }

int main(int argc, char** argv) {
    const int lg = argc > 1 ? std::atoi(argv[1]) : 16;
    const int nthreads = argc > 2 ? std::atoi(argv[2]) : 8;
    const uint32_t n_s = 1u << lg, stride = (1u << 23) / n_s;
    std::atomic<uint64_t> bad{0}, done{0};
    // exponents: scale at 2^0, 2^-7 (typical), 2^-39, 2^39; weight at 2^0, 2^-6, 2^-24 (fp16 subnormal), 2^15
    const int s_exp[] = {0, -7, -39, 39};
    const int w_exp[] = {0, -6, -24, 15};
    auto work = [&](int tidx) {
        uint64_t lbad = 0, ldone = 0;
        for (uint32_t mw = 1024 + tidx; mw < 2048; mw += nthreads) {
            for (uint32_t k = 0; k < n_s; ++k) {
                // cover every significand when exhaustive; otherwise a strided sample with a per-row offset
                const uint32_t ms = (k * stride + (mw * 2654435761u) % stride) & 0x7fffffu;
                for (int ei = 0; ei < (lg >= 23 ? 1 : 4); ++ei) {
                    const float s = from_bits(((127 + s_exp[ei]) << 23) | ms);
                    const float w0 = std::ldexp((float)mw, w_exp[ei] - 10);
                    if (!fastdiv_ok(s)) continue;
                    const float y = 1.0f / s;
                    for (int sg = 0; sg < 2; ++sg) {
                        const float w = sg ? -w0 : w0;
                        const float ref = w / s;
                        const float got = fastdiv(w, s, y);
                        ++ldone;
                        if (!(ref == got)) {   // numeric equality: the sign of a zero quotient is irrelevant downstream
                            if (lbad < 5) std::printf("MISMATCH w=%a s=%a ref=%a got=%a\n", w, s, ref, got);
                            ++lbad;
                        }
                    }
                }
            }
        }
        bad += lbad;
        done += ldone;
    };
    std::vector<std::thread> th;
    for (int t = 0; t < nthreads; ++t) th.emplace_back(work, t);
    for (auto& t : th) t.join();
    // range / qmax with the reciprocal of qmax = 2^b - 1: every fp32 numerator significand, several binades
    for (int b = 2; b <= 8; ++b) {
        const float qmax = (float)((1 << b) - 1), y = 1.0f / qmax;
        const int exps[] = {0, -20, 17, -60};
        for (int e : exps)
            for (uint32_t m = 0; m < (1u << 23); ++m) {
                const float rng = from_bits(((127 + e) << 23) | m);
                ++done;
                if (!(rng / qmax == fastdiv(rng, qmax, y))) {
                    if (bad < 5) std::printf("MISMATCH range=%a qmax=%g\n", rng, qmax);
                    ++bad;
                }
            }
    }
    // exact ties and zero
    const float ties[][2] = {{0.375f, 0.25f}, {0.625f, 0.25f}, {-1.25f, 0.5f}, {0.0f, 0.3f}, {-0.0f, 0.3f}, {2.5f, 1.0f}};
    for (auto& p : ties) {
        const float ref = p[0] / p[1], got = fastdiv(p[0], p[1], 1.0f / p[1]);
        ++done;
        if (!(ref == got)) { std::printf("MISMATCH tie w=%a s=%a\n", p[0], p[1]); ++bad; }
    }
    std::printf("checked %llu quotients, %llu mismatches\n", (unsigned long long)done.load(), (unsigned long long)bad.load());
    return bad.load() ? 1 : 0;
}
