// Driver for the sanitizer build of the library's host-side planner (built and run by test_host_sanitizers.py):
// walks every routine of planner.h over small, irregular layers so that an out-of-bounds access, a signed overflow
// or an invalid shift in them is reported by AddressSanitizer / UndefinedBehaviorSanitizer.
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "planner.h"

static unsigned long long state = 0x9E3779B97F4A7C15ull;
static double uniform()
{
    state += 0x9E3779B97F4A7C15ull;
    unsigned long long z = state;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    z ^= z >> 31;
    return (double)(z >> 11) / 9007199254740992.0 - 0.5;
}

#define REQUIRE(c) do { if (!(c)) { std::printf("check failed at line %d: %s\n", __LINE__, #c); return 1; } } while (0)

int main()
{
    const int shapes[][3] = {{5, 3, 3}, {4, 7, 1}, {12, 5, 5}, {33, 2, 3}, {3, 4, 7}};  // M, C, K
    for (const auto &sh : shapes) {
        const int M = sh[0], C = sh[1], K = sh[2], KK = K * K, R = M < KK ? M : KK;
        std::vector<float> W((size_t)M * C * KK);
        for (auto &w : W) w = (float)uniform();
        for (int m = 0; m < M && C > 1; ++m)          // one channel's slice is zero: rank 0
            for (int t = 0; t < KK; ++t) W[((size_t)m * C + 1) * KK + t] = 0.f;
        std::vector<double> sigma((size_t)C * R);
        std::vector<int32_t> rank(C);
        for (int c = 0; c < C; ++c) {
            std::vector<double> A;
            gdws::slice_of(W.data(), M, C, KK, c, A);
            gdws::SliceSvd svd;
            svd.compute(A.data(), M, KK);
            REQUIRE((int)svd.sigma.size() == R);
            for (int i = 0; i + 1 < R; ++i) REQUIRE(svd.sigma[i] >= svd.sigma[i + 1]);
            for (int i = 0; i < R; ++i) sigma[(size_t)c * R + i] = svd.sigma[i];
            rank[c] = svd.rank;
        }
        if (C > 1) REQUIRE(rank[1] == 0);
        std::vector<int32_t> g(C), g2(C), g3(C);
        const int64_t gamma = gdws::budget_gamma(0.5, C, K, M);
        REQUIRE(gamma >= C && gamma <= (int64_t)R * C);
        gdws::mego(sigma.data(), rank.data(), C, R, nullptr, gamma, R, g.data());
        std::vector<double> alpha(C, 1.0);
        alpha[0] = 3.0;
        gdws::mego(sigma.data(), rank.data(), C, R, alpha.data(), gamma, 0, g2.data());
        gdws::lego(sigma.data(), rank.data(), C, R, nullptr, 0.3, 0, false, g2.data());
        gdws::lego(sigma.data(), rank.data(), C, R, alpha.data(), 0.3, 1, true, g3.data());
        for (int c = 0; c < C; ++c) REQUIRE(g[c] >= 0 && g[c] <= R && g2[c] >= 0 && g2[c] <= R && g3[c] >= 0 && g3[c] <= R);
        g[0] = R;                       // a full-rank channel and, if there is one, the zero slice with g > rank
        if (C > 1) g[1] = 2 <= R ? 2 : 1;
        if (C > 2) g[2] = 0;
        std::vector<int32_t> offsets, chan_of;
        gdws::build_tables(g.data(), C, offsets, chan_of);
        REQUIRE((int)offsets.size() == C + 1 && (int)chan_of.size() == offsets[C]);
        std::vector<float> dw, pw;
        gdws::factorise(W.data(), M, C, K, g.data(), offsets, dw, pw);
        const int G = offsets[C];
        REQUIRE(dw.size() == (size_t)G * KK && pw.size() == (size_t)M * G);
        // channel 0 keeps all its singular values: its slice is reproduced
        double err = 0;
        for (int m = 0; m < M; ++m)
            for (int t = 0; t < KK; ++t) {
                double acc = 0;
                for (int j = offsets[0]; j < offsets[1]; ++j) acc += (double)pw[(size_t)m * G + j] * dw[(size_t)j * KK + t];
                err = std::fmax(err, std::fabs(acc - W[((size_t)m * C + 0) * KK + t]));
            }
        REQUIRE(err < 1e-5);
        std::vector<int32_t> gc, keep;
        std::vector<float> dwc, pwc;
        gdws::compact_factors(C, M, KK, g.data(), dw.data(), pw.data(), gc, dwc, pwc, keep);
        int64_t Gc = 0;
        for (int c = 0; c < C; ++c) Gc += gc[c];
        REQUIRE(Gc == (int64_t)keep.size() && Gc <= G && dwc.size() == (size_t)Gc * KK && pwc.size() == (size_t)M * Gc);
        if (C > 1) REQUIRE(gc[1] == 0);  // the zero slice's filters are dropped
    }
    // extreme budgets clamp
    if (gdws::budget_gamma(0.0, 8, 3, 16) != 8 || gdws::budget_gamma(10.0, 8, 3, 16) != 72) { std::printf("budget clamp\n"); return 1; }
    std::printf("planner sanitizer walk ok\n");
    return 0;
}
