// Host-side construction of a GDWS layer: index tables, per-channel SVD, greedy allocations.
// Sections cited are those of the GDWS paper (Section 3.2 properties, Section 3.3 algorithms,
// appendix proofs).
#include "planner.h"

#include <algorithm>
#include <cmath>
#include <limits>
#include <numeric>

namespace gdws {

// Property 2: channel c owns intermediate channels offsets[c] .. offsets[c+1]-1.
void build_tables(const int32_t *g, int C, std::vector<int32_t> &offsets, std::vector<int32_t> &chan_of)
{
    offsets.assign(C + 1, 0);
    for (int c = 0; c < C; ++c) offsets[c + 1] = offsets[c] + g[c];
    chan_of.resize(offsets[C]);
    for (int c = 0; c < C; ++c)
        for (int j = offsets[c]; j < offsets[c + 1]; ++j) chan_of[j] = c;
}

// One-sided (Hestenes) Jacobi SVD of an m x n matrix held column-major in a[n][m]:
// columns are rotated in pairs until mutually orthogonal; their norms are then the
// singular values, the normalised columns the left vectors, and the accumulated
// rotations the right vectors.
void SliceSvd::compute(const double *A, int m_, int n_)
{
    m = m_; n = n_;
    std::vector<double> a((size_t)n * m), v((size_t)n * n, 0.0);
    for (int j = 0; j < n; ++j) {
        for (int i = 0; i < m; ++i) a[(size_t)j * m + i] = A[(size_t)i * n + j];
        v[(size_t)j * n + j] = 1.0;
    }
    const double eps = std::numeric_limits<double>::epsilon();
    for (int sweep = 0; sweep < 60; ++sweep) {
        bool rotated = false;
        for (int p = 0; p < n - 1; ++p)
            for (int q = p + 1; q < n; ++q) {
                double app = 0, aqq = 0, apq = 0;
                const double *cp = &a[(size_t)p * m], *cq = &a[(size_t)q * m];
                for (int i = 0; i < m; ++i) { app += cp[i] * cp[i]; aqq += cq[i] * cq[i]; apq += cp[i] * cq[i]; }
                if (apq == 0.0 || std::fabs(apq) <= eps * std::sqrt(app * aqq)) continue;
                rotated = true;
                const double zeta = (aqq - app) / (2.0 * apq);
                const double t = (zeta >= 0 ? 1.0 : -1.0) / (std::fabs(zeta) + std::sqrt(1.0 + zeta * zeta));
                const double cs = 1.0 / std::sqrt(1.0 + t * t), sn = cs * t;
                double *wp = &a[(size_t)p * m], *wq = &a[(size_t)q * m];
                for (int i = 0; i < m; ++i) {
                    const double x = wp[i], y = wq[i];
                    wp[i] = cs * x - sn * y; wq[i] = sn * x + cs * y;
                }
                double *vp = &v[(size_t)p * n], *vq = &v[(size_t)q * n];
                for (int i = 0; i < n; ++i) {
                    const double x = vp[i], y = vq[i];
                    vp[i] = cs * x - sn * y; vq[i] = sn * x + cs * y;
                }
            }
        if (!rotated) break;
    }
    std::vector<double> norm(n);
    for (int j = 0; j < n; ++j) {
        double s = 0;
        for (int i = 0; i < m; ++i) s += a[(size_t)j * m + i] * a[(size_t)j * m + i];
        norm[j] = std::sqrt(s);
    }
    std::vector<int> order(n);
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int x, int y) { return norm[x] > norm[y]; });
    const int R = std::min(m, n);
    sigma.assign(R, 0.0);
    u.assign((size_t)R * m, 0.0);
    vt.assign((size_t)R * n, 0.0);
    for (int k = 0; k < R; ++k) {
        const int j = order[k];
        sigma[k] = norm[j];
        // sign convention: the largest-magnitude entry of v_k (lowest index on ties) is positive
        int big = 0;
        for (int i = 1; i < n; ++i)
            if (std::fabs(v[(size_t)j * n + i]) > std::fabs(v[(size_t)j * n + big])) big = i;
        const double sgn = v[(size_t)j * n + big] < 0 ? -1.0 : 1.0;
        for (int i = 0; i < n; ++i) vt[(size_t)k * n + i] = sgn * v[(size_t)j * n + i];
        if (norm[j] > 0)
            for (int i = 0; i < m; ++i) u[(size_t)k * m + i] = sgn * a[(size_t)j * m + i] / norm[j];
    }
    const double thresh = sigma.empty() ? 0.0 : sigma[0] * eps * std::max(m, n);
    rank = 0;
    for (int k = 0; k < R; ++k)
        if (sigma[k] > thresh && sigma[k] > 0.0) ++rank;
}

// W_c: the M x K^2 slice of W [M][C][K][K] belonging to input channel c.
void slice_of(const float *W, int M, int C, int KK, int c, std::vector<double> &out)
{
    out.resize((size_t)M * KK);
    for (int m = 0; m < M; ++m)
        for (int k = 0; k < KK; ++k) out[(size_t)m * KK + k] = W[((size_t)m * C + c) * KK + k];
}

// Lemma 3 + Properties 1, 2: rank-g[c] truncated SVD of every slice; row offsets[c]+i of the
// depthwise matrix is v_i^T, column offsets[c]+i of the pointwise matrix is sigma_i u_i.
// Filters past the slice's numerical rank are zero.
void factorise(const float *W, int M, int C, int K, const int32_t *g, const std::vector<int32_t> &offsets,
               std::vector<float> &dw, std::vector<float> &pw)
{
    const int KK = K * K, G = offsets[C];
    dw.assign((size_t)G * KK, 0.f);
    pw.assign((size_t)M * G, 0.f);
    std::vector<double> Wc;
    SliceSvd svd;
    for (int c = 0; c < C; ++c) {
        if (g[c] == 0) continue;
        slice_of(W, M, C, KK, c, Wc);
        svd.compute(Wc.data(), M, KK);
        for (int i = 0; i < g[c] && i < svd.rank; ++i) {
            const int j = offsets[c] + i;
            for (int k = 0; k < KK; ++k) dw[(size_t)j * KK + k] = (float)svd.vt[(size_t)i * KK + k];
            for (int m = 0; m < M; ++m) pw[(size_t)m * G + j] = (float)(svd.sigma[i] * svd.u[(size_t)i * M + m]);
        }
    }
}

// Algorithm 1.  Each step gives one more filter to the unsaturated channel with the
// largest alpha_c * sigma_{g_c+1,c}^2; stops at sum(g) == gamma or when all are saturated.
void mego(const double *sigma, const int32_t *rank, int C, int R, const double *alpha, int64_t gamma, int cap,
          int32_t *g)
{
    int64_t total = 0;
    for (int c = 0; c < C; ++c) total += g[c];
    while (total < gamma) {
        int best = -1;
        double gain = -1.0;
        for (int c = 0; c < C; ++c) {
            const int lim = cap > 0 ? std::min(rank[c], cap) : rank[c];
            if (g[c] >= lim || g[c] >= R) continue;
            const double s = sigma[(size_t)c * R + g[c]];
            const double v = (alpha ? alpha[c] : 1.0) * s * s;
            if (v > gain) { gain = v; best = c; }
        }
        if (best < 0) break;
        ++g[best];
        ++total;
    }
}

// Algorithm 2: starting from the ranks, drop the filter with the smallest alpha_c * sigma_{g_c,c}^2 while the
// dropped total stays within the bound.  The bound has two readings.  listing == false (Theorem 2 and its proof):
// the total of dropped squared terms stays <= beta^2.  listing == true (the algorithm box taken literally): the
// running total is compared with beta itself, strictly.
void lego(const double *sigma, const int32_t *rank, int C, int R, const double *alpha, double beta, int g_min,
          bool listing, int32_t *g)
{
    for (int c = 0; c < C; ++c) g[c] = std::min(rank[c], R);
    double dropped = 0.0;
    for (;;) {
        int best = -1;
        double term = std::numeric_limits<double>::infinity();
        for (int c = 0; c < C; ++c) {
            if (g[c] <= g_min) continue;
            const double s = sigma[(size_t)c * R + g[c] - 1];
            const double v = (alpha ? alpha[c] : 1.0) * s * s;
            if (v < term) { term = v; best = c; }
        }
        if (best < 0) break;
        if (listing ? !(dropped + term < beta) : dropped + term > beta * beta) break;
        dropped += term;
        --g[best];
    }
}

// eq. 3 against eq. 2: the largest G with G (K^2 + M) <= rho C K^2 M, kept within [C, min(K^2, M) C] so that every
// channel can hold at least one filter and none more than its slice's largest possible rank.
int64_t budget_gamma(double rho, int C, int K, int M)
{
    const double kk = (double)K * K;
    const int64_t gam = (int64_t)std::floor(rho * C * kk * M / (kk + M) + 1e-9);
    const int64_t cap = (int64_t)std::min(K * K, M) * C;
    return std::max<int64_t>(C, std::min(cap, gam));
}

// Appendix B: an intermediate channel whose depthwise filter is all zero produces a zero map, and one whose
// pointwise column is all zero is never read; either way it adds nothing to the output and is dropped.
void compact_factors(int C, int M, int KK, const int32_t *g, const float *dw, const float *pw, std::vector<int32_t> &g_out,
                     std::vector<float> &dw_out, std::vector<float> &pw_out, std::vector<int32_t> &keep)
{
    int G = 0;
    for (int c = 0; c < C; ++c) G += g[c];
    g_out.assign(C, 0);
    keep.clear();
    int j = 0;
    for (int c = 0; c < C; ++c)
        for (int i = 0; i < g[c]; ++i, ++j) {
            bool filter = false, column = false;
            for (int k = 0; k < KK && !filter; ++k) filter = dw[(size_t)j * KK + k] != 0.f;
            for (int m = 0; m < M && !column; ++m) column = pw[(size_t)m * G + j] != 0.f;
            if (filter && column) { keep.push_back(j); ++g_out[c]; }
        }
    const int Gk = (int)keep.size();
    dw_out.resize((size_t)Gk * KK);
    pw_out.resize((size_t)M * Gk);
    for (int q = 0; q < Gk; ++q) {
        std::copy(dw + (size_t)keep[q] * KK, dw + (size_t)(keep[q] + 1) * KK, dw_out.begin() + (size_t)q * KK);
        for (int m = 0; m < M; ++m) pw_out[(size_t)m * Gk + q] = pw[(size_t)m * G + keep[q]];
    }
}

}  // namespace gdws
