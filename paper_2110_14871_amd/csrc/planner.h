// Host-side construction of a GDWS layer (tables, per-channel SVD, greedy allocations).
#pragma once
#include <stdint.h>

#include <vector>

namespace gdws {

void build_tables(const int32_t *g, int C, std::vector<int32_t> &offsets, std::vector<int32_t> &chan_of);

// SVD of one m x n slice: sigma [R] descending, u [R][m], vt [R][n], R = min(m, n).
struct SliceSvd {
    int m = 0, n = 0, rank = 0;
    std::vector<double> sigma, u, vt;
    void compute(const double *A /* row-major m x n */, int m, int n);
};

void slice_of(const float *W, int M, int C, int KK, int c, std::vector<double> &out);

void factorise(const float *W, int M, int C, int K, const int32_t *g, const std::vector<int32_t> &offsets,
               std::vector<float> &dw, std::vector<float> &pw);

void mego(const double *sigma, const int32_t *rank, int C, int R, const double *alpha, int64_t gamma, int cap,
          int32_t *g);
void lego(const double *sigma, const int32_t *rank, int C, int R, const double *alpha, double beta, int g_min,
          bool listing, int32_t *g);
int64_t budget_gamma(double rho, int C, int K, int M);
// g_out [C], the kept filters / columns, keep [G']: index in the original of each kept intermediate channel
void compact_factors(int C, int M, int KK, const int32_t *g, const float *dw, const float *pw, std::vector<int32_t> &g_out,
                     std::vector<float> &dw_out, std::vector<float> &pw_out, std::vector<int32_t> &keep);

}  // namespace gdws
