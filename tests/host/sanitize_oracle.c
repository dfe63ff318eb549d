/* Driver for the sanitizer build of the oracle's C loops (built and run by test_host_sanitizers.py): every routine on
 * small, irregular shapes (odd sizes, strides, padding, zero multipliers) so that an index that leaves a buffer is
 * reported by AddressSanitizer, with exact-size heap buffers. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int64_t oracle_conv_dense(const double *, const double *, const double *, double *, int, int, int, int, int, int, int, int, int);
int64_t oracle_gdw(const double *, const int32_t *, const double *, double *, int, int, int, int, int, int, int, int);
int64_t oracle_pw(const double *, const double *, const double *, double *, int, int, int, int, int);
void oracle_duplicate_channels(const double *, const int32_t *, double *, int, int, int);
void oracle_add_relu(double *, const double *, size_t, int);
void oracle_maxpool(const double *, double *, int, int, int, int, int, int, int);

static double *filled(size_t n, double v)
{
    double *p = (double *)malloc((n ? n : 1) * sizeof(double));
    for (size_t i = 0; i < n; ++i) p[i] = v + 0.001 * (double)(i % 97);
    return p;
}
static int out_size(int in, int K, int s, int p) { return (in + 2 * p - K) / s + 1; }

int main(void)
{
    const int cases[][7] = {/* N, C, H, W, K, stride, pad */
                            {2, 3, 7, 5, 3, 1, 1}, {1, 4, 9, 9, 5, 2, 2}, {3, 2, 4, 6, 1, 1, 0}, {1, 5, 11, 8, 7, 2, 3}, {2, 3, 5, 5, 3, 2, 0}};
    for (size_t k = 0; k < sizeof(cases) / sizeof(cases[0]); ++k) {
        const int N = cases[k][0], C = cases[k][1], H = cases[k][2], W = cases[k][3], K = cases[k][4], s = cases[k][5], p = cases[k][6];
        const int M = 6, Ho = out_size(H, K, s, p), Wo = out_size(W, K, s, p);
        int32_t g[8];
        int G = 0;
        for (int c = 0; c < C; ++c) { g[c] = (c * 2 + (int)k) % 4; G += g[c]; }
        if (G == 0) { g[0] = 1; G = 1; }
        double *x = filled((size_t)N * C * H * W, 0.5), *w = filled((size_t)M * C * K * K, -0.2), *b = filled(M, 0.1);
        double *y = filled((size_t)N * M * Ho * Wo, 0), *d = filled((size_t)G * K * K, 0.3), *t = filled((size_t)N * G * Ho * Wo, 0);
        double *pw = filled((size_t)M * G, -0.1), *y2 = filled((size_t)N * M * Ho * Wo, 0), *xd = filled((size_t)N * G * H * W, 0);
        const int64_t m1 = oracle_conv_dense(x, w, b, y, N, C, H, W, M, K, s, p, 1);
        const int64_t m2 = oracle_gdw(x, g, d, t, N, C, H, W, K, s, p, 1);
        const int64_t m3 = oracle_pw(t, pw, b, y2, N, G, Ho * Wo, M, 1);
        if (m1 != (int64_t)N * M * Ho * Wo * C * K * K || m2 != (int64_t)N * G * Ho * Wo * K * K || m3 != (int64_t)N * M * Ho * Wo * G) {
            printf("MAC counts of case %zu\n", k);
            return 1;
        }
        oracle_duplicate_channels(x, g, xd, N, C, H * W);
        oracle_add_relu(y2, y, (size_t)N * M * Ho * Wo, 1);
        if (Ho >= 2 && Wo >= 2) {
            const int Hp = out_size(Ho, 2, 2, 0), Wp = out_size(Wo, 2, 2, 0);
            double *yp = filled((size_t)N * M * Hp * Wp, 0);
            oracle_maxpool(y2, yp, N, M, Ho, Wo, 2, 2, 0);
            free(yp);
            const int Hq = out_size(Ho, 3, 2, 1), Wq = out_size(Wo, 3, 2, 1);
            double *yq = filled((size_t)N * M * Hq * Wq, 0);
            oracle_maxpool(y2, yq, N, M, Ho, Wo, 3, 2, 1);
            free(yq);
        }
        free(x); free(w); free(b); free(y); free(d); free(t); free(pw); free(y2); free(xd);
    }
    printf("oracle sanitizer walk ok\n");
    return 0;
}
