// Batched singular values of the C slices W_c (M x K^2) of a convolution weight, on the device.
//
// Algorithm 1 (MEGO) and Algorithm 2 (LEGO) start from the singular values of every input channel's slice
// (Section 3.2 "Notation", Lemma 3): sigma_{i,c}, i < min(M, K^2).  The slices are small and many, so one wave takes
// one slice: it forms the K^2 x K^2 Gram matrix W_c^T W_c in fp64, diagonalises it with cyclic Jacobi rotations
// (V^T (W_c^T W_c) V = diag(sigma^2)) and writes sigma in descending order, the numerical rank and, optionally, the
// right singular vectors v_i (the depthwise filters of Lemma 3) with the sign fixed so that the entry of largest
// magnitude, the first of them on ties, is positive.
#include "kernels.h"

namespace gdws {

namespace {

constexpr int kMaxN = 49;     // K <= 7
constexpr int kLd = kMaxN + 1;
constexpr int kRowsPerPass = 32;
constexpr int kMaxSweeps = 40;

struct SvdParams {
    const float *w;
    double *sigma;
    int32_t *rank;
    double *v;
    int M, C, n, R;
};

__global__ __launch_bounds__(64) void svd_gram_jacobi_kernel(SvdParams p)
{
    __shared__ double A[kMaxN * kLd];   // the Gram matrix, then its diagonalised form
    __shared__ double V[kMaxN * kLd];   // columns: eigenvectors
    __shared__ double rows[kRowsPerPass * kMaxN];
    __shared__ int order[kMaxN];
    __shared__ int rotated;
    const int c = blockIdx.x, lane = threadIdx.x, n = p.n;

    // ---- Gram matrix: lanes over the entries, a loop over the M rows of the slice in passes of 32 rows ----
    constexpr int kPerLane = (kMaxN * kMaxN + 63) / 64;
    double acc[kPerLane];
#pragma unroll
    for (int e = 0; e < kPerLane; ++e) acc[e] = 0.0;
    for (int m0 = 0; m0 < p.M; m0 += kRowsPerPass) {
        const int nm = min(kRowsPerPass, p.M - m0);
        __syncthreads();
        for (int i = lane; i < nm * n; i += 64) {
            const int m = m0 + i / n, t = i % n;
            rows[i] = (double)p.w[((size_t)m * p.C + c) * n + t];
        }
        __syncthreads();
#pragma unroll
        for (int e = 0; e < kPerLane; ++e) {
            const int idx = lane + 64 * e;
            if (idx < n * n) {
                const int i = idx / n, j = idx % n;
                double a = acc[e];
                for (int m = 0; m < nm; ++m) a += rows[m * n + i] * rows[m * n + j];
                acc[e] = a;
            }
        }
    }
#pragma unroll
    for (int e = 0; e < kPerLane; ++e) {
        const int idx = lane + 64 * e;
        if (idx < n * n) {
            const int i = idx / n, j = idx % n;
            A[i * kLd + j] = acc[e];
            V[i * kLd + j] = i == j ? 1.0 : 0.0;
        }
    }
    __syncthreads();

    // ---- cyclic Jacobi: every pair (a, b) in turn; lane k updates row/column k of A and row k of V ----
    for (int sweep = 0; sweep < kMaxSweeps; ++sweep) {
        if (lane == 0) rotated = 0;
        __syncthreads();
        for (int a = 0; a < n - 1; ++a)
            for (int b = a + 1; b < n; ++b) {
                const double aaa = A[a * kLd + a], abb = A[b * kLd + b], aab = A[a * kLd + b];
                // (all lanes read the same three values: the branch is uniform)
                if (fabs(aab) > 1e-17 * sqrt(fabs(aaa * abb)) && aab != 0.0) {
                    const double theta = (abb - aaa) / (2.0 * aab);
                    const double t = (theta >= 0.0 ? 1.0 : -1.0) / (fabs(theta) + sqrt(theta * theta + 1.0));
                    const double cs = 1.0 / sqrt(t * t + 1.0), sn = t * cs;
                    __syncthreads();  // every lane has read the pivot entries
                    if (lane < n) {
                        const int k = lane;
                        const double vka = V[k * kLd + a], vkb = V[k * kLd + b];
                        V[k * kLd + a] = cs * vka - sn * vkb;
                        V[k * kLd + b] = sn * vka + cs * vkb;
                        if (k != a && k != b) {
                            const double aka = A[k * kLd + a], akb = A[k * kLd + b];
                            const double na = cs * aka - sn * akb, nb = sn * aka + cs * akb;
                            A[k * kLd + a] = na; A[a * kLd + k] = na;
                            A[k * kLd + b] = nb; A[b * kLd + k] = nb;
                        }
                    }
                    if (lane == 0) {
                        A[a * kLd + a] = aaa - t * aab;
                        A[b * kLd + b] = abb + t * aab;
                        A[a * kLd + b] = 0.0;
                        A[b * kLd + a] = 0.0;
                        rotated = 1;
                    }
                    __syncthreads();
                }
            }
        __syncthreads();
        const int any = rotated;
        __syncthreads();
        if (!any) break;
    }

    // ---- descending order, outputs ----
    if (lane == 0) {
        for (int i = 0; i < n; ++i) order[i] = i;
        for (int i = 0; i < n - 1; ++i) {  // selection sort, stable on ties
            int best = i;
            for (int j = i + 1; j < n; ++j)
                if (A[order[j] * kLd + order[j]] > A[order[best] * kLd + order[best]]) best = j;
            const int tmp = order[best];
            for (int j = best; j > i; --j) order[j] = order[j - 1];
            order[i] = tmp;
        }
    }
    __syncthreads();
    const double lam1 = fmax(A[order[0] * kLd + order[0]], 0.0);
    if (lane < p.R) p.sigma[(size_t)c * p.R + lane] = sqrt(fmax(A[order[lane] * kLd + order[lane]], 0.0));
    if (lane == 0 && p.rank) {
        // an eigenvalue of the Gram matrix carries an absolute error of a few eps * lambda_1, so a singular value
        // counts when its square stands clear of that
        const double thresh = 64.0 * (double)max(p.M, n) * 2.220446049250313e-16 * lam1;
        int r = 0;
        for (int i = 0; i < p.R; ++i) r += A[order[i] * kLd + order[i]] > thresh ? 1 : 0;
        p.rank[c] = r;
    }
    if (p.v && lane < p.R) {
        const int col = order[lane];
        int kbest = 0;
        double vbest = 0.0;
        for (int k = 0; k < n; ++k) {
            const double a = fabs(V[k * kLd + col]);
            if (a > vbest) { vbest = a; kbest = k; }
        }
        const double sgn = V[kbest * kLd + col] < 0.0 ? -1.0 : 1.0;
        for (int k = 0; k < n; ++k) p.v[((size_t)c * p.R + lane) * n + k] = sgn * V[k * kLd + col];
    }
}

}  // namespace

int launch_svd_device(const float *w, int M, int C, int K, double *sigma, int32_t *rank, double *v, hipStream_t s)
{
    if (K < 1 || K * K > kMaxN) return GDWS_EUNSUPPORTED;
    SvdParams p;
    p.w = w; p.sigma = sigma; p.rank = rank; p.v = v;
    p.M = M; p.C = C; p.n = K * K; p.R = M < K * K ? M : K * K;
    svd_gram_jacobi_kernel<<<dim3((unsigned)C), 64, 0, s>>>(p);
    GDWS_HIP_CHECK(hipGetLastError());
    return GDWS_OK;
}

}  // namespace gdws
