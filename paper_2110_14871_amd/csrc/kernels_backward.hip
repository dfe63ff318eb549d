// Backward pass of the GDWS layer through its linear part Y = PW(GDW(X)) + bias: the adjoints of the two operators
// of Section 3.1, for fine-tuning a GDWS network (the paper's Section 4 ablation).  General kernels on the vector
// ALUs (any storage type, layout, K, stride, padding), fp32 accumulation, deterministic (no atomics):
//   T, dT       the intermediate (recomputed) and its gradient dT[n,j,p] = sum_m Pw[m,j] dY[n,m,p], both fp32
//               [N][G][H'W'] in the caller's workspace; tiles of 64 pixels x 16 channels, dY through LDS
//   dPw[m,j]    = sum_{n,p} dY[n,m,p] T[n,j,p]           16 x 16 tiles of (m, j), the pixels staged through LDS
//   dbias[m]    = sum_{n,p} dY[n,m,p]
//   dD[j,u,v]   = sum_{n,y,x} dT[n,j,y,x] X[n,chan_of[j], y s + u - pad, x s + v - pad]     one workgroup per j
//   dX[n,c,y,x] = sum_{j in channel c} sum_{u,v} D[j,u,v] dT[n,j,(y + pad - u)/s,(x + pad - v)/s]   (where divisible)
#include "kernels.h"

namespace gdws {

namespace {

struct BwParams {
    const void *x, *dy;
    void *dx;
    float *g_dw, *g_pw, *g_bias;
    const float *dw, *pw;
    const int32_t *offsets, *chan_of;
    float *T, *dT;
    float *part;     // partial sums of the three reductions over pixels, one set per slab of pixels
    int slabs;       // slabs the N * H' * W' pixels are cut into (each reduction kernel's grid has that many layers)
    int64_t slab_q;  // pixels per slab
    int N, C, H, W, M, G, K, stride, pad, Ho, Wo;
    Strides sx, sy;  // element strides of x / dx and of dy
};

// T and dT for a tile of 64 pixels x 16 intermediate channels of one image.  dT is a small GEMM over the M output
// channels: dy goes through LDS in slices of 32 channels (read along its contiguous dimension in NHWC), the weights
// likewise; a thread owns one pixel and four intermediate channels.
template <typename E>
__global__ __launch_bounds__(256) void bw_intermediates_kernel(BwParams p)
{
    __shared__ float sY[64][33], sP[32][16];
    const int64_t P = (int64_t)p.Ho * p.Wo;
    const int n = blockIdx.z, p0 = blockIdx.x * 64, j0 = blockIdx.y * 16;
    const int px = threadIdx.x % 64, jg = threadIdx.x / 64;
    const int64_t pix = p0 + px;
    const bool pix_in = pix < P;
    const int oy = (int)(pix / p.Wo), ox = (int)(pix % p.Wo);
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    for (int m0 = 0; m0 < p.M; m0 += 32) {
        __syncthreads();
        for (int e = threadIdx.x; e < 64 * 32; e += 256) {
            const int r = e / 32, mm = e % 32;
            const int64_t q = p0 + r;
            float v = 0.f;
            if (q < P && m0 + mm < p.M)
                v = elem<E>::ld((const E *)p.dy + n * p.sy.n + (m0 + mm) * p.sy.c + (q / p.Wo) * p.sy.y + (q % p.Wo) * p.sy.x);
            sY[r][mm] = v;
        }
        for (int e = threadIdx.x; e < 32 * 16; e += 256) {
            const int mm = e / 16, jj = e % 16;
            sP[mm][jj] = (m0 + mm < p.M && j0 + jj < p.G) ? p.pw[(int64_t)(m0 + mm) * p.G + j0 + jj] : 0.f;
        }
        __syncthreads();
#pragma unroll 8
        for (int mm = 0; mm < 32; ++mm) {
            const float y = sY[px][mm];
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[i] += y * sP[mm][jg * 4 + i];
        }
    }
    if (!pix_in) return;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int j = j0 + jg * 4 + i;
        if (j >= p.G) break;
        const int64_t o = ((int64_t)n * p.G + j) * P + pix;
        p.dT[o] = acc[i];
        const int c = p.chan_of[j];
        const E *xs = (const E *)p.x + n * p.sx.n + c * p.sx.c;
        float t = 0.f;
        for (int u = 0; u < p.K; ++u)
            for (int v = 0; v < p.K; ++v) {
                const int iy = oy * p.stride + u - p.pad, ix = ox * p.stride + v - p.pad;
                if (iy >= 0 && iy < p.H && ix >= 0 && ix < p.W)
                    t += p.dw[((int64_t)j * p.K + u) * p.K + v] * elem<E>::ld(xs + iy * p.sx.y + ix * p.sx.x);
            }
        p.T[o] = t;
    }
}

template <typename E>
__global__ __launch_bounds__(256) void bw_dpw_kernel(BwParams p)
{
    __shared__ float sT[16][65], sY[16][65];
    const int tj = threadIdx.x % 16, tm = threadIdx.x / 16;
    const int j0 = blockIdx.x * 16, m0 = blockIdx.y * 16;
    const int64_t P = (int64_t)p.Ho * p.Wo, Qall = (int64_t)p.N * P;
    const int64_t qb = blockIdx.z * p.slab_q, Q = qb + p.slab_q < Qall ? qb + p.slab_q : Qall;
    float acc = 0.f;
    for (int64_t q0 = qb; q0 < Q; q0 += 64) {
        __syncthreads();
        for (int e = threadIdx.x; e < 16 * 64; e += 256) {
            const int r = e / 64, k = e % 64;
            const int64_t q = q0 + k;
            float tv = 0.f, yv = 0.f;
            if (q < Q) {
                const int64_t n = q / P, pix = q % P;
                if (j0 + r < p.G) tv = p.T[(n * p.G + j0 + r) * P + pix];
                if (m0 + r < p.M) {
                    const int oy = (int)(pix / p.Wo), ox = (int)(pix % p.Wo);
                    yv = elem<E>::ld((const E *)p.dy + n * p.sy.n + (m0 + r) * p.sy.c + oy * p.sy.y + ox * p.sy.x);
                }
            }
            sT[r][k] = tv; sY[r][k] = yv;
        }
        __syncthreads();
#pragma unroll 16
        for (int k = 0; k < 64; ++k) acc += sY[tm][k] * sT[tj][k];
    }
    if (m0 + tm < p.M && j0 + tj < p.G)
        p.part[(int64_t)blockIdx.z * ((int64_t)p.M * p.G) + (int64_t)(m0 + tm) * p.G + j0 + tj] = acc;
}

// sum over the workgroup of one value per thread (256 threads); the result is valid in thread 0
__device__ inline float block_sum(float v, float *red)
{
    __syncthreads();
    red[threadIdx.x] = v;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
        __syncthreads();
    }
    return red[0];
}

template <typename E>
__global__ __launch_bounds__(256) void bw_dbias_kernel(BwParams p)
{
    __shared__ float red[256];
    const int m = blockIdx.x;
    const int64_t P = (int64_t)p.Ho * p.Wo, Qall = (int64_t)p.N * P;
    const int64_t qb = blockIdx.z * p.slab_q, Q = qb + p.slab_q < Qall ? qb + p.slab_q : Qall;
    float acc = 0.f;
    for (int64_t q = qb + threadIdx.x; q < Q; q += 256) {
        const int64_t n = q / P, pix = q % P;
        const int oy = (int)(pix / p.Wo), ox = (int)(pix % p.Wo);
        acc += elem<E>::ld((const E *)p.dy + n * p.sy.n + m * p.sy.c + oy * p.sy.y + ox * p.sy.x);
    }
    const float s = block_sum(acc, red);
    if (threadIdx.x == 0) p.part[(int64_t)p.slabs * ((int64_t)p.M * p.G + (int64_t)p.G * p.K * p.K) + (int64_t)blockIdx.z * p.M + m] = s;
}

template <typename E>
__global__ __launch_bounds__(256) void bw_ddw_kernel(BwParams p)
{
    __shared__ float red[256];
    const int j = blockIdx.x, c = p.chan_of[j];
    const int64_t P = (int64_t)p.Ho * p.Wo, Qall = (int64_t)p.N * P;
    const int64_t qb = blockIdx.z * p.slab_q, Q = qb + p.slab_q < Qall ? qb + p.slab_q : Qall;
    float *out = p.part + (int64_t)p.slabs * ((int64_t)p.M * p.G) + (int64_t)blockIdx.z * ((int64_t)p.G * p.K * p.K);
    for (int u = 0; u < p.K; ++u)
        for (int v = 0; v < p.K; ++v) {
            float acc = 0.f;
            for (int64_t q = qb + threadIdx.x; q < Q; q += 256) {
                const int64_t n = q / P, pix = q % P;
                const int oy = (int)(pix / p.Wo), ox = (int)(pix % p.Wo);
                const int iy = oy * p.stride + u - p.pad, ix = ox * p.stride + v - p.pad;
                if (iy >= 0 && iy < p.H && ix >= 0 && ix < p.W)
                    acc += p.dT[(n * p.G + j) * P + pix] *
                           elem<E>::ld((const E *)p.x + n * p.sx.n + c * p.sx.c + iy * p.sx.y + ix * p.sx.x);
            }
            const float s = block_sum(acc, red);
            if (threadIdx.x == 0) out[((int64_t)j * p.K + u) * p.K + v] = s;
        }
}

template <typename E>
__global__ __launch_bounds__(256) void bw_dx_kernel(BwParams p)
{
    const int64_t total = (int64_t)p.N * p.C * p.H * p.W;
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    // (x fastest, then y, c, n: the reads of dT run along its rows)
    const int ix = (int)(i % p.W), iy = (int)((i / p.W) % p.H), c = (int)((i / ((int64_t)p.W * p.H)) % p.C);
    const int64_t n = i / ((int64_t)p.W * p.H * p.C), P = (int64_t)p.Ho * p.Wo;
    float acc = 0.f;
    for (int j = p.offsets[c]; j < p.offsets[c + 1]; ++j)
        for (int u = 0; u < p.K; ++u) {
            const int yy = iy + p.pad - u;
            if (yy < 0 || yy % p.stride) continue;
            const int oy = yy / p.stride;
            if (oy >= p.Ho) continue;
            for (int v = 0; v < p.K; ++v) {
                const int xx = ix + p.pad - v;
                if (xx < 0 || xx % p.stride) continue;
                const int ox = xx / p.stride;
                if (ox >= p.Wo) continue;
                acc += p.dw[((int64_t)j * p.K + u) * p.K + v] * p.dT[(n * p.G + j) * P + (int64_t)oy * p.Wo + ox];
            }
        }
    elem<E>::st((E *)p.dx + n * p.sx.n + c * p.sx.c + iy * p.sx.y + ix * p.sx.x, acc);
}

// dst[i] = sum over the slabs of part[slab][i], in slab order (deterministic)
__global__ __launch_bounds__(256) void bw_sum_slabs_kernel(const float *part, float *dst, int64_t count, int slabs)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= count) return;
    float acc = 0.f;
    for (int k = 0; k < slabs; ++k) acc += part[(int64_t)k * count + i];
    dst[i] = acc;
}

template <typename E>
int launch_bw(const BwParams &p, hipStream_t s)
{
    const int64_t P = (int64_t)p.Ho * p.Wo;
    if ((P + 63) / 64 >= ((int64_t)1 << 31) || p.N > 65535 || (p.G + 15) / 16 > 65535) return GDWS_EUNSUPPORTED;
    bw_intermediates_kernel<E><<<dim3((unsigned)((P + 63) / 64), (unsigned)((p.G + 15) / 16), (unsigned)p.N), 256, 0, s>>>(p);
    const unsigned z = (unsigned)p.slabs;
    const int64_t n_pw = (int64_t)p.M * p.G, n_dw = (int64_t)p.G * p.K * p.K;
    if (p.g_pw) {
        bw_dpw_kernel<E><<<dim3((unsigned)((p.G + 15) / 16), (unsigned)((p.M + 15) / 16), z), 256, 0, s>>>(p);
        bw_sum_slabs_kernel<<<dim3((unsigned)((n_pw + 255) / 256)), 256, 0, s>>>(p.part, p.g_pw, n_pw, p.slabs);
    }
    if (p.g_dw) {
        bw_ddw_kernel<E><<<dim3((unsigned)p.G, 1, z), 256, 0, s>>>(p);
        bw_sum_slabs_kernel<<<dim3((unsigned)((n_dw + 255) / 256)), 256, 0, s>>>(p.part + p.slabs * n_pw, p.g_dw, n_dw,
                                                                               p.slabs);
    }
    if (p.g_bias) {
        bw_dbias_kernel<E><<<dim3((unsigned)p.M, 1, z), 256, 0, s>>>(p);
        bw_sum_slabs_kernel<<<dim3((unsigned)((p.M + 255) / 256)), 256, 0, s>>>(p.part + p.slabs * (n_pw + n_dw), p.g_bias,
                                                                              p.M, p.slabs);
    }
    if (p.dx) {
        const int64_t nx = (int64_t)p.N * p.C * p.H * p.W;
        if ((nx + 255) / 256 >= ((int64_t)1 << 31)) return GDWS_EUNSUPPORTED;
        bw_dx_kernel<E><<<dim3((unsigned)((nx + 255) / 256)), 256, 0, s>>>(p);
    }
    GDWS_HIP_CHECK(hipGetLastError());
    return GDWS_OK;
}

}  // namespace

// Slabs of pixels for the three reductions: about 1024 pixels each, at most 256 of them.
static int backward_slabs(int64_t Q)
{
    const int64_t s = (Q + 1023) / 1024;
    return (int)(s < 1 ? 1 : s > 256 ? 256 : s);
}

size_t backward_workspace_bytes(int N, int M, int G, int K, int Ho, int Wo)
{
    const int64_t Q = (int64_t)N * Ho * Wo;
    return ((size_t)2 * Q * G + (size_t)backward_slabs(Q) * ((size_t)M * G + (size_t)G * K * K + M)) * sizeof(float);
}

int launch_backward(const BackwardArgs &a, hipStream_t s)
{
    BwParams p;
    p.x = a.x; p.dy = a.dy; p.dx = a.dx; p.g_dw = a.g_dw; p.g_pw = a.g_pw; p.g_bias = a.g_bias;
    p.dw = a.dw; p.pw = a.pw; p.offsets = a.offsets; p.chan_of = a.chan_of;
    const size_t nt = (size_t)a.N * a.G * a.Ho * a.Wo;
    p.T = (float *)a.workspace; p.dT = p.T + nt; p.part = p.dT + nt;
    const int64_t Q = (int64_t)a.N * a.Ho * a.Wo;
    p.slabs = backward_slabs(Q);
    p.slab_q = ((Q + p.slabs - 1) / p.slabs + 63) / 64 * 64;  // whole 64-pixel steps of the dPw kernel
    p.N = a.N; p.C = a.C; p.H = a.H; p.W = a.W; p.M = a.M; p.G = a.G; p.K = a.K; p.stride = a.stride; p.pad = a.pad;
    p.Ho = a.Ho; p.Wo = a.Wo;
    p.sx = make_strides(a.layout, a.C, a.H, a.W);
    p.sy = make_strides(a.layout, a.M, a.Ho, a.Wo);
    switch (a.dtype) {
        case GDWS_F32: return launch_bw<float>(p, s);
        case GDWS_F16: return launch_bw<f16_t>(p, s);
        case GDWS_BF16: return launch_bw<bf16_t>(p, s);
        default: return GDWS_EINVAL;
    }
}

}  // namespace gdws
