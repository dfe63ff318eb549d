// Standard 3 x 3 convolution (eq. 1, the layer a GDWS convolution approximates) as an implicit GEMM on the matrix
// cores: 16-bit storage, NHWC, pad 1, stride 1, C a multiple of 16.
//     Y[p][m] = bias[m] + sum over taps (u, v) and channels c of W[m][c][u][v] * X[p + (u, v) - 1][c]
// The contraction runs over (16-channel window, tap): one v_mfma_f32_32x32x16 per window, tap, 32 output channels and
// 32 pixels.  A workgroup of four waves owns a tile of 256 output pixels (TH x TW of one image) and up to 128 output
// channels; a wave owns 64 of the pixels.  The input tile with its halo goes through LDS in chunks of 64 channels,
// pixel-major, double-buffered: the loads of the next chunk are issued before the MFMAs of the current one and
// written to the other buffer after them.  The B operand (16 channels of a pixel, shifted by the tap) is one aligned
// 16-byte LDS read; the A operand (weights) comes from a copy of W repacked in operand order by a small kernel at the
// start of every call (W arrives as a plain [M][C][3][3] device tensor), into the caller's workspace.
// Epilogue: bias in the accumulators' start values, residual add and ReLU in registers, one rounding, and the tile
// goes through LDS so that the stores are 16 bytes per lane.
#include <algorithm>

#include "fused_kernel.h"
#include "kernels.h"

namespace gdws {

using namespace fusedk;

namespace {

constexpr int kCC = 64;              // channels per chunk
constexpr int kPSW = kCC / 2 + 4;    // dwords per pixel in LDS (16 bytes of padding: conflict-free 16-byte reads)
constexpr int kTilePx = 256;
constexpr int kMaxPieces = 11;       // 16-byte pieces of a chunk per thread: ceil(340 pixels * 8 pieces / 256 threads)

struct ConvParams {
    const uint16_t *x;
    uint16_t *y;
    const uint16_t *residual;
    const float *bias;        // [M] or nullptr
    const u32x4_t *frag;      // [C / 16][9][m_blocks_pad][64 lanes]
    int N, C, H, W, M, relu;
    int TH, tiles_x, tiles_y, m_blocks_pad;
    uint32_t x_bytes;
};

struct RepackParams {
    const uint16_t *w;  // [M][C][3][3]
    u32x4_t *frag;
    int M, C, m_blocks_pad, total;
};

// frag[((cw * 9 + tap) * m_blocks_pad + mb) * 64 + lane], element e  <->  W[mb * 32 + lane % 32][cw * 16 + 8 * (lane / 32) + e][tap]
__global__ void conv_repack_kernel(RepackParams p)
{
    const int f = blockIdx.x * blockDim.x + threadIdx.x;
    if (f >= p.total) return;
    const int lane = f & 63, mb = (f >> 6) % p.m_blocks_pad, r = (f >> 6) / p.m_blocks_pad;
    const int tap = r % 9, cw = r / 9;
    const int m = mb * 32 + (lane & 31), c0 = cw * 16 + 8 * (lane >> 5);
    uint32_t h[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) h[e] = m < p.M ? p.w[((int64_t)m * p.C + c0 + e) * 9 + tap] : 0u;
    p.frag[f] = u32x4_t{h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16)};
}

template <int DTYPE, int TW, int MB>
__global__ __launch_bounds__(256, 1) void conv3x3_mfma_kernel(ConvParams p)
{
    using Op = half_ops<DTYPE>;
    constexpr int IW = TW + 2;
    constexpr uint32_t kOutside = 0x80000000u;
    extern __shared__ uint32_t lds[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, t = threadIdx.x;
    const int l32 = lane & 31, lhi = lane >> 5;
    const int TH = p.TH, IH = TH + 2, npix = IH * IW;
    const int stage_w = ((npix * (kCC / 8) + 255) / 256 * 256 / (kCC / 8)) * kPSW;  // whole passes of the loader
    int tile = blockIdx.x;
    const int tx0 = (tile % p.tiles_x) * TW; tile /= p.tiles_x;
    const int ty0 = (tile % p.tiles_y) * TH;
    const int n = tile / p.tiles_y;
    const int mbase = blockIdx.y * MB;

    // ---- loader: a thread owns up to kMaxPieces 16-byte pieces (8 channels of a pixel) of every chunk ----
    constexpr int QC = kCC / 8;
    const int npieces = (npix * QC + 255) / 256;
    uint32_t voff[kMaxPieces];
    const uint32_t c2 = (uint32_t)p.C * 2u;
#pragma unroll
    for (int k = 0; k < kMaxPieces; ++k) {
        const int id = t + 256 * k, pix = id / QC, q = id % QC;
        const int iy = pix / IW, ix = pix % IW;
        const int gy = ty0 - 1 + iy, gx = tx0 - 1 + ix;
        const bool in = pix < npix && (unsigned)gy < (unsigned)p.H && (unsigned)gx < (unsigned)p.W;
        voff[k] = in ? (uint32_t)(((n * p.H + gy) * p.W + gx)) * c2 + q * 16 : kOutside;
    }
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)p.x, 0, p.x_bytes, 0x00020000);
    u32x4_t ld[kMaxPieces];
    auto issue = [&](int chunk) {
        const int c0 = chunk * kCC;
#pragma unroll
        for (int k = 0; k < kMaxPieces; ++k)
            if (k < npieces) {
                // channels past C (the last chunk of a layer whose C is not a multiple of 64) read as zeros
                const int q = (t + 256 * k) % QC;
                const uint32_t gone = c0 + q * 8 < p.C ? 0u : kOutside;
                ld[k] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, voff[k] | gone, c0 * 2, 0);
            }
    };
    auto deposit = [&](int buf) {
#pragma unroll
        for (int k = 0; k < kMaxPieces; ++k)
            if (k < npieces) {
                const int id = t + 256 * k;
                *(u32x4_t *)(lds + buf * stage_w + (id / QC) * kPSW + (id % QC) * 4) = ld[k];
            }
    };

    // ---- accumulators start from the bias: D[m][pixel], register i <-> channel 8*(i/4) + 4*lhi + i%4 ----
    f32x16_t acc[2][MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int m = (mbase + mb) * 32 + 8 * (i / 4) + 4 * lhi + i % 4;
            const float b = (p.bias && m < p.M) ? p.bias[m] : 0.f;
            acc[0][mb][i] = b;
            acc[1][mb][i] = b;
        }
    int base[2];
#pragma unroll
    for (int pb = 0; pb < 2; ++pb) {
        const int pp = wave * 64 + pb * 32 + l32;
        base[pb] = ((pp / TW) * IW + pp % TW) * kPSW + lhi * 4;
    }

    const int nchunks = (p.C + kCC - 1) / kCC;
    const int fstride = p.m_blocks_pad * 64;
    const u32x4_t *fp = p.frag + (int64_t)mbase * 64 + lane;
    // The weights of a step (one window, one tap: MB fragments of 16 bytes per lane) are requested three steps
    // before their MFMAs, into a ring of three register sets: an L2 round trip is several hundred cycles, a step's
    // eight MFMAs are 256.
    constexpr int kRing = 3;
    const int nsteps = (p.C / 16) * 9;
    u32x4_t a[kRing][MB];
    auto fetch = [&](int slot, int step) {
        const u32x4_t *fw = fp + (int64_t)(step < nsteps ? step : nsteps - 1) * fstride;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) a[slot][mb] = fw[mb * 64];
    };
#pragma unroll
    for (int k = 0; k < kRing; ++k) fetch(k, k);
    issue(0);
    deposit(0);
    __syncthreads();
    int step = 0;
    for (int chunk = 0; chunk < nchunks; ++chunk) {
        if (chunk + 1 < nchunks) issue(chunk + 1);
        const uint32_t *buf = lds + (chunk & 1) * stage_w;
        const int nwin = std::min(kCC, p.C - chunk * kCC) / 16;
        for (int win = 0; win < nwin; ++win) {
#pragma unroll
            for (int tap = 0; tap < 9; ++tap) {
                u32x4_t b[2];
#pragma unroll
                for (int pb = 0; pb < 2; ++pb)
                    b[pb] = *(const u32x4_t *)(buf + base[pb] + ((tap / 3) * IW + tap % 3) * kPSW + win * 8);
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                    for (int pb = 0; pb < 2; ++pb) acc[pb][mb] = Op::mfma(a[tap % kRing][mb], b[pb], acc[pb][mb]);
                fetch(tap % kRing, step + tap + kRing);
            }
            step += 9;
        }
        if (chunk + 1 < nchunks) deposit((chunk + 1) & 1);
        __syncthreads();  // the next chunk is in LDS, and every wave is done with this one
    }

    // ---- epilogue: residual and ReLU in registers, rounding, tile -> LDS -> global in 16-byte pieces ----
    constexpr int kRowHalfs = MB * 32 + 8;
    uint16_t *tile16 = (uint16_t *)lds;
    int *pixtab = (int *)(tile16 + kTilePx * kRowHalfs);
    {
        const int op = t, ox = tx0 + op % TW, oy = ty0 + op / TW;
        pixtab[op] = (oy < p.H && ox < p.W) ? (n * p.H + oy) * p.W + ox : -1;
    }
#pragma unroll
    for (int pb = 0; pb < 2; ++pb) {
        const int pp = wave * 64 + pb * 32 + l32;
        const int ox = tx0 + pp % TW, oy = ty0 + pp / TW;
        const bool live = oy < p.H && ox < p.W;
        const int64_t po = (int64_t)((n * p.H + oy) * p.W + ox) * p.M;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                float v[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) v[i] = acc[pb][mb][4 * q4 + i];
                const int m0 = (mbase + mb) * 32 + 8 * q4 + 4 * lhi;
                if (p.residual && live) {
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if (m0 + i < p.M) v[i] += Op::widen(p.residual[po + m0 + i]);
                }
                if (p.relu) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) v[i] = relu_bits(v[i]);
                }
                *(u32x2_t *)(tile16 + pp * kRowHalfs + mb * 32 + 8 * q4 + 4 * lhi) =
                    u32x2_t{Op::pack(v[0], v[1]), Op::pack(v[2], v[3])};
            }
    }
    __syncthreads();
    constexpr int kParts = MB * 4;  // 16-byte pieces per pixel
    const int part = t % kParts;
    const int mch = mbase * 32 + part * 8;
    const bool whole = mch + 7 < p.M && (p.M & 7) == 0;
    for (int op = t / kParts; op < kTilePx; op += 256 / kParts) {
        const int po = pixtab[op];
        if (po < 0 || mch >= p.M) continue;
        const int64_t o = (int64_t)po * p.M + mch;
        if (whole) {
            __builtin_nontemporal_store(*(const u32x4_t *)(tile16 + op * kRowHalfs + part * 8), (u32x4_t *)(p.y + o));
        } else {
            for (int i = 0; i < 8 && mch + i < p.M; ++i) p.y[o + i] = tile16[op * kRowHalfs + part * 8 + i];
        }
    }
}

template <int DTYPE, int TW, int MB>
int launch_conv_instance(const ConvParams &p, dim3 grid, size_t lds_bytes, hipStream_t s)
{
    auto kern = conv3x3_mfma_kernel<DTYPE, TW, MB>;
    static bool raised = false;
    if (!raised) {
        GDWS_HIP_CHECK(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
        raised = true;
    }
    kern<<<grid, 256, lds_bytes, s>>>(p);
    GDWS_HIP_CHECK(hipGetLastError());
    return GDWS_OK;
}

}  // namespace

bool conv_mfma_supported(int dtype, int layout, int K, int stride, int pad, int C, int64_t x_elems)
{
    return (dtype == GDWS_BF16 || dtype == GDWS_F16) && layout == GDWS_NHWC && K == 3 && stride == 1 && pad == 1 &&
           C >= 16 && C % 16 == 0 && x_elems * 2 < ((int64_t)1 << 31);
}

size_t conv_mfma_workspace_bytes(int C, int M)
{
    const int m_blocks = (M + 31) / 32, mb = m_blocks >= 3 ? 4 : 2;
    const int m_blocks_pad = (m_blocks + mb - 1) / mb * mb;
    return (size_t)(C / 16) * 9 * m_blocks_pad * 64 * 16;
}

int launch_conv_mfma(const DenseArgs &a, void *workspace, hipStream_t s)
{
    const int m_blocks = (a.M + 31) / 32, mb = m_blocks >= 3 ? 4 : 2;
    const int m_blocks_pad = (m_blocks + mb - 1) / mb * mb;
    RepackParams r;
    r.w = (const uint16_t *)a.w; r.frag = (u32x4_t *)workspace; r.M = a.M; r.C = a.C; r.m_blocks_pad = m_blocks_pad;
    r.total = (a.C / 16) * 9 * m_blocks_pad * 64;
    conv_repack_kernel<<<(r.total + 255) / 256, 256, 0, s>>>(r);
    GDWS_HIP_CHECK(hipGetLastError());

    ConvParams p;
    p.x = (const uint16_t *)a.x; p.y = (uint16_t *)a.y; p.residual = (const uint16_t *)a.ep.residual;
    p.bias = a.ep.bias; p.frag = (const u32x4_t *)workspace;
    p.N = a.N; p.C = a.C; p.H = a.H; p.W = a.W; p.M = a.M; p.relu = a.ep.relu;
    p.m_blocks_pad = m_blocks_pad;
    p.x_bytes = (uint32_t)((int64_t)a.N * a.C * a.H * a.W * 2);
    const int TW = a.W <= 8 ? 8 : 16;
    p.TH = kTilePx / TW;
    p.tiles_x = (a.W + TW - 1) / TW;
    p.tiles_y = (a.H + p.TH - 1) / p.TH;
    const int npix = (p.TH + 2) * (TW + 2);
    const int stage_w = ((npix * (kCC / 8) + 255) / 256 * 256 / (kCC / 8)) * kPSW;
    const size_t lds = std::max((size_t)2 * stage_w * 4, (size_t)kTilePx * (mb * 32 + 8) * 2 + kTilePx * 4);
    const dim3 grid((unsigned)((int64_t)p.tiles_x * p.tiles_y * a.N), (unsigned)(m_blocks_pad / mb));
#define GDWS_CONV_CASE(dt, tw, m) \
    if (a.dtype == dt && TW == tw && mb == m) return launch_conv_instance<dt, tw, m>(p, grid, lds, s);
    GDWS_CONV_CASE(GDWS_BF16, 16, 4) GDWS_CONV_CASE(GDWS_BF16, 16, 2) GDWS_CONV_CASE(GDWS_BF16, 8, 4) GDWS_CONV_CASE(GDWS_BF16, 8, 2)
    GDWS_CONV_CASE(GDWS_F16, 16, 4) GDWS_CONV_CASE(GDWS_F16, 16, 2) GDWS_CONV_CASE(GDWS_F16, 8, 4) GDWS_CONV_CASE(GDWS_F16, 8, 2)
#undef GDWS_CONV_CASE
    return GDWS_EUNSUPPORTED;
}

}  // namespace gdws
