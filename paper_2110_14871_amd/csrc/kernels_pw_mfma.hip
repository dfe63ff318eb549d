// Pointwise stage as a GEMM on the matrix cores (16-bit storage, NHWC; an fp32 kernel for either layout is at
// the end of the file):
//     Y[p][m] = bias[m] + sum_j Pw[m][j] * T[p][j]          (1 x 1 convolution, G -> M channels)
// T is the intermediate of the unfused path: [pixels][Gp] with Gp = G rounded up to 16 (the surplus
// channels are zero), so the 8 consecutive channels a lane needs for the B operand of
// v_mfma_f32_32x32x16 are one aligned 16-byte global load -- no staging through LDS.  A workgroup of
// four waves owns 256 pixels and up to 128 output channels; a wave owns 64 pixels (two 32-pixel
// blocks) and keeps the 64 x 128 fp32 accumulator tile in registers.  The weights are packed at plan
// time per K-step (16 channels) and 32-wide block of M in the lane order of the A operand.  The
// kernel is bound by the HBM traffic of T and Y; loads run four K-steps ahead of their use.
#include "fused_kernel.h"
#include "kernels.h"

namespace gdws {

using namespace fusedk;

namespace {

struct PwParams {
    const uint16_t *t;
    uint16_t *y;
    const uint16_t *residual;
    const float *bias;      // padded to whole 32-channel blocks
    const u32x4_t *frag;    // [ksteps][m_blocks_pad][64 lanes]
    int P, Gp, M, ksteps, m_blocks_pad, relu;
    int stride, Ho, Wo, H, W;  // stride > 1: output pixel (n, oy, ox) reads input pixel (n, oy*stride, ox*stride)
    int n_slices, n_tiles;     // slices of MB*32 output channels; pixel tiles; work items = tiles x slices
};

constexpr int kAhead = 3;      // K-steps between a load and its use
constexpr int kWavesPerSimd = 2;  // the registers are bounded for this many (256 each): eight waves per CU

// WAVES: waves per workgroup, each with 64 pixels of the tile (4: 256-pixel tiles; 2: 128-pixel tiles, twice as many
// workgroups per CU -- for launches with so few tiles that they would otherwise keep too few loads in flight).
template <int DTYPE, int MB, int WAVES>
__global__ __launch_bounds__(64 * WAVES, kWavesPerSimd) void pw_mfma_kernel(PwParams p)
{
    constexpr int kTilePx = 64 * WAVES, kWgThreads = 64 * WAVES;
    using Op = half_ops<DTYPE>;
    extern __shared__ uint32_t lds[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l32 = lane & 31, lhi = lane >> 5;
    const int t = threadIdx.x;
    const int fstride = p.m_blocks_pad * 64;

    // A workgroup walks over work items (a tile of 256 pixels x a slice of MB*32 output channels).  The first loads
    // of the next item are issued before the epilogue of the current one, which then runs while they are in flight.
    // Order: consecutive workgroup ids run on consecutive XCDs, each with an L2 of its own, so a tile's slices must
    // meet on one XCD for T to be fetched from HBM once: XCD x (workgroups x, x + 8, ...) owns tiles x, x + 8, ...;
    // its workgroups walk over that list slice by slice, so neighbours in the list run at the same time.
    const u32x4_t *tp[2];
    const u32x4_t *fp;
    u32x4_t b[kAhead][2], a[kAhead][MB];
    const int xcd = blockIdx.x & 7, wgs_per_xcd = gridDim.x >> 3;  // (the grid is a multiple of 8)
    const int n_items = p.n_tiles > xcd ? ((p.n_tiles - xcd + 7) >> 3) * p.n_slices : 0;  // of this XCD
    auto tile_of = [&](int item) { return xcd + 8 * (item / p.n_slices); };
    auto start_item = [&](int item) {
        const int64_t p0 = (int64_t)tile_of(item) * kTilePx;
        // the lane's two pixels (clamped: the results of pixels past the end are dropped at the store)
#pragma unroll
        for (int pb = 0; pb < 2; ++pb) {
            int64_t px = p0 + wave * 64 + pb * 32 + l32;
            if (px >= p.P) px = p.P - 1;
            if (p.stride > 1) {  // a strided 1 x 1 convolution: gather the input pixel
                const int ox = (int)(px % p.Wo), oy = (int)((px / p.Wo) % p.Ho);
                const int64_t n = px / ((int64_t)p.Wo * p.Ho);
                px = (n * p.H + (int64_t)oy * p.stride) * p.W + (int64_t)ox * p.stride;
            }
            tp[pb] = (const u32x4_t *)(p.t + px * p.Gp + lhi * 8);
        }
        fp = p.frag + (int64_t)(item % p.n_slices) * MB * 64 + lane;
#pragma unroll
        for (int u = 0; u < kAhead; ++u) {
            if (u < p.ksteps) {
#pragma unroll
                for (int pb = 0; pb < 2; ++pb) b[u][pb] = tp[pb][2 * u];
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) a[u][mb] = fp[u * fstride + mb * 64];
            }
        }
    };

    int item = blockIdx.x >> 3;
    if (item >= n_items) return;  // (the whole workgroup: before any barrier)
    start_item(item);
    while (true) {
        const int mbase = (item % p.n_slices) * MB;
        const int64_t p0 = (int64_t)tile_of(item) * kTilePx;
        f32x16_t acc[2][MB];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            const float *bp = p.bias + (mbase + mb) * 32;  // D[m][pixel]: register i <-> channel 8*(i/4) + 4*lhi + i%4
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const f32x4_t bv = *(const f32x4_t *)(bp + 8 * q4 + 4 * lhi);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    acc[0][mb][4 * q4 + i] = bv[i];
                    acc[1][mb][4 * q4 + i] = bv[i];
                }
            }
        }
        for (int s0 = 0; s0 < p.ksteps; s0 += kAhead) {
#pragma unroll
            for (int u = 0; u < kAhead; ++u) {
                const int s = s0 + u;
                if (s < p.ksteps) {
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb) {
                        acc[0][mb] = Op::mfma(a[u][mb], b[u][0], acc[0][mb]);
                        acc[1][mb] = Op::mfma(a[u][mb], b[u][1], acc[1][mb]);
                    }
                    if (s + kAhead < p.ksteps) {
#pragma unroll
                        for (int pb = 0; pb < 2; ++pb) b[u][pb] = tp[pb][2 * (s + kAhead)];
#pragma unroll
                        for (int mb = 0; mb < MB; ++mb) a[u][mb] = fp[(s + kAhead) * fstride + mb * 64];
                    }
                }
            }
        }
        const int next = item + wgs_per_xcd;
        const bool more = next < n_items;
        if (more) start_item(next);

        // ---- epilogue: the tile goes through LDS so that the stores are 16 bytes per lane and coalesced ----
        // Without a residual: [256 pixels][MB*32 channels] in the storage type (final values), rows padded by 16
        // bytes.  With one: fp32 (the residual is added before the only rounding), in two halves of the output
        // channels one after the other, so that the tile stays under 80 KB and two workgroups fit a CU.
        if (!p.residual) {
            constexpr int kRowHalfs = MB * 32 + 8;
            uint16_t *tile16 = (uint16_t *)lds;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
                    for (int q4 = 0; q4 < 4; ++q4) {
                        f32x4_t v;
#pragma unroll
                        for (int i = 0; i < 4; ++i) v[i] = acc[h][mb][4 * q4 + i];
                        const int row = wave * 64 + h * 32 + l32, col = mb * 32 + 8 * q4 + 4 * lhi;
                        if (p.relu) {
#pragma unroll
                            for (int i = 0; i < 4; ++i) v[i] = relu_bits(v[i]);
                        }
                        *(u32x2_t *)(tile16 + row * kRowHalfs + col) =
                            u32x2_t{Op::pack(v[0], v[1]), Op::pack(v[2], v[3])};
                    }
                }
            }
            __syncthreads();
            constexpr int kParts = MB * 4;  // 16-byte pieces per pixel
            const int part = t % kParts;
            const int mch = mbase * 32 + part * 8;
            const bool whole = mch + 7 < p.M && (p.M & 7) == 0;
            for (int op = t / kParts; op < kTilePx; op += kWgThreads / kParts) {
                const int64_t px = p0 + op;
                if (px >= p.P || mch >= p.M) continue;
                const int64_t o = px * p.M + mch;
                const uint16_t *src = tile16 + op * kRowHalfs + part * 8;
                if (whole) {
                    __builtin_nontemporal_store(*(const u32x4_t *)src, (u32x4_t *)(p.y + o));  // y is not read again here
                } else {
                    for (int i = 0; i < 8 && mch + i < p.M; ++i) p.y[o + i] = src[i];
                }
            }
        } else {
            constexpr int HB = MB / 2;               // 32-wide blocks per half
            constexpr int kRowFloats = HB * 32 + 4;
            float *tile32 = (float *)lds;
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                if (half) __syncthreads();  // the first half has been read out
#pragma unroll
                for (int h = 0; h < 2; ++h) {
#pragma unroll
                    for (int mbl = 0; mbl < HB; ++mbl) {
#pragma unroll
                        for (int q4 = 0; q4 < 4; ++q4) {
                            f32x4_t v;
#pragma unroll
                            for (int i = 0; i < 4; ++i) v[i] = acc[h][half * HB + mbl][4 * q4 + i];
                            const int row = wave * 64 + h * 32 + l32, col = mbl * 32 + 8 * q4 + 4 * lhi;
                            *(f32x4_t *)(tile32 + row * kRowFloats + col) = v;
                        }
                    }
                }
                __syncthreads();
                constexpr int kParts = HB * 4;  // 16-byte pieces of y per pixel and half
                const int part = t % kParts;
                const int mch = (mbase + half * HB) * 32 + part * 8;
                const bool whole = mch + 7 < p.M && (p.M & 7) == 0;
                constexpr int kStep = kWgThreads / kParts, kIter = kTilePx / kStep;
                if ((p.M & 7) == 0) {
                    // the residual pieces of all the thread's pixels are requested first, unconditionally (from the
                    // start of the tensor where the thread has nothing to read), then consumed: one trip to memory
                    // for all of them instead of one per pixel
                    // (in batches: the registers hold the next item's first operands at this point)
                    static_assert(kIter % 2 == 0, "pixels per thread come in pairs");
                    constexpr int kBatch = 2;  // (measured: 2 beats 4 and 8, which spill)
#pragma unroll
                    for (int i0 = 0; i0 < kIter; i0 += kBatch) {
                        u32x4_t res[kBatch];
#pragma unroll
                        for (int i = 0; i < kBatch; ++i) {
                            const int64_t px = p0 + t / kParts + (i0 + i) * kStep;
                            const bool ok = px < p.P && mch < p.M;
                            res[i] = *(const u32x4_t *)(p.residual + (ok ? px * p.M + mch : 0));
                        }
#pragma unroll
                        for (int i = 0; i < kBatch; ++i) {
                            const int64_t px = p0 + t / kParts + (i0 + i) * kStep;
                            if (px >= p.P || mch >= p.M) continue;
                            const float *src = tile32 + (t / kParts + (i0 + i) * kStep) * kRowFloats + part * 8;
                            float v[8];
#pragma unroll
                            for (int e = 0; e < 8; ++e)
                                v[e] = src[e] + Op::widen((uint16_t)(res[i][e / 2] >> (16 * (e & 1))));
                            if (p.relu) {
#pragma unroll
                                for (int e = 0; e < 8; ++e) v[e] = relu_bits(v[e]);
                            }
                            __builtin_nontemporal_store(u32x4_t{Op::pack(v[0], v[1]), Op::pack(v[2], v[3]),
                                                                Op::pack(v[4], v[5]), Op::pack(v[6], v[7])},
                                                        (u32x4_t *)(p.y + px * p.M + mch));
                        }
                    }
                    continue;  // (the next half)
                }
                for (int op = t / kParts; op < kTilePx; op += kStep) {
                    const int64_t px = p0 + op;
                    if (px >= p.P || mch >= p.M) continue;
                    const int64_t o = px * p.M + mch;
                    const float *src = tile32 + op * kRowFloats + part * 8;
                    float v[8];
#pragma unroll
                    for (int i = 0; i < 8; ++i) v[i] = src[i];
                    if (whole) {
                        const u32x4_t r = *(const u32x4_t *)(p.residual + o);
#pragma unroll
                        for (int i = 0; i < 8; ++i) v[i] += Op::widen((uint16_t)(r[i / 2] >> (16 * (i & 1))));
                        if (p.relu) {
#pragma unroll
                            for (int i = 0; i < 8; ++i) v[i] = relu_bits(v[i]);
                        }
                        __builtin_nontemporal_store(u32x4_t{Op::pack(v[0], v[1]), Op::pack(v[2], v[3]),
                                                            Op::pack(v[4], v[5]), Op::pack(v[6], v[7])},
                                                    (u32x4_t *)(p.y + o));
                    } else {
                        for (int i = 0; i < 8 && mch + i < p.M; ++i) {
                            float w = v[i] + Op::widen(p.residual[o + i]);
                            if (p.relu) w = fmaxf(w, 0.f);
                            p.y[o + i] = (uint16_t)Op::pack(w, 0.f);
                        }
                    }
                }
            }
        }
        if (!more) break;
        item = next;
        __syncthreads();  // the tile in LDS has been read out
    }
}

// ---- fp32: v_mfma_f32_32x32x2_f32, either layout -----------------------------------------------
// D[m][pixel] += Pw[m][k] * T[pixel][k], two channels per MFMA: lane (l % 32, l / 32) holds one element of A
// (row m = l % 32, k = l / 32) and one of B (pixel l % 32, k = l / 32).  A wave owns 64 pixels x 64 output
// channels; operands come straight from global memory (fp32 layers are small: this path is about using the
// matrix cores at full precision, not about bandwidth).  Output element (m, pixel) of accumulator register i
// is row 8*(i/4) + 4*(l/32) + i%4, column l % 32.
struct PwF32Params {
    const float *t;
    float *y;
    const float *pw;        // [M][G]
    const float *bias;      // [M] or nullptr
    const float *residual;  // like y, or nullptr
    int relu, G, M;
    int64_t P, HW;          // pixels in all, per image
    Strides st, sy;         // element strides of T and of y (n, c, and the pixel stride in x)
};

__global__ __launch_bounds__(256) void pw_mfma_f32_kernel(PwF32Params p)
{
    constexpr int MBF = 2;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l32 = lane & 31, lhi = lane >> 5;
    const int m0 = blockIdx.y * MBF * 32;
    f32x16_t acc[2][MBF];
#pragma unroll
    for (int pb = 0; pb < 2; ++pb)
#pragma unroll
        for (int mb = 0; mb < MBF; ++mb)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[pb][mb][i] = 0.f;
    // pixel -> (image, position); a pixel's elements are at n*s.n + pos*s.x + c*s.c (s.x is the pixel stride)
    const float *tp[2];
    int64_t opix[2];
    bool live[2];
#pragma unroll
    for (int pb = 0; pb < 2; ++pb) {
        int64_t px = (int64_t)blockIdx.x * 256 + wave * 64 + pb * 32 + l32;
        live[pb] = px < p.P;
        if (!live[pb]) px = p.P - 1;
        const int64_t n = px / p.HW, pos = px % p.HW;
        tp[pb] = p.t + n * p.st.n + pos * p.st.x + (int64_t)lhi * p.st.c;
        opix[pb] = n * p.sy.n + pos * p.sy.x;
    }
    const float *ap[MBF];
    bool arow[MBF];
#pragma unroll
    for (int mb = 0; mb < MBF; ++mb) {
        const int m = m0 + mb * 32 + l32;
        arow[mb] = m < p.M;
        ap[mb] = p.pw + (int64_t)(arow[mb] ? m : 0) * p.G + lhi;
    }
    for (int k = 0; k < p.G; k += 2) {
        const bool kin = k + lhi < p.G;  // odd G: the last step has one channel
        float b[2], a[MBF];
#pragma unroll
        for (int pb = 0; pb < 2; ++pb) b[pb] = kin ? tp[pb][(int64_t)k * p.st.c] : 0.f;
#pragma unroll
        for (int mb = 0; mb < MBF; ++mb) a[mb] = (kin && arow[mb]) ? ap[mb][k] : 0.f;
#pragma unroll
        for (int pb = 0; pb < 2; ++pb)
#pragma unroll
            for (int mb = 0; mb < MBF; ++mb)
                acc[pb][mb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[mb], b[pb], acc[pb][mb], 0, 0, 0);
    }
#pragma unroll
    for (int pb = 0; pb < 2; ++pb) {
        if (!live[pb]) continue;
#pragma unroll
        for (int mb = 0; mb < MBF; ++mb)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int m = m0 + mb * 32 + 8 * (i / 4) + 4 * lhi + i % 4;
                if (m >= p.M) continue;
                const int64_t o = opix[pb] + (int64_t)m * p.sy.c;
                float v = acc[pb][mb][i];
                if (p.bias) v += p.bias[m];
                if (p.residual) v += p.residual[o];
                if (p.relu) v = fmaxf(v, 0.f);
                p.y[o] = v;
            }
    }
}

template <int DTYPE, int MB, int WAVES>
int launch_pw_instance(const PwParams &p, dim3 grid, size_t lds_bytes, hipStream_t s)
{
    auto kern = pw_mfma_kernel<DTYPE, MB, WAVES>;
    static bool raised = false;
    if (!raised) {
        GDWS_HIP_CHECK(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
        raised = true;
    }
    kern<<<grid, 64 * WAVES, lds_bytes, s>>>(p);
    GDWS_HIP_CHECK(hipGetLastError());
    return GDWS_OK;
}

uint16_t half_bits(float v, int dtype)
{
    if (dtype == GDWS_BF16) return float_to_bf16(v);
    _Float16 h = (_Float16)v;
    uint16_t b;
    __builtin_memcpy(&b, &h, 2);
    return b;
}

}  // namespace

void build_pw_mfma_tables(PwMfmaTables &tb, int dtype, int G, int M, const float *pw, const float *bias)
{
    tb = PwMfmaTables{};
    tb.Gp = (G + 15) & ~15;
    tb.ksteps = tb.Gp / 16;
    const int m_blocks = (M + 31) / 32;
    tb.mb_per_wg = m_blocks >= 3 ? 4 : 2;
    tb.m_blocks_pad = (m_blocks + tb.mb_per_wg - 1) / tb.mb_per_wg * tb.mb_per_wg;
    tb.bias_pad.assign((size_t)tb.m_blocks_pad * 32, 0.f);
    if (bias) std::copy(bias, bias + M, tb.bias_pad.begin());
    tb.frag.reserve((size_t)tb.ksteps * tb.m_blocks_pad * 64 * 8);
    // K-step s, block mb, lane l = (m = l % 32, half = l / 32), element e  <->  Pw[mb*32 + m][16 s + 8 half + e]
    for (int s = 0; s < tb.ksteps; ++s)
        for (int mb = 0; mb < tb.m_blocks_pad; ++mb)
            for (int l = 0; l < 64; ++l)
                for (int e = 0; e < 8; ++e) {
                    const int m = mb * 32 + (l & 31), j = 16 * s + 8 * (l >> 5) + e;
                    tb.frag.push_back(half_bits((m < M && j < G) ? pw[(size_t)m * G + j] : 0.f, dtype));
                }
    tb.valid = true;
}

int launch_pw_mfma_f32(const PwArgs &a, hipStream_t s)
{
    PwF32Params p;
    p.t = (const float *)a.t; p.y = (float *)a.y; p.pw = a.pw; p.bias = a.ep.bias;
    p.residual = (const float *)a.ep.residual; p.relu = a.ep.relu; p.G = a.G; p.M = a.M;
    p.HW = (int64_t)a.Ho * a.Wo; p.P = (int64_t)a.N * p.HW;
    p.st = make_strides(a.layout, a.Gt, a.Ho, a.Wo);
    p.sy = make_strides(a.layout, a.M, a.Ho, a.Wo);
    if (p.P == 0) return GDWS_OK;
    const dim3 grid((unsigned)((p.P + 255) / 256), (unsigned)((a.M + 63) / 64));
    pw_mfma_f32_kernel<<<grid, 256, 0, s>>>(p);
    GDWS_HIP_CHECK(hipGetLastError());
    return GDWS_OK;
}

int launch_pw_mfma(const PwMfmaArgs &a, hipStream_t s)
{
    const PwMfmaTables &tb = *a.tables;
    if (a.P >= ((int64_t)1 << 31)) return GDWS_EUNSUPPORTED;  // the kernel counts pixels in 32 bits
    PwParams p;
    p.t = (const uint16_t *)a.t; p.y = (uint16_t *)a.y; p.residual = (const uint16_t *)a.ep.residual;
    p.bias = tb.d_bias_pad; p.frag = (const u32x4_t *)tb.d_frag;
    p.P = (int)a.P; p.Gp = tb.Gp; p.M = a.M; p.ksteps = tb.ksteps; p.m_blocks_pad = tb.m_blocks_pad; p.relu = a.ep.relu;
    p.stride = a.stride; p.Ho = a.Ho; p.Wo = a.Wo; p.H = a.H; p.W = a.W;
    const int mb = tb.mb_per_wg;
    p.n_slices = tb.m_blocks_pad / mb;
    // 256-pixel tiles, or 128-pixel ones when there are too few of the former to give every CU two workgroups
    const int waves = ((a.P + 255) / 256) * p.n_slices < 256 * kWavesPerSimd ? 2 : 4;
    const int tile_px = 64 * waves;
    const int64_t items = ((a.P + tile_px - 1) / tile_px) * p.n_slices;
    if (items >= ((int64_t)1 << 31)) return GDWS_EUNSUPPORTED;
    p.n_tiles = (int)(items / p.n_slices);
    // the resident workgroups of the chip's 256 CUs share the work items out between them (a multiple of 8
    // workgroups: every XCD gets the same number)
    const int64_t xcd_items = (p.n_tiles + 7) / 8 * (int64_t)p.n_slices;  // the longest of the eight lists
    const dim3 grid((unsigned)(8 * std::min<int64_t>(xcd_items, 32 * (4 * kWavesPerSimd / waves))));
    const size_t lds = a.ep.residual ? (size_t)tile_px * (mb / 2 * 32 + 4) * 4 : (size_t)tile_px * (mb * 32 + 8) * 2;
#define GDWS_PW_CASE(dt, m, w) \
    if (a.dtype == dt && mb == m && waves == w) return launch_pw_instance<dt, m, w>(p, grid, lds, s);
    GDWS_PW_CASE(GDWS_BF16, 4, 4) GDWS_PW_CASE(GDWS_BF16, 2, 4) GDWS_PW_CASE(GDWS_BF16, 4, 2) GDWS_PW_CASE(GDWS_BF16, 2, 2)
    GDWS_PW_CASE(GDWS_F16, 4, 4) GDWS_PW_CASE(GDWS_F16, 2, 4) GDWS_PW_CASE(GDWS_F16, 4, 2) GDWS_PW_CASE(GDWS_F16, 2, 2)
#undef GDWS_PW_CASE
    return GDWS_EUNSUPPORTED;
}

}  // namespace gdws
