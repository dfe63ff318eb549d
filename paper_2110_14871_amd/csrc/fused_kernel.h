// Device code of the fused GDWS kernel (K = 3, pad = 1, 16-bit storage); included by the files that
// instantiate it.  See fused.h for the decomposition into tiles, stages, chunks and row blocks.
//
// Depthwise stage of one row block (<= 32 intermediate channels drawing on a 16-channel window), for
// 32 pixels:   T[j][p] = sum over taps (u,v) of  A_uv[j][c] * X[c][p + (u,v)]
// A_uv has a single non-zero per row (tap (u,v) of filter j, in the column of its input channel), so two taps
// side by side are a 32 x 32 matrix with at most one non-zero in every group of four columns: the operand form of
// the 2:4 sparse MFMA (v_smfmac_f32_32x32x32), which multiplies two taps in the time a dense MFMA takes for one.
// Nine taps are one dense MFMA and four sparse ones.  Each lane builds its slice of a row with a byte permute and
// four ANDs from the packed taps and four masks that are fixed for the row block.  X[.][p + (u,v)] is a 16-byte
// LDS read: the input tile is stored pixel-major, so the 8 consecutive channels a lane needs are contiguous and a
// tap is just an address offset.  Accumulation is fp32 inside the matrix instructions.
//
// Pointwise stage: the fp32 tile is rounded to the storage type (nearest even) where it sits; in the
// MFMA register layout a lane then already holds what the B operand of the next MFMA expects, in a
// K order that the pointwise weight fragments are packed to match at plan time.
//
// Epilogue: accumulators start from the bias; residual add and ReLU in registers; the tile goes
// through LDS once so that the global stores are 16 bytes per lane and coalesced in either layout.
// Optionally (NHWC, no residual) the stores are those of the 2 x 2, stride-2 max-pool of the tile.
//
// Synchronisation is by workgroup barriers only, executed in the same order by all eight waves:
// one per chunk of input channels (the loader waves arrive when the chunk is in LDS, the compute
// waves when they first need it), one when the last row block is done, one between the two halves
// of the epilogue.  (A variant for layers of one input stage has no loader waves: its four waves
// load the stage, then compute.)
//
// A depthwise-only mode (GDWONLY) stops after the depthwise stage and writes the intermediate
// tensor: the generalized depthwise stage as a kernel of its own, for the unfused path.
#pragma once
#include <type_traits>

#include "fused.h"

namespace gdws {
namespace fusedk {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) __bf16 bf16x16_t;
typedef __attribute__((ext_vector_type(16))) _Float16 f16x16_t;
typedef __attribute__((ext_vector_type(8))) uint32_t u32x8_t;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8_t;
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2_t;
typedef __attribute__((ext_vector_type(2))) float f32x2_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2_t;
typedef u32x4_t __attribute__((aligned(8))) u32x4_a8_t;  // 16 bytes at an 8-byte aligned address

constexpr int kComputeThreads = 256;  // waves 0-3
constexpr int kLoaderThreads = 256;   // waves 4-7
constexpr int kThreads = kComputeThreads + kLoaderThreads;
// LDS reads of the depthwise B operand run this many reads ahead (4, 6 and 12 measured the same)
constexpr int kReadAhead = 6;
constexpr int kMaxEnt = 10;  // NHWC loader: pixels per thread

template <int DTYPE> struct half_ops;

template <> struct half_ops<GDWS_BF16> {
    __device__ static uint32_t pack(float a, float b)
    {
        f32x2_t v = {a, b};
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
    }
    __device__ static f32x16_t mfma(u32x4_t a, u32x4_t b, f32x16_t c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b),
                                                       c, 0, 0, 0);
    }
    // D += A B with A 32 x 32 in the 2:4 compressed form (eight values per lane and two index bits for each) and
    // B 32 x 32 dense: lane (column n, half hb) holds K elements 8 hb .. 8 hb + 7 (b0) and 16 + 8 hb .. 23 + 8 hb (b1)
    __device__ static f32x16_t smfmac(u32x4_t a, u32x4_t b0, u32x4_t b1, f32x16_t c, int index)
    {
        const u32x8_t b = {b0[0], b0[1], b0[2], b0[3], b1[0], b1[1], b1[2], b1[3]};
        return __builtin_amdgcn_smfmac_f32_32x32x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x16_t, b),
                                                         c, index, 0, 0);
    }
    __device__ static float widen(uint16_t h) { return bf16_to_float(h); }
};

template <> struct half_ops<GDWS_F16> {
    __device__ static uint32_t pack(float a, float b)
    {
        f32x2_t v = {a, b};
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2_t));
    }
    __device__ static f32x16_t mfma(u32x4_t a, u32x4_t b, f32x16_t c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c,
                                                      0, 0, 0);
    }
    __device__ static f32x16_t smfmac(u32x4_t a, u32x4_t b0, u32x4_t b1, f32x16_t c, int index)
    {
        const u32x8_t b = {b0[0], b0[1], b0[2], b0[3], b1[0], b1[1], b1[2], b1[3]};
        return __builtin_amdgcn_smfmac_f32_32x32x32_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x16_t, b),
                                                        c, index, 0, 0);
    }
    __device__ static float widen(uint16_t h) { return (float)__builtin_bit_cast(_Float16, h); }
};

// max(v, 0) as one integer maximum on the bits (a negative float, -0 included, is a negative integer); fmaxf costs a
// second instruction that canonicalises its operand.  A NaN with the sign bit clear passes through.
__device__ inline float relu_bits(float v)
{
    const int b = __builtin_bit_cast(int, v);
    return __builtin_bit_cast(float, b > 0 ? b : 0);
}


struct FusedParams {
    const uint16_t *x;
    uint16_t *y;
    const uint16_t *residual;
    const float *bias;
    const int32_t *stage_tab;
    const u32x4_t *rec_a;
    const u32x2_t *rec_b;
    const u32x4_t *pwfrag;
    int n_stages, n_rowblocks, final_waits, m_blocks_pad, relu;
    int N, C, H, W, M, Ho, Wo;
    int TH, TN, IH;  // tile rows / images, input rows per tile
    int th_log2;     // TH is a power of two
    int stage_w;     // dwords per LDS stage buffer
    uint32_t x_bytes;  // size of x (below 2 GiB): the bound of the loader's buffer descriptor
    uint32_t y_bytes;  // depthwise-only mode: size of T (below 2 GiB), the bound of the stores' buffer descriptor
    int tiles_x, tiles_y;
    int c_begin0, c_count0;  // stage 0's entry of stage_tab
    int out_off;             // depthwise-only mode: dword offset in LDS of the waves' output staging areas
    int pool, Hp, Wp;        // pool != 0 (NHWC, no residual): y is the 2 x 2 / stride-2 max-pool of the output, Hp x Wp
    int lut_off;             // dword offset in LDS of the table of A-operand selectors (kLutBytes, behind all else)
};


// LDS geometry: the tile's input pixels (halo included), each holding the stage's channels.
template <int TW, int STRIDE, bool BIG> struct Geom {
    static constexpr int SC = STRIDE == 1 ? (BIG ? 128 : 64) : (BIG ? 32 : 16);  // channels per stage
    static constexpr int CC = STRIDE == 1 ? 32 : 16;    // channels per chunk
    static constexpr int NCH = SC / CC;                 // chunks per stage, at most
    static constexpr int PSW = lds_pixel_dwords(SC, STRIDE);  // dwords per pixel
    static constexpr int IW = (TW - 1) * STRIDE + 3;    // input columns per tile row
    static constexpr int RP = IW * PSW + lds_row_pad(TW, STRIDE);  // dwords per tile row
};

// NCHW loader of one chunk (channels [cb, cb + cn) of the stage buffer, filled with zeros past c_count): a thread
// takes (channel, input row) pairs and walks along the row, so the position is decoded once per row and the 2-byte
// loads of a thread run along contiguous memory (the transposition to the pixel-major LDS layout is the 2-byte
// LDS writes).
template <int TW, int STRIDE, bool BIG>
__device__ inline void load_chunk_nchw(const FusedParams &p, uint32_t *lds, int tid, int c_begin, int c_count, int cb,
                                       int cn, int n0, int ty0, int tx0)
{
    using Gm = Geom<TW, STRIDE, BIG>;
    const int rows = p.TN * p.IH;
    uint16_t *lds16 = (uint16_t *)lds;
    for (int it = tid; it < cn * rows; it += kLoaderThreads) {
        const int cs = cb + it % cn, r = it / cn;  // consecutive lanes: consecutive channels (conflict-free LDS writes)
        const int iy = r % p.IH, tn = r / p.IH;
        const int n = n0 + tn, gy = ty0 * STRIDE - 1 + iy, gx0 = tx0 * STRIDE - 1;
        const bool row_in = n < p.N && gy >= 0 && gy < p.H && cs < c_count;
        const uint16_t *src = p.x + (((int64_t)n * p.C + c_begin + cs) * p.H + gy) * p.W + gx0;
        uint16_t *dst = lds16 + r * (Gm::RP * 2) + cs;
#pragma unroll 6
        for (int ix = 0; ix < Gm::IW; ++ix) {
            const int gx = gx0 + ix;
            const uint16_t v = (row_in && gx >= 0 && gx < p.W) ? src[ix] : (uint16_t)0;
            dst[ix * (Gm::PSW * 2)] = v;
        }
    }
}

// Sparse depthwise stage: how a lane places its tap in the A operand depends only on the row's window column cw
// (16 values) and on the lane's half, so the 32 cases are worked out once per workgroup, by 32 threads, into a table in
// LDS that every row block reads with three loads (the compares and selects they replace are the slowest vector
// instructions of the loop).  An entry is nine dwords in twelve: byte selectors of v_perm_b32 that put the lane's
// tap of a record dword into A dword d of a pair of taps (0-3) and the first tap into A dword d of the dense
// MFMA (4-7) -- selector byte 0x0c yields zero -- and the index operand of the sparse MFMAs (8).
// The row's column cw lies in compressed slot 2 (cw / 4) + (cw % 4 == 3), with index code cw % 4; the other slot
// of each pair is zero under a code that keeps the pair ordered (even slot 0, odd slot 3).  For the dense tap a
// lane holds columns 8 lh .. 8 lh + 7 as they are.  (A workgroup barrier must lie between these writes and the
// first read: in the kernels here the first one every wave passes before its first row block.)
__device__ inline void write_selector_entry(uint32_t *e, uint32_t cw, uint32_t lh)
{
    const uint32_t pr = cw >> 2, code = cw & 3u;
    const uint32_t tap = lh ? 0x0302u : 0x0100u;  // a record dword holds a pair's first tap below its second
    const uint32_t sp = code == 3u ? (tap << 16 | 0x0C0Cu) : (0x0C0C0000u | tap);
    const int rel = (int)cw - 8 * (int)lh;
    const uint32_t sd = (rel & 1) ? 0x01000C0Cu : 0x0C0C0100u;
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        e[d] = pr == (uint32_t)d ? sp : 0x0C0C0C0Cu;
        e[4 + d] = (rel >> 1) == d ? sd : 0x0C0C0C0Cu;
    }
    e[8] = 0xCCCCu | ((code == 3u ? 0u : code) << (4u * pr));
}

// NPB: 32-pixel blocks per compute wave.  2: a workgroup's tile is 256 output pixels.  1 (NHWC): 128 pixels, half the
// MFMAs per row block and wave -- for layers with so few tiles that 256-pixel tiles leave the chip idle.
// SELF (NHWC, layers whose input channels are one stage): no loader waves.  The workgroup is the four compute waves,
// which first load the stage themselves; with half the waves per workgroup twice as many workgroups are resident per
// CU for the same registers, and their prologues and epilogues overlap the others' arithmetic.
// TAP2 (NHWC): the depthwise MFMA's K dimension holds two filter taps of an 8-channel window instead of one tap of a
// 16-channel window -- K element 8 h + c is tap 2 i + h of window channel c in MFMA i, so the lanes' upper half
// (h = 1) builds its A operand from the odd tap and reads its B operand at the odd tap's pixel.  Nine taps are five
// MFMAs instead of nine, with five LDS reads per pixel block and no lane exchange; the price is that a row block's
// rows must come from 8 input channels, so layers with few filters per channel need more row blocks.  The plan
// chooses per layer (build_fused_schedule).
template <int DTYPE, int TW, int STRIDE, bool BIG, int MB, bool NHWC, bool GDWONLY = false, int NPB = 2, bool SELF = false,
          bool TAP2 = false>
__global__ __launch_bounds__(SELF ? kComputeThreads : kThreads, (NPB == 1 && MB == 2) ? 4 : 1)  // (four waves per SIMD: 128 registers)
void gdws_fused_kernel(FusedParams params)
{
    static_assert(!SELF || NHWC, "workgroups without loader waves exist for the NHWC kernels");
    static_assert(!TAP2 || (NHWC && !GDWONLY), "the two-tap depthwise stage exists for the fused NHWC kernels");
    constexpr int kWgThreads = SELF ? kComputeThreads : kThreads;
    static_assert(NPB == 2 || (NPB == 1 && NHWC), "128-pixel tiles exist for the NHWC kernels");
    static_assert(TW >= 8 || NHWC, "tiles four pixels wide exist for the NHWC kernels (NCHW stores 8 pixels of a row)");
    constexpr int kTilePx = 128 * NPB;
    // The integer kernel arguments are fetched in the entry block, in one batch of scalar loads with a single wait;
    // left to itself the compiler fetches them block by block, each time with a round trip to memory on the critical
    // path.  (Pointers are left alone: passing them through an asm statement would lose their address space.)
    FusedParams p = params;
#define GDWS_PIN(f) asm volatile("" : "+s"(p.f))
    GDWS_PIN(n_stages); GDWS_PIN(n_rowblocks); GDWS_PIN(final_waits); GDWS_PIN(m_blocks_pad);
    GDWS_PIN(relu); GDWS_PIN(N); GDWS_PIN(C); GDWS_PIN(H); GDWS_PIN(W); GDWS_PIN(M); GDWS_PIN(Ho); GDWS_PIN(Wo);
    GDWS_PIN(TH); GDWS_PIN(TN); GDWS_PIN(IH); GDWS_PIN(th_log2); GDWS_PIN(stage_w); GDWS_PIN(x_bytes); GDWS_PIN(y_bytes); GDWS_PIN(tiles_x);
    GDWS_PIN(tiles_y); GDWS_PIN(c_begin0); GDWS_PIN(c_count0); GDWS_PIN(out_off); GDWS_PIN(lut_off);
#undef GDWS_PIN
    using Op = half_ops<DTYPE>;
    using Gm = Geom<TW, STRIDE, BIG>;
    extern __shared__ uint32_t lds[];

    const int lane = threadIdx.x & 63, wave = (threadIdx.x >> 6) & 3;
    int tile = blockIdx.x;
    const int tx0 = (tile % p.tiles_x) * TW; tile /= p.tiles_x;
    const int ty0 = (tile % p.tiles_y) * p.TH;
    const int n0 = (tile / p.tiles_y) * p.TN;
    const int mbase = blockIdx.y * MB;
    const int npix = p.TN * p.IH * Gm::IW;

    // output tile in LDS (after the last row block): NHWC [256 pixels][MB*32 channels], NCHW [MB*32 channels][256 pixels],
    // rows padded by 16 bytes; in the storage type, final values, without a residual; in fp32, before the residual
    // add, with one.  Behind it, NHWC only, the pixel index in y of each of the 256 tile pixels (-1: outside).
    constexpr int kRowElems = NHWC ? MB * 32 : kTilePx, kRows = NHWC ? kTilePx : MB * 32;
    constexpr int kRowHalfs = kRowElems + 8, kRowFloats = kRowElems + 4;
    uint16_t *tile16 = (uint16_t *)lds;
    float *tile32 = (float *)lds;
    int *pixtab = p.residual ? (int *)(tile32 + kRows * kRowFloats) : (int *)(tile16 + kRows * kRowHalfs);

    if constexpr (!TAP2) {
        if (threadIdx.x < 32) write_selector_entry(lds + p.lut_off + threadIdx.x * kLutEntry, threadIdx.x & 15u, threadIdx.x >> 4);
    }
    if (SELF || threadIdx.x >= kComputeThreads) {
        // ================================ loader waves ================================
        const int tid = SELF ? threadIdx.x : threadIdx.x - kComputeThreads;
        constexpr int QC = Gm::CC / 8;              // 16-byte pieces of a pixel per chunk
        constexpr int PSTEP = kLoaderThreads / QC;  // pixels per pass of the loader threads
        const int q = tid % QC, pix0 = tid / QC;
        const int nent = (npix + PSTEP - 1) / PSTEP;  // the host guarantees nent <= kMaxEnt
        if (NHWC) {
            // A thread owns one 16-byte piece position of every PSTEP-th pixel of the input tile, the same pixels in
            // every chunk and stage.  Their byte offsets in x are worked out once; pixels outside the image (and
            // entries past the tile) get an offset beyond the buffer descriptor's bound, for which the hardware
            // returns zeros: the padding costs no branch.  A chunk is then nent loads and nent LDS writes.
            constexpr uint32_t kOutside = 0x80000000u;
            uint32_t voff[kMaxEnt];
            uint32_t loff[kMaxEnt];  // dword offset of the entry's pixel in a stage buffer
            // walk over the thread's pixels: (column, row, image) inside the input tile, advanced by PSTEP pixels
            int ix = pix0 % Gm::IW, iy, tn;
            {
                const int r = pix0 / Gm::IW;
                iy = r % p.IH, tn = r / p.IH;
            }
            constexpr int dix = PSTEP % Gm::IW, dr = PSTEP / Gm::IW;
            int diy = dr, dtn = 0;
            while (diy >= p.IH) { diy -= p.IH; ++dtn; }
            const int gy0 = ty0 * STRIDE - 1, gx0 = tx0 * STRIDE - 1;
            const uint32_t c2 = (uint32_t)p.C * 2u;
            auto next_offset = [&](uint32_t &lds_off) {
                const int n = n0 + tn, gy = gy0 + iy, gx = gx0 + ix;
                lds_off = (uint32_t)((tn * p.IH + iy) * Gm::RP + ix * Gm::PSW);
                const bool in = tn < p.TN && n < p.N && (unsigned)gy < (unsigned)p.H && (unsigned)gx < (unsigned)p.W;
                // 24-bit multiplies: the host admits fewer than 2^24 input pixels
                const uint32_t pixel = __umul24(__umul24(n, p.H) + gy, p.W) + gx;
                const uint32_t off = in ? __umul24(pixel, c2) + q * 16 : kOutside;
                ix += dix; iy += diy; tn += dtn;
                if (ix >= Gm::IW) { ix -= Gm::IW; ++iy; }
                if (iy >= p.IH) { iy -= p.IH; ++tn; }
                return off;
            };
            const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)p.x, 0, p.x_bytes, 0x00020000);
            uint32_t *dst0 = lds + q * 4;
            // In the first stage the offsets are worked out as the first chunk's loads go out, so that the first of
            // them is in flight after a few dozen instructions.
            auto run_stage = [&](int st, int c_begin, int c_count, auto first) {
                const int cfill = (c_count + 15) & ~15;  // channels the row blocks may read (zeros past c_count)
                const int nch = (cfill + Gm::CC - 1) / Gm::CC;
                uint32_t *dst = dst0 + (st & 1) * p.stage_w;
                // two chunks are in flight at a time: enough to keep the memory system busy, and a chunk is handed
                // to the compute waves as soon as it has landed rather than behind the issue of all later loads
                u32x4_t v[Gm::NCH > 1 ? 2 : 1][kMaxEnt];
                auto issue = [&](int ch) {
                    const uint32_t gone = ch * Gm::CC + q * 8 < c_count ? 0u : kOutside;  // channels past the layer's
#pragma unroll
                    for (int k = 0; k < kMaxEnt; ++k)
                        if (k < nent) {
                            if (first && ch == 0) voff[k] = next_offset(loff[k]);
                            v[ch & 1][k] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, voff[k] | gone,
                                                                             (c_begin + ch * Gm::CC) * 2, 0);
                        }
                };
                issue(0);
                if (Gm::NCH > 1 && nch > 1) issue(1);
#pragma unroll
                for (int ch = 0; ch < Gm::NCH; ++ch) {
                    if (ch < nch) {
                        // the stage buffer has room for the pixels of the last pass that lie past the tile
#pragma unroll
                        for (int k = 0; k < kMaxEnt; ++k)
                            if (k < nent) *(u32x4_a8_t *)(dst + loff[k] + ch * (Gm::CC / 2)) = v[ch & 1][k];
                        __syncthreads();  // chunk ch of stage st is in LDS
                        if (ch + 2 < Gm::NCH && ch + 2 < nch) issue(ch + 2);
                    }
                }
            };
            run_stage(0, p.c_begin0, p.c_count0, std::true_type{});
            if constexpr (!SELF) {
                for (int st = 1; st < p.n_stages; ++st)
                    run_stage(st, p.stage_tab[2 * st + 0], p.stage_tab[2 * st + 1], std::false_type{});
            }
        } else {
            for (int st = 0; st < p.n_stages; ++st) {
                const int c_begin = p.stage_tab[2 * st + 0], c_count = p.stage_tab[2 * st + 1];
                const int cfill = (c_count + 15) & ~15;
                for (int cb = 0; cb < cfill; cb += Gm::CC) {
                    load_chunk_nchw<TW, STRIDE, BIG>(p, lds + (st & 1) * p.stage_w, tid, c_begin, c_count, cb,
                                                     cfill - cb < Gm::CC ? cfill - cb : Gm::CC, n0, ty0, tx0);
                    __syncthreads();  // the chunk is in LDS
                }
            }
        }
        if constexpr (!SELF) __syncthreads();  // the compute waves are done with the input
    }
    if (SELF || threadIdx.x < kComputeThreads) {
        // ================================ compute waves ================================
        const int l32 = lane & 31, lhi = lane >> 5;
        // LDS dword offset of the top-left tap of this lane's pixel in each of the wave's two 32-pixel blocks,
        // plus the lane's half of the 16-channel window
        int base[NPB];
#pragma unroll
        for (int pb = 0; pb < NPB; ++pb) {
            const int pp = wave * (32 * NPB) + pb * 32 + l32;
            const int tx = pp % TW, ty = (pp / TW) & (p.TH - 1), tn = (pp / TW) >> p.th_log2;
            base[pb] = (tn * p.IH + ty * STRIDE) * Gm::RP + tx * STRIDE * Gm::PSW + (TAP2 ? 0 : lhi * 4);
        }

        // accumulators start from the bias
        constexpr int MBA = GDWONLY ? 0 : MB;  // the depthwise-only mode has no pointwise stage
        f32x16_t acc[NPB][MBA ? MBA : 1];
#pragma unroll
        for (int mb = 0; mb < MBA; ++mb) {
            // NHWC: D[m][pixel], register i <-> channel 8*(i/4) + 4*lhi + i%4; NCHW: D[pixel][m], lane <-> channel
            const float *bp = p.bias + (mbase + mb) * 32;  // padded with zeros to whole 32-channel blocks
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                f32x4_t bv;
                if (NHWC) bv = *(const f32x4_t *)(bp + 8 * q4 + 4 * lhi);
                else bv = f32x4_t{bp[l32], bp[l32], bp[l32], bp[l32]};
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int pb = 0; pb < NPB; ++pb) acc[pb][mb][4 * q4 + i] = bv[i];
            }
        }

        // Records are fetched two row blocks ahead: the load issued when a row block's depthwise stage is done has a
        // whole row block to arrive before it is copied into the current record's registers (fetched only one ahead,
        // the wave waited several hundred cycles for it at the top of every row block).  The pointwise fragments are
        // reloaded in place right after their last use.
        // (all table addresses are a wave-uniform base plus the lane: scalar registers hold the bases)
        u32x4_t ra = p.rec_a[lane], na = p.rec_a[64 + lane];
        u32x2_t rb = p.rec_b[lane], nb = p.rec_b[64 + lane];
        const int rb_stride = 2 * p.m_blocks_pad * 64;  // 16-byte units of pointwise fragments per row block
        const u32x4_t *fp = p.pwfrag + (int64_t)mbase * 64;  // uniform
        u32x4_t pwf[2][MBA ? MBA : 1];
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int mb = 0; mb < MBA; ++mb) pwf[s][mb] = (fp + s * p.m_blocks_pad * 64)[mb * 64 + lane];

        // Depthwise-only mode: a wave's block of T (its pixels x 32 channels) goes through a staging area of its own in
        // LDS ([pixel][32 channels], rows of 80 bytes) so that it leaves in 16-byte pieces: lane l stores quarter l % 4
        // (8 channels) of pixels l / 4 + 16 k.  The row blocks of this mode own whole groups of 8 intermediate channels.
        constexpr int kOutRow = 20;  // dwords per pixel in the staging area
        uint32_t *ostage = lds + p.out_off + wave * (32 * NPB * kOutRow);
        // The stores go through a buffer descriptor, and a lane with nothing to store (a pixel outside the image, a
        // quarter the row block does not own) gets an offset beyond the descriptor's bound, for which the hardware
        // drops the store.  So every row block issues the same store instructions, without a branch around them, and
        // the compiler's counts of outstanding memory operations stay exact: the wave waits for the records it
        // loaded, not for the stores it issued after them (stores and loads share one in-order counter, and with
        // conditional stores every wait for a load was also a wait for the previous row block's stores to land).
        constexpr uint32_t kDropped = 0x80000000u;
        uint32_t opix[2 * NPB];      // byte offset in T of the lane's piece of its pixels, kDropped: outside the image
        const __amdgpu_buffer_rsrc_t yrsrc = __builtin_amdgcn_make_buffer_rsrc((void *)p.y, 0, p.y_bytes, 0x00020000);
        if (GDWONLY) {
#pragma unroll
            for (int k = 0; k < 2 * NPB; ++k) {
                const int pp = wave * (32 * NPB) + (lane >> 2) + 16 * k, row = pp / TW;
                const int ox = tx0 + (pp & (TW - 1)), oy = ty0 + (row & (p.TH - 1)), on = n0 + (row >> p.th_log2);
                opix[k] = (on < p.N && oy < p.Ho && ox < p.Wo)
                              ? (uint32_t)((on * p.Ho + oy) * p.Wo + ox) * (uint32_t)(p.M * 2) + (lane & 3) * 16
                              : kDropped;
            }
        }

        int stage = 0;
        const uint32_t *buf = lds;
        f32x16_t zero;
#pragma unroll
        for (int i = 0; i < 16; ++i) zero[i] = 0.f;

        constexpr bool kShare = STRIDE == 1 && !TAP2;
        // LDS reads of the depthwise B operand run this many reads ahead
        constexpr int kReads = NPB * (TAP2 ? 5 : kShare ? 6 : 9);  // LDS reads per row block
        constexpr int kDepth = TAP2 ? 5 : NPB == 1 ? 3 : kReadAhead;
        static_assert(kReads % kDepth == 0, "queue slots line up across row blocks only if the depth divides the reads");
        u32x4_t bq[kDepth];
        bool fill = true;

        auto tap_offset = [](int tap) { return (tap / 3) * Gm::RP + (tap % 3) * Gm::PSW; };
        // the taps whose operand comes from LDS, in reading order (each for all pixel blocks): at stride 1 the left
        // and the right tap of each filter row (the middle one is derived from them), else all nine
        auto read_tap = [](int r) { return kShare ? 3 * (r / 2) + 2 * (r % 2) : r; };
        // two-tap stage: the lane's tap of each of the five MFMAs (tap 8 stands alone: the upper half multiplies it by
        // zero) as an LDS offset, and the byte selector that duplicates the lane's tap of a record dword
        int toff[5];
        if constexpr (TAP2) {
#pragma unroll
            for (int i = 0; i < 5; ++i) toff[i] = tap_offset(i == 4 ? 8 : lhi ? 2 * i + 1 : 2 * i);
        }
        // the byte selector that duplicates the lane's tap of a record dword (lower half of the lanes: the first tap
        // of the pair, upper half: the second)
        const uint32_t psel = lhi ? 0x03020302u : 0x01000100u;

        // sparse depthwise stage: the current record's entry of the selector table
        u32x4_t sp, sd;
        int sidx = 0;
        auto read_lut = [&]() {
            const uint32_t *lut = lds + p.lut_off + (((rb[0] >> 16) & 15u) | (uint32_t)lhi << 4) * kLutEntry;
            sp = *(const u32x4_t *)lut;
            sd = *(const u32x4_t *)(lut + 4);
            sidx = (int)lut[8];
        };

        for (int idx = 0; idx < p.n_rowblocks; ++idx) {
            const uint32_t ctrl = (uint32_t)__builtin_amdgcn_readfirstlane((int)rb[1]);
            const int win_off = ctrl & 0xff, nwait = (ctrl >> 8) & 0xf, next_off = (ctrl >> 16) & 0xff;
            const bool chain = ctrl & kCtrlChainNext;
            if (ctrl & kCtrlNewStage) {
                ++stage;
                buf = lds + (stage & 1) * p.stage_w;
            }
            if constexpr (!SELF) {  // (without loader waves the whole stage is in LDS before the first row block)
                for (int w = 0; w < nwait; ++w) __syncthreads();  // the chunks the window lies in have landed
            }
            // A window starts at a multiple of four channels, so a lane's 16 bytes are 8-byte aligned: a pair of
            // 8-byte reads in one instruction.
            const uint32_t *src[NPB];
#pragma unroll
            for (int pb = 0; pb < NPB; ++pb) src[pb] = buf + base[pb] + win_off;
            const int next_delta = next_off - win_off;  // the next row block's window, relative to this one's
            auto read16 = [](const uint32_t *ptr) { return *(const u32x4_a8_t *)ptr; };
            if (fill) {
#pragma unroll
                for (int i = 0; i < kDepth; ++i)
                    bq[i] = read16(src[i % NPB] + (TAP2 ? toff[i / NPB] : tap_offset(read_tap(i / NPB))));
            }
            fill = SELF ? false : !chain;  // (without loader waves the stage is complete: every row block reads ahead)

            // ---- depthwise: NPB 32-pixel blocks x nine taps; each block is rounded to the storage type when
            // done: register i of a lane pairs up as K element i % 8 of K-step i / 8 ----
            // The blocks advance together, tap by tap, so that the A operand of a tap is built once.
            f32x16_t t[NPB];
            u32x4_t tb[NPB][2];
            if constexpr (TAP2) {
                // masks: which of the lane's four A dwords, and which half of it, holds the row's column
                const uint32_t sel = rb[0] >> 16;
                const uint32_t hm = (sel & 8) ? 0xFFFF0000u : 0x0000FFFFu;
                uint32_t m[4];
#pragma unroll
                for (int d = 0; d < 4; ++d) m[d] = (sel & 7) == (uint32_t)d ? hm : 0u;
#pragma unroll
                for (int i5 = 0; i5 < 5; ++i5) {
                    const uint32_t word = i5 < 4 ? ra[i5] : (rb[0] & 0xffffu);  // (tap 8's partner is zero)
                    const uint32_t dup = __builtin_amdgcn_perm(word, word, psel);
                    const u32x4_t a = u32x4_t{dup & m[0], dup & m[1], dup & m[2], dup & m[3]};
#pragma unroll
                    for (int pb = 0; pb < NPB; ++pb) {
                        const int i = NPB * i5 + pb;  // position in the sequence of LDS reads
                        t[pb] = Op::mfma(a, bq[i % kDepth], i5 == 0 ? zero : t[pb]);
                        const int n = i + kDepth;     // the read that takes the freed queue slot
                        if (n < kReads) {
                            bq[i % kDepth] = read16(src[n % NPB] + toff[n / NPB]);
                        } else {  // (read in vain when the next row block does not chain)
                            bq[i % kDepth] = read16(src[n % NPB] + next_delta + toff[(n - kReads) / NPB]);
                        }
                    }
                }
            } else {
                // One tap of the 16-channel window is a 32 x 16 matrix with a single non-zero per row, so two taps side
                // by side (K = 32) satisfy the 2:4 pattern of the sparse MFMA, which multiplies them in the time of one
                // dense tap.  Tap 0 goes first, as a dense MFMA that starts the accumulation from zero; taps (1,2),
                // (3,4), (5,6), (7,8) follow as four sparse ones: the lower half of the lanes carries the first tap of
                // a pair in its eight compressed A slots, the upper half the second (the record packs them so), and B
                // is the two taps' 16-byte LDS reads side by side.
                // The byte selectors that place the lane's taps (sp, sd), and the index operand, come from the table in
                // LDS: they were read when the record became the current one.
                if (idx == 0) read_lut();
                auto pair_a = [&](int i) {
                    return u32x4_t{__builtin_amdgcn_perm(ra[i], ra[i], sp[0]), __builtin_amdgcn_perm(ra[i], ra[i], sp[1]),
                                   __builtin_amdgcn_perm(ra[i], ra[i], sp[2]), __builtin_amdgcn_perm(ra[i], ra[i], sp[3])};
                };
                auto slot = [](int r, int pb) { return (NPB * r + pb) % kDepth; };
                // read r of block pb has been consumed: the read kDepth further on takes its queue slot
                auto refill = [&](int r, int pb) {
                    const int i = NPB * r + pb, n = i + kDepth;
                    if (n < kReads) {
                        bq[i % kDepth] = read16(src[n % NPB] + tap_offset(read_tap(n / NPB)));
                    } else {  // (read in vain when the next row block does not chain)
                        bq[i % kDepth] = read16(src[n % NPB] + next_delta + tap_offset(read_tap((n - kReads) / NPB)));
                    }
                };
                const u32x4_t a_first = u32x4_t{__builtin_amdgcn_perm(rb[0], rb[0], sd[0]), __builtin_amdgcn_perm(rb[0], rb[0], sd[1]),
                                                __builtin_amdgcn_perm(rb[0], rb[0], sd[2]), __builtin_amdgcn_perm(rb[0], rb[0], sd[3])};
                if constexpr (kShare) {
                    // Stride 1: the middle tap of a filter row is not read from LDS.  Its operand is, lane by lane, the
                    // left tap's operand of the next pixel or the right tap's of the previous one, both in registers of
                    // neighbouring lanes of the same 16-lane row: two DPP moves per dword (lanes 0-3 and 8-11 of a row
                    // take the former, lanes 4-7 and 12-15 the latter, so no lane reaches across a tile row's end).
                    // Reads in order: left and right tap of filter row 0, of row 1, of row 2 (each for all blocks).
                    auto middle = [&](const u32x4_t &bl, const u32x4_t &br) {
                        u32x4_t mid;
#pragma unroll
                        for (int d = 0; d < 4; ++d) {
                            // (written to all lanes, zero where the neighbour is outside the row: the second
                            // move overwrites those, and no register has to be cleared first)
                            if constexpr (TW >= 8) {
                                const uint32_t x = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)bl[d], 0x101, 0xf, 0xf, true);
                                mid[d] = (uint32_t)__builtin_amdgcn_update_dpp((int)x, (int)br[d], 0x111, 0xf, 0xa, false);
                            } else {
                                // four-pixel tile rows are the quads: lanes 0-1 of a quad take the left tap of the
                                // next lane, lanes 2-3 the right tap of the previous one
                                const uint32_t nx = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)bl[d], 0xE9, 0xf, 0xf, false);
                                const uint32_t pv = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)br[d], 0x90, 0xf, 0xf, false);
                                mid[d] = (lane & 2) ? pv : nx;
                            }
                        }
                        return mid;
                    };
                    {   // tap 0 alone, then taps (1, 2): middle and right of filter row 0
                        const u32x4_t a = pair_a(0);
#pragma unroll
                        for (int pb = 0; pb < NPB; ++pb) t[pb] = Op::mfma(a_first, bq[slot(0, pb)], zero);
#pragma unroll
                        for (int pb = 0; pb < NPB; ++pb) {
                            const u32x4_t mid = middle(bq[slot(0, pb)], bq[slot(1, pb)]);
                            t[pb] = Op::smfmac(a, mid, bq[slot(1, pb)], t[pb], sidx);
                            refill(0, pb);
                            refill(1, pb);
                        }
                    }
                    {   // taps (3, 4): left and middle of filter row 1
                        const u32x4_t a = pair_a(1);
#pragma unroll
                        for (int pb = 0; pb < NPB; ++pb) {
                            const u32x4_t mid = middle(bq[slot(2, pb)], bq[slot(3, pb)]);
                            t[pb] = Op::smfmac(a, bq[slot(2, pb)], mid, t[pb], sidx);
                            refill(2, pb);
                        }
                    }
                    {   // taps (5, 6): right of filter row 1, left of row 2
                        const u32x4_t a = pair_a(2);
#pragma unroll
                        for (int pb = 0; pb < NPB; ++pb) {
                            t[pb] = Op::smfmac(a, bq[slot(3, pb)], bq[slot(4, pb)], t[pb], sidx);
                            refill(3, pb);
                        }
                    }
                    {   // taps (7, 8): middle and right of filter row 2
                        const u32x4_t a = pair_a(3);
#pragma unroll
                        for (int pb = 0; pb < NPB; ++pb) {
                            const u32x4_t mid = middle(bq[slot(4, pb)], bq[slot(5, pb)]);
                            t[pb] = Op::smfmac(a, mid, bq[slot(5, pb)], t[pb], sidx);
                            refill(4, pb);
                            refill(5, pb);
                        }
                    }
                } else {
#pragma unroll
                    for (int pb = 0; pb < NPB; ++pb) {
                        t[pb] = Op::mfma(a_first, bq[slot(0, pb)], zero);
                        refill(0, pb);
                    }
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const u32x4_t a = pair_a(i);
#pragma unroll
                        for (int pb = 0; pb < NPB; ++pb) {
                            t[pb] = Op::smfmac(a, bq[slot(2 * i + 1, pb)], bq[slot(2 * i + 2, pb)], t[pb], sidx);
                            refill(2 * i + 1, pb);
                            refill(2 * i + 2, pb);
                        }
                    }
                }
            }
#pragma unroll
            for (int pb = 0; pb < NPB; ++pb)
#pragma unroll
                for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
                    for (int d = 0; d < 4; ++d)
                        tb[pb][s2][d] = Op::pack(t[pb][8 * s2 + 2 * d], t[pb][8 * s2 + 2 * d + 1]);
            // ---- the next record becomes the current one; the record of row block idx + 2 is requested ----
            const uint32_t rb0 = (uint32_t)__builtin_amdgcn_readfirstlane((int)rb[0]);  // (the upper bits are uniform)
            {
                const uint32_t ri = (uint32_t)(idx + 2) * 64u + (uint32_t)lane;  // 32-bit offset from a scalar base
                ra = na;
                rb = nb;
                na = p.rec_a[ri];
                nb = p.rec_b[ri];
                if constexpr (!TAP2) read_lut();
            }
            if constexpr (GDWONLY) {
                // ---- the block of T leaves: registers -> staging area -> global, 16 bytes per lane ----
                const uint32_t own = rb0 >> 20;             // first group of 8 channels (bits 0-9), groups - 1 (bits 10-11)
                const int jb = (int)(own & 0x3ff) * 8, ng = (int)(own >> 10) + 1;
#pragma unroll
                for (int pb = 0; pb < NPB; ++pb)
#pragma unroll
                    for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
                        for (int h = 0; h < 2; ++h)   // rows 16*s2 + 8*h + 4*lhi .. +3: two dwords
                            *(u32x2_t *)(ostage + (pb * 32 + l32) * kOutRow + 8 * s2 + 4 * h + 2 * lhi) =
                                u32x2_t{tb[pb][s2][2 * h], tb[pb][s2][2 * h + 1]};
                const int quarter = lane & 3;
                const uint32_t gone = quarter < ng ? 0u : kDropped;
#pragma unroll
                for (int k = 0; k < 2 * NPB; ++k) {
                    const u32x4_t v = *(const u32x4_t *)(ostage + ((lane >> 2) + 16 * k) * kOutRow + quarter * 4);
                    __builtin_amdgcn_raw_buffer_store_b128(v, yrsrc, (opix[k] + (uint32_t)jb * 2u) | gone, 0, 0);
                }
            } else {
            // ---- pointwise ----
                fp += rb_stride;
    #pragma unroll
                for (int s = 0; s < 2; ++s)
    #pragma unroll
                    for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
                        for (int pb = 0; pb < NPB; ++pb) {
                            if (NHWC) acc[pb][mb] = Op::mfma(pwf[s][mb], tb[pb][s], acc[pb][mb]);  // D[m][pixel]
                            else acc[pb][mb] = Op::mfma(tb[pb][s], pwf[s][mb], acc[pb][mb]);       // D[pixel][m]
                        }
                        // fragment of the next row block
                        pwf[s][mb] = (fp + s * p.m_blocks_pad * 64)[mb * 64 + lane];
                    }
            }
        }
        if constexpr (!SELF) {
            for (int w = 0; w < p.final_waits; ++w) __syncthreads();  // chunks that no row block needed
        }
        __syncthreads();  // every wave is done with the input: the tile may overwrite it

        // ---- epilogue, part 1 (compute waves): residual, ReLU, rounding; the tile goes to LDS ----
        if (NHWC && !GDWONLY && threadIdx.x < kTilePx) {
            const int op = threadIdx.x, row = op / TW;
            const int ox = tx0 + (op & (TW - 1)), oy = ty0 + (row & (p.TH - 1)), on = n0 + (row >> p.th_log2);
            pixtab[op] = (on < p.N && oy < p.Ho && ox < p.Wo) ? (on * p.Ho + oy) * p.Wo + ox : -1;
        }
        auto to_lds = [&](auto raw, auto relu) {
#pragma unroll
            for (int h = 0; h < NPB; ++h) {
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
                    for (int q4 = 0; q4 < 4; ++q4) {
                        f32x4_t v;
#pragma unroll
                        for (int i = 0; i < 4; ++i) v[i] = acc[h][mb][4 * q4 + i];
                        // NHWC: lane = pixel h*32 + l32, registers = 4 consecutive output channels;
                        // NCHW: lane = output channel, registers = 4 consecutive pixels of the tile row
                        const int px0 = wave * (32 * NPB) + h * 32;  // first pixel of the block
                        const int row = NHWC ? px0 + l32 : mb * 32 + l32;
                        const int col = NHWC ? mb * 32 + 8 * q4 + 4 * lhi : px0 + 8 * q4 + 4 * lhi;
                        if (raw) {
                            *(f32x4_t *)(tile32 + row * kRowFloats + col) = v;
                        } else {
                            if (relu) {
#pragma unroll
                                for (int i = 0; i < 4; ++i) v[i] = relu_bits(v[i]);
                            }
                            *(u32x2_t *)(tile16 + row * kRowHalfs + col) = u32x2_t{Op::pack(v[0], v[1]), Op::pack(v[2], v[3])};
                        }
                    }
                }
            }
        };
        using std::false_type;
        using std::true_type;
        if constexpr (!GDWONLY) {
            if (p.residual) to_lds(true_type{}, false_type{});
            else if (p.relu) to_lds(false_type{}, true_type{});
            else to_lds(false_type{}, false_type{});
        }
    }

    // ---- epilogue, part 2 (all eight waves): LDS -> global in 16-byte pieces ----
    __syncthreads();
    if (GDWONLY) return;
    const int t = threadIdx.x;
    // eight values of a tile row: as stored (no residual), or fp32 + residual, ReLU, rounding
    auto finish = [&](int row, int col, const uint16_t *res) {
        if (!p.residual) return *(const u32x4_t *)(tile16 + row * kRowHalfs + col);
        const f32x4_t lo = *(const f32x4_t *)(tile32 + row * kRowFloats + col);
        const f32x4_t hi = *(const f32x4_t *)(tile32 + row * kRowFloats + col + 4);
        const u32x4_t r = *(const u32x4_t *)res;
        float v[8];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[i] = lo[i] + Op::widen((uint16_t)(r[i / 2] >> (16 * (i & 1))));
            v[4 + i] = hi[i] + Op::widen((uint16_t)(r[2 + i / 2] >> (16 * (i & 1))));
        }
        if (p.relu) {
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] = relu_bits(v[i]);
        }
        return u32x4_t{Op::pack(v[0], v[1]), Op::pack(v[2], v[3]), Op::pack(v[4], v[5]), Op::pack(v[6], v[7])};
    };
    // the same, one element at a time (ragged edges)
    auto finish1 = [&](int row, int col, const uint16_t *res) -> uint16_t {
        if (!p.residual) return tile16[row * kRowHalfs + col];
        float v = tile32[row * kRowFloats + col] + Op::widen(*res);
        if (p.relu) v = fmaxf(v, 0.f);
        return (uint16_t)Op::pack(v, 0.f);
    };
    if (NHWC) {
        constexpr int kParts = MB * 4;  // 16-byte pieces per pixel
        const int part = t % kParts;
        const int mch = mbase * 32 + part * 8;
        const bool whole = mch + 7 < p.M && (p.M & 7) == 0;
        if (p.pool) {
            // 2 x 2 max-pool: tile origins and sizes are even, so every window lies inside one tile (M % 8 == 0 here)
            constexpr int kTw2 = TW / 2;
            const int th2 = p.TH >> 1;
            for (int q = t / kParts; q < kTilePx / 4; q += kWgThreads / kParts) {
                const int qx = q & (kTw2 - 1), r = q / kTw2, qy = r & (th2 - 1), qn = r >> (p.th_log2 - 1);
                const int py = (ty0 >> 1) + qy, px = (tx0 >> 1) + qx, on = n0 + qn;
                if (on >= p.N || py >= p.Hp || px >= p.Wp || mch >= p.M) continue;
                const int op = ((qn << p.th_log2) + 2 * qy) * TW + 2 * qx;
                const u32x4_t a = *(const u32x4_t *)(tile16 + op * kRowHalfs + part * 8);
                const u32x4_t b = *(const u32x4_t *)(tile16 + (op + 1) * kRowHalfs + part * 8);
                const u32x4_t c = *(const u32x4_t *)(tile16 + (op + TW) * kRowHalfs + part * 8);
                const u32x4_t d = *(const u32x4_t *)(tile16 + (op + TW + 1) * kRowHalfs + part * 8);
                u32x4_t v;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    float m[2];
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        const int sh = 16 * h;
                        m[h] = fmaxf(fmaxf(Op::widen((uint16_t)(a[i] >> sh)), Op::widen((uint16_t)(b[i] >> sh))),
                                     fmaxf(Op::widen((uint16_t)(c[i] >> sh)), Op::widen((uint16_t)(d[i] >> sh))));
                    }
                    v[i] = Op::pack(m[0], m[1]);
                }
                const int64_t o = ((int64_t)(on * p.Hp + py) * p.Wp + px) * p.M + mch;
                __builtin_nontemporal_store(v, (u32x4_t *)(p.y + o));
            }
            return;
        }
#pragma unroll
        for (int op = t / kParts; op < kTilePx; op += kWgThreads / kParts) {
            const int po = pixtab[op];
            if (po < 0 || mch >= p.M) continue;
            const int64_t o = (int64_t)po * p.M + mch;
            if (whole) {
                __builtin_nontemporal_store(finish(op, part * 8, p.residual + o), (u32x4_t *)(p.y + o));
            } else {
                for (int i = 0; i < 8 && mch + i < p.M; ++i) p.y[o + i] = finish1(op, part * 8 + i, p.residual + o + i);
            }
        }
    } else {
        constexpr int kTwLog2 = TW == 8 ? 3 : TW == 16 ? 4 : 5;
        constexpr int kParts = 32;  // 16-byte pieces (8 pixels) per channel row
        const int part = t % kParts;
        const int op = part * 8, row = op >> kTwLog2;
        const int ox = tx0 + (op & (TW - 1)), oy = ty0 + (row & (p.TH - 1)), on = n0 + (row >> p.th_log2);
        const bool in = on < p.N && oy < p.Ho && ox < p.Wo;
        const int64_t plane = (int64_t)p.Ho * p.Wo;
        const int64_t o0 = ((int64_t)on * p.M * p.Ho + oy) * p.Wo + ox;
        const bool wide = ox + 7 < p.Wo && ((o0 | plane) & 7) == 0;
#pragma unroll 4
        for (int ml = t / kParts; ml < MB * 32; ml += kWgThreads / kParts) {
            const int mch = mbase * 32 + ml;
            if (!in || mch >= p.M) continue;
            const int64_t o = o0 + mch * plane;
            if (wide) {
                __builtin_nontemporal_store(finish(ml, op, p.residual + o), (u32x4_t *)(p.y + o));
            } else {
                for (int i = 0; i < 8 && ox + i < p.Wo; ++i) p.y[o + i] = finish1(ml, op + i, p.residual + o + i);
            }
        }
    }
}

// One launcher per (dtype, stride); each lives in a source file of its own so that the instances compile in parallel.
typedef int (*fused_launcher_t)(const FusedParams &p, int TW, bool big, int mb, bool nhwc, int npb, bool self, bool tap2,
                                dim3 grid, size_t lds_bytes, hipStream_t s);
// (mb = 0 selects the depthwise-only instances, NHWC; npb = 1, the 128-pixel-tile instances, exists for NHWC; self,
// the workgroups without loader waves, for NHWC, stride 1, npb = 1 and mb = 0 or 2)
int launch_fused_bf16_s1(const FusedParams &, int, bool, int, bool, int, bool, bool, dim3, size_t, hipStream_t);
int launch_fused_bf16_s2(const FusedParams &, int, bool, int, bool, int, bool, bool, dim3, size_t, hipStream_t);
int launch_fused_f16_s1(const FusedParams &, int, bool, int, bool, int, bool, bool, dim3, size_t, hipStream_t);
int launch_fused_f16_s2(const FusedParams &, int, bool, int, bool, int, bool, bool, dim3, size_t, hipStream_t);

template <int DTYPE, int TW, int STRIDE, bool BIG, int MB, bool NHWC, bool GDWONLY = false, int NPB = 2, bool SELF = false,
          bool TAP2 = false>
int launch_instance(const FusedParams &p, dim3 grid, size_t lds_bytes, hipStream_t s)
{
    auto kern = gdws_fused_kernel<DTYPE, TW, STRIDE, BIG, MB, NHWC, GDWONLY, NPB, SELF, TAP2>;
    static bool raised = false;  // one flag per kernel instance
    if (!raised) {
        GDWS_HIP_CHECK(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
        raised = true;
    }
    kern<<<grid, SELF ? kComputeThreads : kThreads, lds_bytes, s>>>(p);
    GDWS_HIP_CHECK(hipGetLastError());
    return GDWS_OK;
}

template <int DTYPE, int STRIDE>
int launch_dispatch(const FusedParams &p, int TW, bool big, int mb, bool nhwc, int npb, bool self, bool tap2, dim3 grid,
                    size_t lds_bytes, hipStream_t s)
{
    if (tap2) {  // (the two-tap depthwise stage: NHWC, both strides, with loader waves, or without for 64-channel workgroups)
        if (!nhwc || mb == 0) return GDWS_EUNSUPPORTED;
#define GDWS_CASE_T2(tw, bg, m, np, sf)                                                               \
    if (TW == tw && big == bg && mb == m && npb == np && self == sf)                                  \
        return launch_instance<DTYPE, tw, STRIDE, bg, m, true, false, np, sf, true>(p, grid, lds_bytes, s);
#define GDWS_CASES_T2(tw)                                                                             \
    GDWS_CASE_T2(tw, false, 2, 2, false) GDWS_CASE_T2(tw, false, 4, 2, false) GDWS_CASE_T2(tw, true, 2, 2, false)   \
    GDWS_CASE_T2(tw, true, 4, 2, false) GDWS_CASE_T2(tw, false, 2, 1, false) GDWS_CASE_T2(tw, false, 4, 1, false)   \
    GDWS_CASE_T2(tw, true, 2, 1, false) GDWS_CASE_T2(tw, true, 4, 1, false)
        GDWS_CASES_T2(4) GDWS_CASES_T2(8) GDWS_CASES_T2(16) GDWS_CASES_T2(32)
        if constexpr (STRIDE == 1) {
            GDWS_CASE_T2(4, false, 2, 1, true) GDWS_CASE_T2(4, true, 2, 1, true) GDWS_CASE_T2(8, false, 2, 1, true)
            GDWS_CASE_T2(8, true, 2, 1, true) GDWS_CASE_T2(16, false, 2, 1, true) GDWS_CASE_T2(16, true, 2, 1, true)
            GDWS_CASE_T2(32, false, 2, 1, true) GDWS_CASE_T2(32, true, 2, 1, true)
        }
#undef GDWS_CASES_T2
#undef GDWS_CASE_T2
        return GDWS_EUNSUPPORTED;
    }
    if constexpr (STRIDE == 1) {
        if (self) {
#define GDWS_CASE_SELF(tw, bg)                                                                        \
    if (TW == tw && big == bg && mb == 2 && nhwc && npb == 1)                                         \
        return launch_instance<DTYPE, tw, STRIDE, bg, 2, true, false, 1, true>(p, grid, lds_bytes, s);    \
    if (TW == tw && big == bg && mb == 0 && nhwc && npb == 1)                                         \
        return launch_instance<DTYPE, tw, STRIDE, bg, 2, true, true, 1, true>(p, grid, lds_bytes, s);
            GDWS_CASE_SELF(4, false) GDWS_CASE_SELF(4, true) GDWS_CASE_SELF(8, false) GDWS_CASE_SELF(8, true)
            GDWS_CASE_SELF(16, false) GDWS_CASE_SELF(16, true) GDWS_CASE_SELF(32, false) GDWS_CASE_SELF(32, true)
#undef GDWS_CASE_SELF
            return GDWS_EUNSUPPORTED;
        }
    } else if (self) {
        return GDWS_EUNSUPPORTED;
    }
#define GDWS_CASE(tw, bg, m, nh, np)                                                                  \
    if (TW == tw && big == bg && mb == m && nhwc == nh && npb == np)                                  \
        return launch_instance<DTYPE, tw, STRIDE, bg, m, nh, false, np>(p, grid, lds_bytes, s);
#define GDWS_CASE_GDW(tw, bg, np)                                                                     \
    if (TW == tw && big == bg && mb == 0 && nhwc && npb == np)                                        \
        return launch_instance<DTYPE, tw, STRIDE, bg, 2, true, true, np>(p, grid, lds_bytes, s);
#define GDWS_CASES(tw)                                                                                \
    GDWS_CASE(tw, false, 2, false, 2) GDWS_CASE(tw, false, 2, true, 2) GDWS_CASE(tw, false, 4, false, 2)  \
    GDWS_CASE(tw, false, 4, true, 2) GDWS_CASE(tw, true, 2, false, 2) GDWS_CASE(tw, true, 2, true, 2)     \
    GDWS_CASE(tw, true, 4, false, 2) GDWS_CASE(tw, true, 4, true, 2) GDWS_CASE_GDW(tw, false, 2)          \
    GDWS_CASE_GDW(tw, true, 2) GDWS_CASE(tw, false, 4, true, 1) GDWS_CASE(tw, true, 4, true, 1)             \
    GDWS_CASE(tw, false, 2, true, 1) GDWS_CASE(tw, true, 2, true, 1) GDWS_CASE_GDW(tw, false, 1)            \
    GDWS_CASE_GDW(tw, true, 1)
// tiles four pixels wide (images up to four pixels wide): NHWC only
#define GDWS_CASES_NARROW(tw)                                                                         \
    GDWS_CASE(tw, false, 2, true, 2) GDWS_CASE(tw, false, 4, true, 2) GDWS_CASE(tw, true, 2, true, 2)     \
    GDWS_CASE(tw, true, 4, true, 2) GDWS_CASE_GDW(tw, false, 2) GDWS_CASE_GDW(tw, true, 2)                \
    GDWS_CASE(tw, false, 4, true, 1) GDWS_CASE(tw, true, 4, true, 1) GDWS_CASE(tw, false, 2, true, 1)     \
    GDWS_CASE(tw, true, 2, true, 1) GDWS_CASE_GDW(tw, false, 1) GDWS_CASE_GDW(tw, true, 1)
    GDWS_CASES_NARROW(4) GDWS_CASES(8) GDWS_CASES(16) GDWS_CASES(32)
#undef GDWS_CASES_NARROW
#undef GDWS_CASES
#undef GDWS_CASE_GDW
#undef GDWS_CASE
    return GDWS_EUNSUPPORTED;
}

}  // namespace fusedk
}  // namespace gdws
