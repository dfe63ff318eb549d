// Fused GDWS kernel for the deep layers of a network: few pixels, many input and output channels
// (K = 3, stride 1, pad 1, 16-bit NHWC, 128 < C <= 512, M >= 256).
//
// On such layers the general fused kernel (fused_kernel.h) has to cut the output channels into slices of 64 to get
// a workgroup per CU, and every slice repeats the depthwise stage of the tile, which is most of a row block's
// instructions.  Here the four waves of a workgroup share ONE block of 32 output pixels and split the output
// channels instead (64 each, 256 per workgroup): the row blocks are taken four at a time, wave w computes the
// depthwise stage of row block 4 k + w for the 32 pixels (one dense and four sparse MFMAs, as in the general kernel:
// A from the row block's record, B a 16-byte LDS read of the input tile, the middle tap of a filter row from the
// neighbouring lanes), rounds the 32 x 32 result and puts it into LDS in the layout the pointwise MFMA wants for its B operand
// (16 bytes per lane and K-step: conflict-free to write and to read); after a barrier every wave runs the
// pointwise MFMAs of all four row blocks against its own 64 output channels.  The depthwise work of a tile is thus
// done once per 256 output channels, and a wave issues 21 MFMAs per group of four row blocks where the general
// kernel's 64-channel slices issue 36.
//
// The whole input tile (32 pixels with halo, all C channels, pixel-major, 16 bytes of padding per pixel) is loaded
// into LDS by the four waves before the first row block: one stage, no loader waves.  Records, pointwise
// fragments and bias are the general kernel's (build_fused_schedule with its deep_stage argument: one stage, the
// row blocks padded to a multiple of four, the output channels to a multiple of 256).
//
// Small launches (a batch of one or two images: a handful of pixel blocks) additionally split the groups of row blocks
// over workgroups (SPLIT): workgroup z takes a run of groups, loads only the input channels those draw on, and writes
// its fp32 partial sums to a workspace; a second kernel adds the partial sums in a fixed order, then bias, residual,
// ReLU, rounding (and the 2 x 2 max-pool).  The chain of row blocks that one workgroup walks through is what such a
// launch waits for; cut into S runs it is S times shorter.
#include <algorithm>

#include "fused_kernel.h"

namespace gdws {

using namespace fusedk;

namespace {

constexpr int kDeepThreads = 256;
constexpr int kDeepPx = 32;                  // output pixels per workgroup
constexpr int kDeepMbWave = 2;               // 32-wide blocks of output channels per wave
constexpr int kDeepMbWg = 4 * kDeepMbWave;   // per workgroup: 256 channels
constexpr int kDeepMaxLds = 160 * 1024;
constexpr int kTSlotDwords = 2 * 4 * 2 * 64 * 4;  // two buffers x four row blocks x two K-steps x 64 lanes x 16 bytes

struct DeepParams {
    const uint16_t *x;
    uint16_t *y;
    const uint16_t *residual;
    const float *bias;
    const u32x4_t *rec_a;
    const u32x2_t *rec_b;
    const u32x4_t *pwfrag;
    int n_groups;  // row blocks / 4
    int m_blocks_pad, relu;
    int N, C, H, W, M, Ho, Wo;
    int TH, TN, IH, th_log2;
    uint32_t x_bytes;
    int tiles_x, tiles_y;
    int tslot_off;  // dword offset in LDS of the intermediate's slots (behind the input tile)
    int lut_off;    // dword offset in LDS of the table of A-operand selectors (behind the slots)
    int pool, Hp, Wp;
    // SPLIT: groups per workgroup, per-group channel ranges (lo | hi << 16), the partial sums [slice][pixel][channel]
    int groups_per_slice;
    const uint32_t *group_chan;
    float *part;
    int64_t part_slice;  // floats per slice: pixels of y x padded channels
};

// CS: channels the LDS tile holds per pixel (256 or 512).
template <int DTYPE, int TW, int CS, bool SPLIT>
__global__ __launch_bounds__(kDeepThreads, 1) void gdws_deep_kernel(DeepParams params)
{
    using Op = half_ops<DTYPE>;
    const DeepParams &p = params;
    constexpr int PSW = CS / 2 + 4;  // dwords per LDS pixel
    constexpr int IW = TW + 2;
    constexpr int QP = CS / 8;       // 16-byte pieces per pixel
    extern __shared__ uint32_t lds[];

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l32 = lane & 31, lhi = lane >> 5;
    int tile = blockIdx.x;
    const int tx0 = (tile % p.tiles_x) * TW; tile /= p.tiles_x;
    const int ty0 = (tile % p.tiles_y) * p.TH;
    const int n0 = (tile / p.tiles_y) * p.TN;
    const int mslice = blockIdx.y;                                // 256 output channels
    const int mb0 = mslice * kDeepMbWg + wave * kDeepMbWave;      // the wave's first 32-wide block of them

    // the workgroup's groups of row blocks: all of them, or its run of them
    const int g_begin = SPLIT ? (int)blockIdx.z * p.groups_per_slice : 0;
    const int g_end = SPLIT ? min(g_begin + p.groups_per_slice, p.n_groups) : p.n_groups;

    // ---- records and pointwise fragments of the first group: requested before anything else ----
    const int r0 = g_begin * 4 + wave;
    u32x4_t ra = p.rec_a[r0 * 64 + lane], na = p.rec_a[(r0 + 4) * 64 + lane];
    u32x2_t rb = p.rec_b[r0 * 64 + lane], nb = p.rec_b[(r0 + 4) * 64 + lane];
    const int kstep_stride = p.m_blocks_pad * 64;          // 16-byte units per K-step of a row block
    const u32x4_t *fp = p.pwfrag + (int64_t)g_begin * 8 * kstep_stride + (int64_t)mb0 * 64 + lane;  // (first row block, K-step 0, the wave's blocks)
    u32x4_t pwf[4][2][kDeepMbWave];
#pragma unroll
    for (int s = 0; s < 4; ++s)
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
            for (int mb = 0; mb < kDeepMbWave; ++mb) pwf[s][s2][mb] = fp[(s * 2 + s2) * kstep_stride + mb * 64];

    // ---- the input tile: 16-byte pieces, consecutive threads along a pixel's channels ----
    // the table of A-operand selectors of the sparse depthwise stage (the barrier behind the tile's load orders it)
    if (threadIdx.x < 32) write_selector_entry(lds + p.lut_off + threadIdx.x * kLutEntry, threadIdx.x & 15u, threadIdx.x >> 4);
    constexpr uint32_t kOutside = 0x80000000u;  // beyond the descriptor's bound: the load returns zeros
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)p.x, 0, p.x_bytes, 0x00020000);
    if constexpr (SPLIT) {
        // only the channels the workgroup's row blocks draw on (the rest of the tile is never read): a few pieces per
        // pixel, dealt out over all threads so that they are in flight together
        const int lo = (int)(p.group_chan[g_begin] & 0xffffu), hi = (int)(p.group_chan[g_end - 1] >> 16);
        const int q_lo = lo / 8, nq = (hi + 7) / 8 - q_lo;
        const int total = p.TN * p.IH * IW * nq;
        constexpr int kBatch = 4;
        for (int i0 = threadIdx.x; i0 < total; i0 += kDeepThreads * kBatch) {
            u32x4_t v[kBatch];
            int dst[kBatch];
#pragma unroll
            for (int k = 0; k < kBatch; ++k) {
                const int i = i0 + kDeepThreads * k;
                const int pix = i / nq, q = q_lo + i - pix * nq;
                const int ix = pix % IW, r = pix / IW, iy = r % p.IH, tn = r / p.IH;
                const int n = n0 + tn, gy = ty0 - 1 + iy, gx = tx0 - 1 + ix;
                const bool in = i < total && q * 8 < p.C && n < p.N && (unsigned)gy < (unsigned)p.H && (unsigned)gx < (unsigned)p.W;
                const uint32_t pixel = __umul24(__umul24(n, p.H) + gy, p.W) + gx;
                v[k] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, in ? __umul24(pixel, (uint32_t)p.C * 2u) + q * 16 : kOutside, 0, 0);
                dst[k] = i < total ? pix * PSW + q * 4 : -1;
            }
#pragma unroll
            for (int k = 0; k < kBatch; ++k)
                if (dst[k] >= 0) *(u32x4_t *)(lds + dst[k]) = v[k];
        }
    } else {
        const int npix = p.TN * p.IH * IW;
        const int total = npix * QP;
        constexpr int kStepPix = kDeepThreads / QP;  // pixels from one of a thread's pieces to its next (4 or 8)
        constexpr int kStepX = kStepPix % IW, kStepY = kStepPix / IW;
        static_assert(kStepY <= 1, "the walk over the tile's pixels advances by less than two rows per step");
        const int q = threadIdx.x % QP;
        int pix = threadIdx.x / QP;
        int ix = pix % IW, iy, tn;
        {
            const int r = pix / IW;
            iy = r % p.IH; tn = r / p.IH;
        }
        const int gy0 = ty0 - 1, gx0 = tx0 - 1;
        const uint32_t c2 = (uint32_t)p.C * 2u;
        const bool chan_in = q * 8 < p.C;
        constexpr int kBatch = 8;
        for (int i0 = threadIdx.x; i0 < total; i0 += kDeepThreads * kBatch) {
            u32x4_t v[kBatch];
#pragma unroll
            for (int k = 0; k < kBatch; ++k) {
                const int n = n0 + tn, gy = gy0 + iy, gx = gx0 + ix;
                const bool in = chan_in && tn < p.TN && n < p.N && (unsigned)gy < (unsigned)p.H && (unsigned)gx < (unsigned)p.W;
                // 24-bit multiplies: the host admits fewer than 2^24 input pixels and x below 2 GiB
                const uint32_t pixel = __umul24(__umul24(n, p.H) + gy, p.W) + gx;
                const uint32_t off = in ? __umul24(pixel, c2) + q * 16 : kOutside;
                v[k] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, off, 0, 0);
                ix += kStepX; iy += kStepY;
                if (ix >= IW) { ix -= IW; ++iy; }
                if (iy >= p.IH) { iy -= p.IH; ++tn; }  // (IH >= 3 > the two rows a step can add)
            }
#pragma unroll
            for (int k = 0; k < kBatch; ++k) {
                const int i = i0 + kDeepThreads * k;
                if (i < total) *(u32x4_t *)(lds + (pix + kStepPix * k) * PSW + q * 4) = v[k];
            }
            pix += kStepPix * kBatch;
        }
    }
    __syncthreads();

    // ---- compute ----
    // LDS dword offset of the top-left tap of the lane's pixel, plus the lane's half of the 16-channel window
    int base;
    {
        const int tx = l32 % TW, ty = (l32 / TW) & (p.TH - 1), tn = (l32 / TW) >> p.th_log2;
        base = ((tn * p.IH + ty) * IW + tx) * PSW + lhi * 4;
    }
    // accumulators start from the bias: D[m][pixel], register i <-> channel 8 * (i / 4) + 4 * lhi + i % 4
    f32x16_t acc[kDeepMbWave];
#pragma unroll
    for (int mb = 0; mb < kDeepMbWave; ++mb) {
        const float *bp = p.bias + (mb0 + mb) * 32;  // padded with zeros to whole blocks
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
            f32x4_t bv = *(const f32x4_t *)(bp + 8 * q4 + 4 * lhi);
            if (SPLIT) bv = f32x4_t{0.f, 0.f, 0.f, 0.f};  // (the second kernel adds the bias)
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[mb][4 * q4 + i] = bv[i];
        }
    }
    f32x16_t zero;
#pragma unroll
    for (int i = 0; i < 16; ++i) zero[i] = 0.f;
    uint32_t *tslots = lds + p.tslot_off;

    auto tap_offset = [](int tap) { return ((tap / 3) * IW + (tap % 3)) * PSW; };
    auto read16 = [](const uint32_t *ptr) { return *(const u32x4_a8_t *)ptr; };
    // the six operands that come from LDS: left and right tap of each filter row
    u32x4_t bq[6];
    auto read_operands = [&](uint32_t ctrl) {
        const uint32_t *src = lds + base + (ctrl & 0xff);
#pragma unroll
        for (int i = 0; i < 6; ++i) bq[i] = read16(src + tap_offset(3 * (i / 2) + 2 * (i % 2)));
    };
    read_operands((uint32_t)__builtin_amdgcn_readfirstlane((int)rb[1]));
    // the current record's entry of the selector table: byte selectors for a pair of taps (sp) and for the first tap
    // (sd), and the index operand of the sparse MFMAs
    u32x4_t sp, sd;
    int sidx;
    auto read_lut = [&]() {
        const uint32_t *lut = lds + p.lut_off + (((rb[0] >> 16) & 15u) | (uint32_t)lhi << 4) * kLutEntry;
        sp = *(const u32x4_t *)lut;
        sd = *(const u32x4_t *)(lut + 4);
        sidx = (int)lut[8];
    };
    read_lut();

    for (int gi = g_begin; gi < g_end; ++gi) {
        // ---- depthwise stage of row block 4 gi + wave: tap 0 as a dense MFMA that starts from zero, then the pairs
        // (1,2), (3,4), (5,6), (7,8) on the sparse MFMA, as in the general kernel ----
        auto pair_a = [&](int i) {
            return u32x4_t{__builtin_amdgcn_perm(ra[i], ra[i], sp[0]), __builtin_amdgcn_perm(ra[i], ra[i], sp[1]),
                           __builtin_amdgcn_perm(ra[i], ra[i], sp[2]), __builtin_amdgcn_perm(ra[i], ra[i], sp[3])};
        };
        auto middle = [&](const u32x4_t &bl, const u32x4_t &br) {
            u32x4_t mid;
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                if constexpr (TW >= 8) {
                    // lanes 0-3 and 8-11 of a 16-lane row take the left tap of the next pixel, the others the
                    // right tap of the previous one: no lane reaches across the end of an 8-pixel tile row
                    const uint32_t x = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)bl[d], 0x101, 0xf, 0xf, true);
                    mid[d] = (uint32_t)__builtin_amdgcn_update_dpp((int)x, (int)br[d], 0x111, 0xf, 0xa, false);
                } else {
                    // four-pixel tile rows are the quads
                    const uint32_t nx = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)bl[d], 0xE9, 0xf, 0xf, false);
                    const uint32_t pv = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)br[d], 0x90, 0xf, 0xf, false);
                    mid[d] = (lane & 2) ? pv : nx;
                }
            }
            return mid;
        };
        const u32x4_t a_first = u32x4_t{__builtin_amdgcn_perm(rb[0], rb[0], sd[0]), __builtin_amdgcn_perm(rb[0], rb[0], sd[1]),
                                        __builtin_amdgcn_perm(rb[0], rb[0], sd[2]), __builtin_amdgcn_perm(rb[0], rb[0], sd[3])};
        f32x16_t t = Op::mfma(a_first, bq[0], zero);
        t = Op::smfmac(pair_a(0), middle(bq[0], bq[1]), bq[1], t, sidx);
        t = Op::smfmac(pair_a(1), bq[2], middle(bq[2], bq[3]), t, sidx);
        t = Op::smfmac(pair_a(2), bq[3], bq[4], t, sidx);
        t = Op::smfmac(pair_a(3), middle(bq[4], bq[5]), bq[5], t, sidx);
        // rounded to the storage type; register i of a lane is K element i % 8 of K-step i / 8 of the pointwise MFMA
        uint32_t *slot = tslots + ((gi & 1) * 4 + wave) * (2 * 64 * 4) + lane * 4;
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
            u32x4_t tb;
#pragma unroll
            for (int d = 0; d < 4; ++d)
                tb[d] = Op::pack(t[8 * s2 + 2 * d], t[8 * s2 + 2 * d + 1]);
            *(u32x4_t *)(slot + s2 * (64 * 4)) = tb;
        }
        // the next group's record becomes the current one; the one after it is requested
        {
            const uint32_t ri = (uint32_t)((gi + 2) * 4 + wave) * 64u + (uint32_t)lane;
            ra = na; rb = nb;
            na = p.rec_a[ri]; nb = p.rec_b[ri];
            read_lut();
        }
        __syncthreads();  // the four row blocks of the group are in LDS
        // the next group's operands are requested now: they arrive during the pointwise MFMAs
        read_operands((uint32_t)__builtin_amdgcn_readfirstlane((int)rb[1]));
        // ---- pointwise stage: four row blocks x two K-steps against the wave's 64 output channels ----
        fp += 8 * kstep_stride;  // the next group's fragments
        const uint32_t *tsrc = tslots + (gi & 1) * 4 * (2 * 64 * 4) + lane * 4;
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2) {
                const u32x4_t b = *(const u32x4_t *)(tsrc + (s * 2 + s2) * (64 * 4));
#pragma unroll
                for (int mb = 0; mb < kDeepMbWave; ++mb) {
                    acc[mb] = Op::mfma(pwf[s][s2][mb], b, acc[mb]);
                    pwf[s][s2][mb] = fp[(s * 2 + s2) * kstep_stride + mb * 64];
                }
            }
    }
    if constexpr (SPLIT) {
        // ---- the partial sums leave as they are: 16 bytes (four consecutive channels) per lane and store ----
        const int row = l32 / TW;
        const int ox = tx0 + (l32 & (TW - 1)), oy = ty0 + (row & (p.TH - 1)), on = n0 + (row >> p.th_log2);
        if (on >= p.N || oy >= p.Ho || ox >= p.Wo) return;
        const int64_t pix = ((int64_t)on * p.Ho + oy) * p.Wo + ox;
        float *dst = p.part + (int64_t)blockIdx.z * p.part_slice + pix * (p.m_blocks_pad * 32);
#pragma unroll
        for (int mb = 0; mb < kDeepMbWave; ++mb)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4)
                *(f32x4_t *)(dst + (mb0 + mb) * 32 + 8 * q4 + 4 * lhi) =
                    f32x4_t{acc[mb][4 * q4], acc[mb][4 * q4 + 1], acc[mb][4 * q4 + 2], acc[mb][4 * q4 + 3]};
        return;
    }
    __syncthreads();  // every wave is done with the input tile and the slots: the output tile may overwrite them

    // ---- epilogue, part 1: residual, ReLU, rounding in registers; the tile goes to LDS ----
    constexpr int kRowHalfs = kDeepMbWg * 32 + 8;  // [32 pixels][256 channels], rows padded by 16 bytes
    uint16_t *tile16 = (uint16_t *)lds;
    int *pixtab = (int *)(tile16 + kDeepPx * kRowHalfs);
    int my_pix;
    {
        const int row = l32 / TW;
        const int ox = tx0 + (l32 & (TW - 1)), oy = ty0 + (row & (p.TH - 1)), on = n0 + (row >> p.th_log2);
        my_pix = (on < p.N && oy < p.Ho && ox < p.Wo) ? (on * p.Ho + oy) * p.Wo + ox : -1;
        if (wave == 0 && lhi == 0) pixtab[l32] = my_pix;
    }
#pragma unroll
    for (int mb = 0; mb < kDeepMbWave; ++mb)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
            const int col = (wave * kDeepMbWave + mb) * 32 + 8 * q4 + 4 * lhi;  // four consecutive output channels
            const int mch = mslice * (kDeepMbWg * 32) + col;
            float v[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) v[i] = acc[mb][4 * q4 + i];
            if (p.residual && my_pix >= 0 && mch < p.M) {  // (M is a multiple of 8: the four channels are inside together)
                const u32x2_t r = *(const u32x2_t *)(p.residual + (int64_t)my_pix * p.M + mch);
#pragma unroll
                for (int i = 0; i < 4; ++i) v[i] += Op::widen((uint16_t)(r[i / 2] >> (16 * (i & 1))));
            }
            if (p.relu) {
#pragma unroll
                for (int i = 0; i < 4; ++i) v[i] = relu_bits(v[i]);
            }
            *(u32x2_t *)(tile16 + l32 * kRowHalfs + col) = u32x2_t{Op::pack(v[0], v[1]), Op::pack(v[2], v[3])};
        }
    __syncthreads();

    // ---- epilogue, part 2: LDS -> global in 16-byte pieces, 32 per pixel ----
    const int part = threadIdx.x % 32;
    const int mch = mslice * (kDeepMbWg * 32) + part * 8;
    if (mch >= p.M) return;
    if (p.pool) {
        // 2 x 2 max-pool: tile origins and sizes are even, so every window lies inside the tile; eight windows per tile
        constexpr int kTw2 = TW / 2;
        const int th2 = p.TH >> 1;
        const int q = threadIdx.x / 32;
        const int qx = q & (kTw2 - 1), r = q / kTw2, qy = r & (th2 - 1), qn = r >> (p.th_log2 - 1);
        const int py = (ty0 >> 1) + qy, px = (tx0 >> 1) + qx, on = n0 + qn;
        if (on >= p.N || py >= p.Hp || px >= p.Wp) return;
        const int op = ((qn << p.th_log2) + 2 * qy) * TW + 2 * qx;
        const u32x4_t a = *(const u32x4_t *)(tile16 + op * kRowHalfs + part * 8);
        const u32x4_t b = *(const u32x4_t *)(tile16 + (op + 1) * kRowHalfs + part * 8);
        const u32x4_t c = *(const u32x4_t *)(tile16 + (op + TW) * kRowHalfs + part * 8);
        const u32x4_t d = *(const u32x4_t *)(tile16 + (op + TW + 1) * kRowHalfs + part * 8);
        u32x4_t v;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float mx[2];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int sh = 16 * h;
                mx[h] = fmaxf(fmaxf(Op::widen((uint16_t)(a[i] >> sh)), Op::widen((uint16_t)(b[i] >> sh))),
                              fmaxf(Op::widen((uint16_t)(c[i] >> sh)), Op::widen((uint16_t)(d[i] >> sh))));
            }
            v[i] = Op::pack(mx[0], mx[1]);
        }
        const int64_t o = ((int64_t)(on * p.Hp + py) * p.Wp + px) * p.M + mch;
        __builtin_nontemporal_store(v, (u32x4_t *)(p.y + o));
        return;
    }
#pragma unroll
    for (int op = threadIdx.x / 32; op < kDeepPx; op += kDeepThreads / 32) {
        const int po = pixtab[op];
        if (po < 0) continue;
        const u32x4_t v = *(const u32x4_t *)(tile16 + op * kRowHalfs + part * 8);
        __builtin_nontemporal_store(v, (u32x4_t *)(p.y + (int64_t)po * p.M + mch));
    }
}

// Second kernel of a split launch: y (or its 2 x 2 max-pool) from the partial sums, 8 channels per thread.
struct DeepFinishParams {
    const float *part;
    int64_t part_slice;
    int slices, mpad;
    const float *bias;  // padded to mpad
    const uint16_t *residual;
    uint16_t *y;
    int relu, pool;
    int N, M, Ho, Wo, Hp, Wp;
};

template <int DTYPE>
__global__ __launch_bounds__(256) void gdws_deep_finish_kernel(DeepFinishParams p)
{
    using Op = half_ops<DTYPE>;
    const int parts = p.M / 8;
    // one thread per pixel of the layer's output and group of 8 channels; with the pooled epilogue the four pixels of a
    // window are four neighbouring lanes (the two lowest bits of the thread index), which then take their maximum
    const int64_t outs = (int64_t)p.N * (p.pool ? p.Hp * p.Wp * 4 : p.Ho * p.Wo);
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const bool live = i < outs * parts;
    const int sub = p.pool ? (int)(i & 3) : 0;
    const int64_t iq = p.pool ? i >> 2 : i;
    const int part = (int)(iq % parts), mch = part * 8;
    const int64_t o = iq / parts;
    int64_t pix = o;
    if (p.pool) {
        const int px = (int)(o % p.Wp), py = (int)((o / p.Wp) % p.Hp);
        const int64_t n = o / ((int64_t)p.Wp * p.Hp);
        pix = (n * p.Ho + 2 * py + (sub >> 1)) * p.Wo + 2 * px + (sub & 1);
    }
    // partial sums in slice order, bias, residual, ReLU, rounding
    float v[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) v[k] = 0.f;
    if (live) {
        // (the loads of eight slices go out together: one round trip to memory per batch instead of one per slice;
        // the additions stay in slice order)
        constexpr int kBatch = 8;
        const float *src0 = p.part + pix * p.mpad + mch;
        for (int z0 = 0; z0 < p.slices; z0 += kBatch) {
            f32x4_t a[kBatch], b[kBatch];
#pragma unroll
            for (int j = 0; j < kBatch; ++j) {
                const int z = z0 + j < p.slices ? z0 + j : z0;  // (past the last slice: read again, not added)
                const float *src = src0 + z * p.part_slice;
                a[j] = *(const f32x4_t *)src;
                b[j] = *(const f32x4_t *)(src + 4);
            }
#pragma unroll
            for (int j = 0; j < kBatch; ++j) {
                if (z0 + j < p.slices) {
#pragma unroll
                    for (int k = 0; k < 4; ++k) { v[k] += a[j][k]; v[4 + k] += b[j][k]; }
                }
            }
        }
#pragma unroll
        for (int k = 0; k < 8; ++k) v[k] += p.bias[mch + k];
        if (p.residual) {
            const u32x4_t r = *(const u32x4_t *)(p.residual + pix * p.M + mch);
#pragma unroll
            for (int k = 0; k < 8; ++k) v[k] += Op::widen((uint16_t)(r[k / 2] >> (16 * (k & 1))));
        }
        if (p.relu) {
#pragma unroll
            for (int k = 0; k < 8; ++k) v[k] = relu_bits(v[k]);
        }
    }
    u32x4_t out = u32x4_t{Op::pack(v[0], v[1]), Op::pack(v[2], v[3]), Op::pack(v[4], v[5]), Op::pack(v[6], v[7])};
    if (p.pool) {
        // the maximum of the rounded values of the window, as the separate pooling pass takes it
#pragma unroll
        for (int step = 1; step <= 2; step <<= 1) {
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const uint32_t other = (uint32_t)__shfl_xor((int)out[k], step);
                const float a0 = Op::widen((uint16_t)out[k]), a1 = Op::widen((uint16_t)(out[k] >> 16));
                const float b0 = Op::widen((uint16_t)other), b1 = Op::widen((uint16_t)(other >> 16));
                out[k] = Op::pack(fmaxf(a0, b0), fmaxf(a1, b1));
            }
        }
        if (sub) return;
    }
    if (live) *(u32x4_t *)(p.y + o * p.M + mch) = out;
}

template <int DTYPE, int TW, int CS, bool SPLIT>
int launch_deep_instance(const DeepParams &p, dim3 grid, size_t lds_bytes, hipStream_t s)
{
    auto kern = gdws_deep_kernel<DTYPE, TW, CS, SPLIT>;
    static bool raised = false;  // one flag per kernel instance
    if (!raised) {
        GDWS_HIP_CHECK(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, kDeepMaxLds));
        raised = true;
    }
    kern<<<grid, kDeepThreads, lds_bytes, s>>>(p);
    GDWS_HIP_CHECK(hipGetLastError());
    return GDWS_OK;
}

constexpr int64_t kDeepSplitBelow = 192;   // workgroups below which a launch is split over runs of row-block groups
constexpr int64_t kDeepSplitTarget = 256;  // ... into about this many workgroups

struct DeepTile {
    int TW, TH, TN, cs;
    size_t lds_bytes;
    double cost;
};

// The tile of 32 output pixels (TN images x TH rows x TW columns, TW 4 or 8) that wastes the fewest lanes.
DeepTile choose_deep_tile(int Ho, int Wo, int C, bool pool)
{
    DeepTile best{0, 0, 0, 0, ~(size_t)0, 1e30};
    const int cs = C <= 256 ? 256 : 512;
    for (int TW : {4, 8})
        for (int TH = pool ? 2 : 1; TH * TW <= kDeepPx; TH *= 2) {
            const int TN = kDeepPx / (TW * TH);
            const size_t npix = (size_t)TN * (TH + 2) * (TW + 2);
            const size_t in_bytes = npix * (cs / 2 + 4) * 4;
            const size_t out_bytes = (size_t)kDeepPx * (kDeepMbWg * 32 + 8) * 2 + kDeepPx * 4;
            const size_t lds = std::max(in_bytes + (size_t)kTSlotDwords * 4 + kLutBytes, out_bytes);
            if (lds > (size_t)kDeepMaxLds) continue;
            const double cover = (double)((Wo + TW - 1) / TW * TW) * ((Ho + TH - 1) / TH * TH) / ((double)Wo * Ho);
            const double halo = (double)(TH + 2) * (TW + 2) / (TH * TW);
            const double cost = cover * (1.0 + 0.15 * (halo - 1.0)) + 1e-4 * TN;
            if (cost < best.cost) best = DeepTile{TW, TH, TN, cs, lds, cost};
        }
    return best;
}

}  // namespace

bool deep_shape_supported(int dtype, int layout, int K, int stride, int pad, int C, int M)
{
    return (dtype == GDWS_BF16 || dtype == GDWS_F16) && layout == GDWS_NHWC && K == 3 && stride == 1 && pad == 1 &&
           C > 128 && C <= 512 && (C % 8) == 0 && M >= 256 && (M % 8) == 0;
}

// Workgroups the deep kernel would launch, or 0 if it cannot take the image.
int64_t deep_workgroups(const FusedSchedule &sc, int N, int C, int H, int W, int M, int Ho, int Wo, bool pool)
{
    if (!sc.valid) return 0;
    const int64_t x_bytes = (int64_t)N * C * H * W * 2;
    if (x_bytes >= ((int64_t)1 << 31) || (int64_t)N * H * W >= (1 << 24)) return 0;
    if (pool && ((Ho | Wo) & 1)) return 0;
    const DeepTile t = choose_deep_tile(Ho, Wo, C, pool);
    if (t.lds_bytes > (size_t)kDeepMaxLds) return 0;
    return (int64_t)((Wo + t.TW - 1) / t.TW) * ((Ho + t.TH - 1) / t.TH) * ((N + t.TN - 1) / t.TN) *
           ((M + kDeepMbWg * 32 - 1) / (kDeepMbWg * 32));
}

// Split of a small launch over runs of row-block groups: the number of runs, 1 if the launch is not split.
static int deep_slices(const FusedSchedule &sc, int64_t wgs)
{
    const int n_groups = sc.n_rowblocks / 4;
    if (wgs >= kDeepSplitBelow || n_groups < 2 || sc.group_chan.empty()) return 1;
    const int want = (int)std::min<int64_t>(n_groups, (kDeepSplitTarget + wgs - 1) / wgs);
    const int per = (n_groups + want - 1) / want;
    return (n_groups + per - 1) / per;
}

size_t deep_split_workspace_bytes(const FusedSchedule &sc, int N, int C, int H, int W, int M, int Ho, int Wo, bool pool)
{
    const int64_t wgs = deep_workgroups(sc, N, C, H, W, M, Ho, Wo, pool);
    if (!wgs) return 0;
    const int S = deep_slices(sc, wgs);
    return S > 1 ? (size_t)S * N * Ho * Wo * sc.m_blocks_pad * 32 * sizeof(float) : 0;
}

int launch_fused_deep(const FusedArgs &a, void *workspace, size_t workspace_bytes, hipStream_t s)
{
    const FusedSchedule &sc = *a.sched;
    if (!sc.valid || a.layout != GDWS_NHWC || a.stride != 1) return GDWS_EUNSUPPORTED;
    const int64_t wgs = deep_workgroups(sc, a.N, a.C, a.H, a.W, a.M, a.Ho, a.Wo, a.pool != 0);
    if (!wgs) return GDWS_EUNSUPPORTED;
    if (a.pool && a.ep.residual) return GDWS_EUNSUPPORTED;
    if (sc.n_rowblocks % 4 || sc.m_blocks_pad % kDeepMbWg) return GDWS_EINVAL;  // (not a deep schedule)
    const DeepTile t = choose_deep_tile(a.Ho, a.Wo, a.C, a.pool != 0);
    DeepParams p;
    p.x = (const uint16_t *)a.x; p.y = (uint16_t *)a.y;
    p.residual = (const uint16_t *)a.ep.residual; p.bias = sc.d_bias_pad;
    p.rec_a = (const u32x4_t *)sc.d_records;
    p.rec_b = (const u32x2_t *)(sc.d_records + (size_t)sc.record_slots * 64 * 4);
    p.pwfrag = (const u32x4_t *)sc.d_pwfrag;
    p.n_groups = sc.n_rowblocks / 4; p.m_blocks_pad = sc.m_blocks_pad; p.relu = a.ep.relu;
    p.N = a.N; p.C = a.C; p.H = a.H; p.W = a.W; p.M = a.M; p.Ho = a.Ho; p.Wo = a.Wo;
    p.TH = t.TH; p.TN = t.TN; p.IH = t.TH + 2;
    p.th_log2 = 0;
    while ((1 << p.th_log2) < t.TH) ++p.th_log2;
    p.x_bytes = (uint32_t)((int64_t)a.N * a.C * a.H * a.W * 2);
    p.tiles_x = (a.Wo + t.TW - 1) / t.TW;
    p.tiles_y = (a.Ho + t.TH - 1) / t.TH;
    p.tslot_off = t.TN * (t.TH + 2) * (t.TW + 2) * (t.cs / 2 + 4);
    p.lut_off = p.tslot_off + kTSlotDwords;
    p.pool = a.pool; p.Hp = a.Ho / 2; p.Wp = a.Wo / 2;
    p.groups_per_slice = p.n_groups; p.group_chan = sc.d_group_chan; p.part = nullptr; p.part_slice = 0;
    const int tiles_n = (a.N + t.TN - 1) / t.TN;
    // a small launch is split over runs of row-block groups when the caller's workspace can take the partial sums
    int S = deep_slices(sc, wgs);
    const size_t need = (size_t)S * a.N * a.Ho * a.Wo * sc.m_blocks_pad * 32 * sizeof(float);
    if (S > 1 && (!workspace || workspace_bytes < need || !sc.d_group_chan)) S = 1;
    if (S > 1) {
        p.groups_per_slice = (p.n_groups + S - 1) / S;
        p.part = (float *)workspace;
        p.part_slice = (int64_t)a.N * a.Ho * a.Wo * sc.m_blocks_pad * 32;
    }
    const dim3 grid((unsigned)((int64_t)p.tiles_x * p.tiles_y * tiles_n), (unsigned)(sc.m_blocks_pad / kDeepMbWg),
                    (unsigned)S);
    int rc = GDWS_EUNSUPPORTED;
#define GDWS_DEEP_CASE(DT_, TW_, CS_)                                                                  \
    if (a.dtype == DT_ && t.TW == TW_ && t.cs == CS_)                                                  \
        rc = S > 1 ? launch_deep_instance<DT_, TW_, CS_, true>(p, grid, t.lds_bytes, s)                \
                   : launch_deep_instance<DT_, TW_, CS_, false>(p, grid, t.lds_bytes, s);
    GDWS_DEEP_CASE(GDWS_BF16, 4, 256) GDWS_DEEP_CASE(GDWS_BF16, 4, 512) GDWS_DEEP_CASE(GDWS_BF16, 8, 256)
    GDWS_DEEP_CASE(GDWS_BF16, 8, 512) GDWS_DEEP_CASE(GDWS_F16, 4, 256) GDWS_DEEP_CASE(GDWS_F16, 4, 512)
    GDWS_DEEP_CASE(GDWS_F16, 8, 256) GDWS_DEEP_CASE(GDWS_F16, 8, 512)
#undef GDWS_DEEP_CASE
    if (rc != GDWS_OK || S == 1) return rc;
    DeepFinishParams f;
    f.part = p.part; f.part_slice = p.part_slice; f.slices = S; f.mpad = sc.m_blocks_pad * 32;
    f.bias = sc.d_bias_pad; f.residual = p.residual; f.y = p.y; f.relu = p.relu; f.pool = p.pool;
    f.N = a.N; f.M = a.M; f.Ho = a.Ho; f.Wo = a.Wo; f.Hp = p.Hp; f.Wp = p.Wp;
    const int64_t outs = (int64_t)a.N * (a.pool ? p.Hp * p.Wp * 4 : a.Ho * a.Wo) * (a.M / 8);
    if (outs == 0) return GDWS_OK;
    const dim3 fgrid((unsigned)((outs + 255) / 256));
    if (a.dtype == GDWS_BF16) gdws_deep_finish_kernel<GDWS_BF16><<<fgrid, 256, 0, s>>>(f);
    else gdws_deep_finish_kernel<GDWS_F16><<<fgrid, 256, 0, s>>>(f);
    GDWS_HIP_CHECK(hipGetLastError());
    return GDWS_OK;
}

}  // namespace gdws
