// Host side of the fused GDWS kernel: plan-time schedule (stages, chunks, row blocks, packed
// records and pointwise fragments), tile choice and launch.  The device code is in fused_kernel.h.
#include <algorithm>
#include <cstring>
#include <numeric>

#include "fused_kernel.h"

namespace gdws {

using namespace fusedk;

namespace {

constexpr int kMaxLds = 160 * 1024;
constexpr int kSmallGrid = 160;  // workgroups: below this a 256-CU chip is left more than a third idle
constexpr int kFullGrid = 256;   // workgroups: one per CU
constexpr int kWindowAlign = 4;  // channels: a window's 16-byte LDS reads are then 8-byte aligned

uint16_t to_half_bits(float v, int dtype)
{
    if (dtype == GDWS_BF16) return float_to_bf16(v);
    _Float16 h = (_Float16)v;
    uint16_t b;
    std::memcpy(&b, &h, 2);
    return b;
}

// Stage size class for a layer: all channels at once when they fit the larger class, else a double buffer
// of the smaller one.
struct StageGeometry {
    bool big;
    int stage_channels, chunk_channels, buffers;
};

StageGeometry stage_geometry(int stride, int C)
{
    const int small = stride == 1 ? 64 : 16, large = stride == 1 ? 128 : 32;
    StageGeometry sg;
    sg.chunk_channels = stride == 1 ? 32 : 16;
    if (C <= small) { sg.big = false; sg.stage_channels = small; sg.buffers = 1; }
    else if (C <= large) { sg.big = true; sg.stage_channels = large; sg.buffers = 1; }
    else { sg.big = false; sg.stage_channels = small; sg.buffers = 2; }
    return sg;
}

struct TileChoice {
    int TW, TH, TN;
    int IH, stage_w, th_log2;
    size_t lds_bytes;
    double cover;  // lanes per output pixel: tile pixels outside the image are wasted
};

// Pick the tile of tile_px (256, or 128) pixels (TN x TH x TW, all powers of two) that wastes the fewest lanes
// among those whose buffers fit LDS (and, NHWC, whose pixel count the loader's per-thread list can hold) and that
// have at least min_th rows; lds_bytes is SIZE_MAX if none does.
TileChoice choose_tile(int Ho, int Wo, int stride, int C, int mb, bool nhwc, bool residual, bool gdw_only = false,
                       int tile_px = 256, int min_th = 1, bool narrow = true)
{
    const StageGeometry sg = stage_geometry(stride, C);
    const int row_elems = nhwc ? mb * 32 : tile_px, rows = nhwc ? tile_px : mb * 32;
    const size_t out_bytes = (residual ? (size_t)rows * (row_elems + 4) * 4 : (size_t)rows * (row_elems + 8) * 2) +
                             (nhwc ? tile_px * 4 : 0);
    // NHWC loader: a thread holds one 16-byte piece of every pstep-th pixel; the last pass may run past the tile,
    // so a stage buffer holds whole passes
    const int pstep = kLoaderThreads / (sg.chunk_channels / 8);
    TileChoice best{8, 8, 4, 0, 0, 0, ~(size_t)0, 1e30};
    double best_cost = 1e30;
    for (int TW : {4, 8, 16, 32}) {
        // (four-pixel rows: NHWC, and only for images that narrow: they have the most halo per pixel)
        if (TW == 4 && (!narrow || !nhwc || Wo > 4)) continue;
        for (int TH = min_th; TH <= tile_px / TW; TH *= 2) {
            const int TN = tile_px / (TW * TH);
            const int IH = (TH - 1) * stride + 3, IW = (TW - 1) * stride + 3;
            const int npix = TN * IH * IW;
            const int nent = (npix + pstep - 1) / pstep;
            if (nhwc && nent > kMaxEnt) continue;
            // rows of IW pixels plus the row pad; the NHWC loader's last pass may run past the tile
            const int in_rows = nhwc ? (nent * pstep + IW - 1) / IW : TN * IH;
            const int stage_w = in_rows * (IW * lds_pixel_dwords(sg.stage_channels, stride) + lds_row_pad(TW, stride));
            // (depthwise-only mode: no output tile, but the waves' staging areas sit behind the input buffers)
            const size_t lds = ((gdw_only ? (size_t)sg.buffers * stage_w * 4 + (size_t)tile_px * 80
                                          : std::max((size_t)sg.buffers * stage_w * 4, out_bytes)) + 15) / 16 * 16 +
                               kLutBytes;
            if (lds > (size_t)kMaxLds) continue;
            const double cover = (double)((Wo + TW - 1) / TW * TW) * ((Ho + TH - 1) / TH * TH) / ((double)Wo * Ho);
            // halo rows/columns fetched per useful pixel; prefer fewer images per tile on ties
            const double halo = (double)(TH + 2) * (TW + 2) / (TH * TW);
            const double cost = cover * (1.0 + 0.15 * (halo - 1.0)) + 1e-4 * TN;
            if (cost < best_cost) {
                best_cost = cost;
                best = TileChoice{TW, TH, TN, IH, stage_w, 0, lds, cover};
            }
        }
    }
    while ((1 << best.th_log2) < best.TH) ++best.th_log2;
    return best;
}

}  // namespace

namespace {

// Row blocks a layer is cut into when a row block's rows must come from `window` input channels (the greedy cut of
// build_fused_schedule, counted only).
int count_row_blocks(int C, int stage_channels, const int32_t *offsets, int window)
{
    int n = 0;
    for (int c0 = 0; c0 < C; c0 += stage_channels) {
        const int cnt = std::min(stage_channels, C - c0), cfill = (cnt + 15) & ~15;
        int c = c0;  // channel of the next row
        int left = c < c0 + cnt ? offsets[c + 1] - offsets[c] : 0;
        auto skip_empty = [&]() { while (c < c0 + cnt && left == 0) { ++c; left = c < c0 + cnt ? offsets[c + 1] - offsets[c] : 0; } };
        skip_empty();
        while (c < c0 + cnt) {
            const int cb0 = std::min(((c - c0) / kWindowAlign) * kWindowAlign, cfill - window);
            int rows = 0;
            while (c < c0 + cnt && rows < kRowBlock && c - c0 - cb0 < window) {
                const int take = std::min(left, kRowBlock - rows);
                rows += take; left -= take;
                if (left == 0) { ++c; left = c < c0 + cnt ? offsets[c + 1] - offsets[c] : 0; skip_empty(); }
            }
            ++n;
        }
    }
    return n;
}

}  // namespace

void build_fused_schedule(FusedSchedule &s, int dtype, int stride, int C, int M, const int32_t *g,
                          const int32_t *offsets, const float *dw, const float *pw, const float *bias, bool gdw_only,
                          int deep_stage, bool allow_tap2)
{
    (void)g;
    const int G = offsets[C];
    s = FusedSchedule{};
    s.gdw_only = gdw_only;
    const StageGeometry sg = deep_stage ? StageGeometry{false, deep_stage, 32, 1} : stage_geometry(stride, C);
    s.stride = stride;
    s.big = sg.big;
    s.stage_channels = sg.stage_channels;
    s.chunk_channels = sg.chunk_channels;
    s.buffers = sg.buffers;
    s.m_blocks = (M + 31) / 32;
    s.mb_per_wg = deep_stage ? 8 : s.m_blocks >= 3 ? 4 : 2;
    // Depthwise stage on a 16-channel window (taps paired on the sparse MFMA) or on an 8-channel window (two taps per
    // dense MFMA, see the kernel): both take five matrix instructions per row block and pixel block; the second needs
    // fewer vector instructions (no lane exchange for the middle taps) but, with few filters per channel, more row
    // blocks.  Row-block costs in MFMA slots (the pointwise stage is 2 per 32 output channels; the vector
    // instructions of a row block counted as 5.5 and 4 slots: measured on config 2's g = 9 layer, where both cut the
    // layer into the same row blocks, and on the network shapes).
    s.tap2 = false;
    if (allow_tap2 && !gdw_only && !deep_stage && G > 0) {
        const int mbw = std::min(s.mb_per_wg, s.m_blocks);
        const double c16 = 5 + 2 * mbw + 5.5, c8 = 5 + 2 * mbw + 4;
        s.tap2 = count_row_blocks(C, sg.stage_channels, offsets, 8) * c8 < count_row_blocks(C, sg.stage_channels, offsets, kWindow) * c16;
    }
    const int window = s.tap2 ? 8 : kWindow;
    // the one-tap stage (general and deep-layer kernel) pairs taps on the sparse MFMA and reads its records in that form
    s.sparse = !s.tap2;
    s.m_blocks_pad = (s.m_blocks + s.mb_per_wg - 1) / s.mb_per_wg * s.mb_per_wg;
    s.bias_pad.assign((size_t)s.m_blocks_pad * 32, 0.f);
    if (bias) std::copy(bias, bias + M, s.bias_pad.begin());
    std::vector<int> chan(G);
    for (int c = 0; c < C; ++c)
        for (int j = offsets[c]; j < offsets[c + 1]; ++j) chan[j] = c;

    // rows[r] = intermediate channel in row r of the block, or -1
    auto push_fragments = [&](const int *rows) {
        // K-step s2, lane l = (m = l % 32, half = l / 32), element e  <->  row 16*s2 + 8*(e/4) + 4*half + e%4
        for (int s2 = 0; s2 < 2; ++s2)
            for (int mb = 0; mb < s.m_blocks_pad; ++mb)
                for (int l = 0; l < 64; ++l)
                    for (int e = 0; e < 8 && !gdw_only; ++e) {
                        const int m = mb * 32 + (l & 31), r = 16 * s2 + 8 * (e / 4) + 4 * (l >> 5) + (e % 4);
                        const int j = rows ? rows[r] : -1;
                        s.pwfrag.push_back(to_half_bits((m < M && j >= 0) ? pw[(size_t)m * G + j] : 0.f, dtype));
                    }
    };
    struct RowBlock {
        int c0, cb0, rows[kRowBlock];
        int stage;       // index among the non-empty stages
        int last_chunk;  // chunk barriers (counted over the whole layer) that must have passed before it runs
        uint32_t own;    // depthwise-only mode: first group of 8 channels | (groups - 1) << 10
    };
    std::vector<RowBlock> rbs;
    int chunk_base = 0;  // chunks of the stages before the current one
    if (gdw_only) {
        // Row blocks own whole groups of 8 consecutive intermediate channels (16-byte pieces of a row of T), up to the
        // padded channel count; rows past G have no filter and produce the zero padding.  A layer of several stages
        // (stride 1) loads stages that overlap by 8 input channels, so that a group whose filters sit on at most 8
        // consecutive input channels lies inside one stage; a group takes the first stage that holds it.
        const int Gp = (G + 15) & ~15;
        const bool multi = C > s.stage_channels;
        if (multi && stride != 1) { s.valid = false; return; }
        const int step = multi ? s.stage_channels - 8 : s.stage_channels;
        int jb = 0;
        for (int c0 = 0; c0 < C && jb < Gp; c0 += step) {
            const int cnt = std::min(s.stage_channels, C - c0);
            const int cfill = (cnt + 15) & ~15;
            // the channels of group jb .. jb + 7 lie in [c0, c0 + cnt)
            auto in_stage = [&](int j0) {
                for (int q = j0; q < std::min(j0 + 8, G); ++q)
                    if (chan[q] < c0 || chan[q] >= c0 + cnt) return false;
                return true;
            };
            const size_t first_rb = rbs.size();
            while (jb < Gp && (jb >= G || in_stage(jb))) {  // (padding follows the last group, in its stage)
                RowBlock rb;
                rb.c0 = c0;
                rb.stage = s.n_stages;
                const int jf = std::min(jb, G - 1);  // a block of padding only takes the last window
                rb.cb0 = std::min(((chan[jf] - c0) / kWindowAlign) * kWindowAlign, cfill - kWindow);
                int ng = 0;
                while (ng < 4 && jb + 8 * (ng + 1) <= Gp) {
                    bool fits = true;
                    for (int q = jb + 8 * ng; q < std::min(jb + 8 * (ng + 1), G); ++q)
                        fits = fits && chan[q] - c0 >= rb.cb0 && chan[q] - c0 - rb.cb0 < kWindow && chan[q] < c0 + cnt;
                    if (!fits) break;
                    ++ng;
                }
                if (ng == 0) { s.valid = false; return; }  // eight channels that span more than one window
                for (int r = 0; r < kRowBlock; ++r) rb.rows[r] = (r < 8 * ng && jb + r < G) ? jb + r : -1;
                rb.own = (uint32_t)(jb / 8) | ((uint32_t)(ng - 1) << 10);
                rb.last_chunk = chunk_base + (rb.cb0 + kWindow - 1) / s.chunk_channels + 1;
                rbs.push_back(rb);
                jb += 8 * ng;
            }
            if (rbs.size() == first_rb) continue;  // no group lies in this stage: it is never loaded
            s.stage_tab.push_back(c0);
            s.stage_tab.push_back(cnt);
            ++s.n_stages;
            chunk_base += (cfill + s.chunk_channels - 1) / s.chunk_channels;
        }
        if (jb < Gp) { s.valid = false; return; }  // a group spans more input channels than two stages share
    }
    for (int c0 = 0; c0 < C && !gdw_only; c0 += s.stage_channels) {
        const int cnt = std::min(s.stage_channels, C - c0);
        const int cfill = (cnt + 15) & ~15;
        int j = offsets[c0];
        const int jend = offsets[c0 + cnt];
        if (j == jend) continue;  // no filters on any channel of this stage: it is never loaded
        while (j < jend) {
            RowBlock rb;
            rb.c0 = c0;
            rb.stage = s.n_stages;
            // the 16-channel window starts at a multiple of 4 (8-byte aligned LDS reads) and stays inside the
            // zero-filled stage
            rb.cb0 = std::min(((chan[j] - c0) / kWindowAlign) * kWindowAlign, cfill - window);
            int nrows = 0;
            while (j < jend && nrows < kRowBlock && chan[j] - c0 - rb.cb0 < window) rb.rows[nrows++] = j++;
            for (int r = nrows; r < kRowBlock; ++r) rb.rows[r] = -1;
            rb.own = 0;
            rb.last_chunk = chunk_base + (rb.cb0 + window - 1) / s.chunk_channels + 1;
            rbs.push_back(rb);
        }
        s.stage_tab.push_back(c0);
        s.stage_tab.push_back(cnt);
        ++s.n_stages;
        chunk_base += (cfill + s.chunk_channels - 1) / s.chunk_channels;
    }
    s.n_chunks = chunk_base;
    while (deep_stage && !rbs.empty() && rbs.size() % 4) {  // empty row blocks: no rows, no weights
        RowBlock rb{};
        for (int r = 0; r < kRowBlock; ++r) rb.rows[r] = -1;
        // (their operands are read all the same and multiplied by zero: they take the last window, which every
        // workgroup that runs them has loaded -- stale LDS contents could be infinities or NaNs)
        rb.cb0 = rbs.back().cb0;
        rb.last_chunk = rbs.back().last_chunk;
        rbs.push_back(rb);
    }
    s.n_rowblocks = (int)rbs.size();
    if (deep_stage) {
        // per group of four row blocks, the input channels its windows reach (padding row blocks have no rows)
        for (size_t k = 0; k < rbs.size(); k += 4) {
            int lo = 1 << 15, hi = 0;
            for (size_t r = k; r < k + 4; ++r)
                if (rbs[r].rows[0] >= 0) { lo = std::min(lo, rbs[r].cb0); hi = std::max(hi, rbs[r].cb0 + kWindow); }
            if (hi == 0) lo = 0;
            s.group_chan.push_back((uint32_t)lo | ((uint32_t)hi << 16));
        }
    }
    // all-zero records behind the last row block: the general kernel reads two row blocks ahead, the deep-layer
    // kernel two groups of four
    const size_t slots = rbs.size() + (deep_stage ? 8 : 2);
    s.record_slots = (int)slots;
    s.records.assign(slots * 64 * 6, 0u);
    uint32_t *rec_a = s.records.data(), *rec_b = s.records.data() + slots * 64 * 4;
    int passed = 0;  // chunk barriers the compute waves have executed so far
    s.valid = s.n_rowblocks > 0;
    for (size_t k = 0; k < rbs.size(); ++k) {
        const RowBlock &rb = rbs[k];
        const int nwait = std::max(0, rb.last_chunk - passed);
        if (nwait > 15) s.valid = false;  // the wait count of a record has four bits
        passed += nwait;
        const bool new_stage = k > 0 && rb.stage != rbs[k - 1].stage && s.buffers == 2;
        bool chain = false;
        if (k + 1 < rbs.size()) {
            const RowBlock &nx = rbs[k + 1];
            chain = nx.stage == rb.stage && nx.last_chunk <= passed;
        }
        uint32_t ctrl = (uint32_t)(rb.cb0 / 2) | ((uint32_t)(nwait & 15) << 8);
        if (new_stage) ctrl |= kCtrlNewStage;
        if (chain) ctrl |= kCtrlChainNext;
        // (the next window of the same stage is stored also without the chain bit: workgroups without loader waves
        // have the whole stage in LDS and read ahead regardless)
        if (k + 1 < rbs.size() && rbs[k + 1].stage == rb.stage) ctrl |= (uint32_t)(rbs[k + 1].cb0 / 2) << 16;
        for (int l = 0; l < 64; ++l) {
            const int jr = rb.rows[l & 31];
            uint32_t *qa = rec_a + (k * 64 + l) * 4, *qb = rec_b + (k * 64 + l) * 2;
            uint32_t sel = 4;
            if (jr >= 0) {
                uint16_t h[9];
                for (int t = 0; t < 9; ++t) h[t] = to_half_bits(dw[(size_t)jr * 9 + t], dtype);
                if (s.sparse) {
                    // tap 0 alone, then the pairs (1,2), (3,4), (5,6), (7,8); the select field is the row's column
                    // of the window, the same in both halves of the lanes
                    for (int d = 0; d < 4; ++d) qa[d] = (uint32_t)h[2 * d + 1] | ((uint32_t)h[2 * d + 2] << 16);
                    qb[0] = h[0];
                    sel = (uint32_t)(chan[jr] - rb.c0 - rb.cb0);
                } else {
                    for (int d = 0; d < 4; ++d) qa[d] = (uint32_t)h[2 * d] | ((uint32_t)h[2 * d + 1] << 16);
                    qb[0] = h[8];
                    // two-tap stage: both halves of the lanes hold the same 8 channels, each for its own tap; the
                    // row's only column is the channel
                    const int pos = chan[jr] - rb.c0 - rb.cb0;
                    if (pos >= 0 && pos < 8) sel = (uint32_t)(pos / 2) | ((pos & 1) ? 8u : 0u);
                }
            }
            if (s.sparse && jr < 0) sel = 0;  // (a row without a filter: all taps zero, any column)
            qb[0] |= (sel << 16) | (rb.own << 20);
            qb[1] = ctrl;
        }
        push_fragments(rb.rows);
    }
    s.final_waits = s.n_chunks - passed;
    for (int k = 0; k < (deep_stage ? 4 : 1); ++k) push_fragments(nullptr);  // read ahead by one row block (one group)
}

bool fused_shape_supported(int dtype, int layout, int K, int stride, int pad, int C, int M)
{
    (void)M;
    if (dtype != GDWS_BF16 && dtype != GDWS_F16) return false;
    if (K != 3 || pad != 1 || (stride != 1 && stride != 2)) return false;
    if (layout == GDWS_NHWC && (C % 8) != 0) return false;  // 16-byte channel vectors
    return true;
}

bool fused_image_supported(const FusedSchedule &s, int layout, int stride, int C, int Ho, int Wo, bool residual,
                           int64_t x_elems)
{
    // the loader addresses x with 31-bit byte offsets and 24-bit pixel indices
    if (!s.valid || x_elems * 2 >= ((int64_t)1 << 31) || x_elems / C >= (1 << 24)) return false;
    if (s.gdw_only && layout != GDWS_NHWC) return false;
    return choose_tile(Ho, Wo, stride, C, s.mb_per_wg, layout == GDWS_NHWC, residual, s.gdw_only).lds_bytes <=
           (size_t)kMaxLds;
}

int launch_fused(const FusedArgs &a, hipStream_t s)
{
    const FusedSchedule &sc = *a.sched;
    if (!sc.valid) return GDWS_EUNSUPPORTED;
    const bool nhwc = a.layout == GDWS_NHWC;
    if (sc.gdw_only && !nhwc) return GDWS_EUNSUPPORTED;
    const bool res = a.ep.residual != nullptr;
    auto wgs = [&](const TileChoice &t, int m) {
        return (int64_t)((a.Wo + t.TW - 1) / t.TW) * ((a.Ho + t.TH - 1) / t.TH) * ((a.N + t.TN - 1) / t.TN) *
               (sc.gdw_only ? 1 : sc.m_blocks_pad / m);
    };
    TileChoice tc;
    int mb, npb;
    auto configure = [&](bool narrow) {
        auto pick = [&](int m, bool gdw_only, int tile_px) {  // (the pooled epilogue needs its 2 x 2 windows inside a tile)
            return choose_tile(a.Ho, a.Wo, a.stride, a.C, m, nhwc, res, gdw_only, tile_px, a.pool ? 2 : 1, narrow);
        };
        tc = pick(sc.mb_per_wg, sc.gdw_only, 256);
        mb = sc.mb_per_wg; npb = 2;
        if (tc.lds_bytes > (size_t)kMaxLds) return;
        // A workgroup covers 256 pixels x 128 output channels (or 64).  When that grid is too small to fill the chip
        // it is doubled: NHWC, first by 128-pixel tiles (half the MFMAs per row block and wave); then, or else, by
        // 64-channel slices (each workgroup repeats the depthwise stage but has half the pointwise work).
        if (mb == 4 && !sc.gdw_only) {
            if (nhwc) {
                // (also when only the smaller tile has a shape that fits the image: four-pixel rows with their halo,
                // double-buffered, fit LDS at 128 pixels but not at 256)
                const TileChoice t1 = pick(4, false, 128);
                if (t1.lds_bytes <= (size_t)kMaxLds && (wgs(tc, mb) <= kSmallGrid || t1.cover < 0.75 * tc.cover)) {
                    tc = t1; npb = 1;
                }
            }
            if (wgs(tc, mb) <= kSmallGrid) {
                const TileChoice t2 = pick(2, false, 128 * npb);
                if (t2.lds_bytes <= (size_t)kMaxLds) { tc = t2; mb = 2; }
            }
        }
        // 64-channel workgroups on 128-pixel tiles need 112 registers per wave, so two of them are resident per CU
        // and one's loading and storing overlaps the other's arithmetic: taken whenever both fit LDS.
        if (npb == 2 && nhwc && (mb == 2 || sc.gdw_only)) {  // (the depthwise-only instances need 107 registers)
            const TileChoice t1 = pick(2, sc.gdw_only, 128);
            if (t1.lds_bytes <= (size_t)kMaxLds / 2) { tc = t1; npb = 1; }
        }
    };
    // Tiles four pixels wide waste fewer lanes on images that narrow, but their LDS reads are slower (measured: a
    // row block takes a quarter longer): they pay when the lanes saved shorten the work of a full chip, not when the
    // grid they leave is smaller than the chip.
    configure(true);
    if (tc.TW == 4 && wgs(tc, mb) < kFullGrid) configure(false);
    if (tc.lds_bytes > (size_t)kMaxLds) return GDWS_EUNSUPPORTED;
    // the pooled epilogue: whole 16-byte pieces, the 16-bit tile, windows inside a tile
    if (a.pool && (!nhwc || sc.gdw_only || res || (a.M & 7) || tc.TH < 2)) return GDWS_EUNSUPPORTED;
    const int64_t x_bytes = (int64_t)a.N * a.C * a.H * a.W * 2;
    if (x_bytes >= ((int64_t)1 << 31) || (int64_t)a.N * a.H * a.W >= (1 << 24)) return GDWS_EUNSUPPORTED;
    // (depthwise-only mode: T is stored through a buffer descriptor with 32-bit offsets)
    const int64_t y_bytes = sc.gdw_only ? (int64_t)a.N * a.Ho * a.Wo * a.M * 2 : 0;
    if (y_bytes >= ((int64_t)1 << 31)) return GDWS_EUNSUPPORTED;
    FusedParams p;
    p.x = (const uint16_t *)a.x; p.y = (uint16_t *)a.y;
    p.residual = (const uint16_t *)a.ep.residual; p.bias = sc.d_bias_pad;
    p.stage_tab = sc.d_stage_tab;
    p.rec_a = (const u32x4_t *)sc.d_records;
    p.rec_b = (const u32x2_t *)(sc.d_records + (size_t)sc.record_slots * 64 * 4);
    p.pwfrag = (const u32x4_t *)sc.d_pwfrag;
    p.n_stages = sc.n_stages; p.n_rowblocks = sc.n_rowblocks; p.final_waits = sc.final_waits;
    p.m_blocks_pad = sc.m_blocks_pad; p.relu = a.ep.relu;
    p.N = a.N; p.C = a.C; p.H = a.H; p.W = a.W; p.M = a.M; p.Ho = a.Ho; p.Wo = a.Wo;
    p.TH = tc.TH; p.TN = tc.TN; p.IH = tc.IH; p.th_log2 = tc.th_log2;
    p.stage_w = tc.stage_w; p.x_bytes = (uint32_t)x_bytes; p.y_bytes = (uint32_t)y_bytes;
    p.c_begin0 = sc.stage_tab[0]; p.c_count0 = sc.stage_tab[1];
    p.pool = a.pool; p.Hp = a.Ho / 2; p.Wp = a.Wo / 2;
    p.out_off = stage_geometry(a.stride, a.C).buffers * tc.stage_w;
    p.lut_off = (int)((tc.lds_bytes - kLutBytes) / 4);
    p.tiles_x = (a.Wo + tc.TW - 1) / tc.TW;
    p.tiles_y = (a.Ho + tc.TH - 1) / tc.TH;
    const int tiles_n = (a.N + tc.TN - 1) / tc.TN;
    const dim3 grid((unsigned)((int64_t)p.tiles_x * p.tiles_y * tiles_n),
                    sc.gdw_only ? 1u : (unsigned)(sc.m_blocks_pad / mb));
    fused_launcher_t fn;
    if (a.dtype == GDWS_BF16) fn = a.stride == 1 ? launch_fused_bf16_s1 : launch_fused_bf16_s2;
    else fn = a.stride == 1 ? launch_fused_f16_s1 : launch_fused_f16_s2;
    // Layers of one input stage whose workgroups are the small ones: without loader waves (see the kernel), when
    // LDS then holds three or more workgroups per CU.
    const bool self = nhwc && a.stride == 1 && npb == 1 && (mb == 2 || sc.gdw_only) && sc.n_stages == 1 &&
                      tc.lds_bytes <= (size_t)kMaxLds / 3;
    return fn(p, tc.TW, sc.big, sc.gdw_only ? 0 : mb, nhwc, npb, self, sc.tap2, grid, tc.lds_bytes, s);
}

}  // namespace gdws
