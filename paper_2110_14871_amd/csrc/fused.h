// Fused depthwise -> pointwise kernel for K = 3, 16-bit storage: plan-time schedule and launcher.
//
// Work decomposition.  A workgroup owns a tile of 256 output pixels (TN images x TH rows x TW
// columns) and up to 128 output channels; each of its four compute waves owns 64 of the pixels,
// four more waves stream the input channels, pixel-major, into LDS.  (Per launch the tile may be
// 128 pixels -- 32 per compute wave -- and the channel slice 64: see launch_fused.)  The input channels are cut
// into stages (all channels at once when they fit, else a double buffer) and every stage into
// chunks; a chunk is announced with a workgroup barrier as soon as it has landed, so the compute
// waves start on the first chunk while the rest of the stage is still in flight.
//
// Both stages of the layer run on the matrix cores.  The intermediate channels are cut, in channel
// order, into "row blocks" of at most 32 whose input channels fit one 16-channel window.  For a
// row block the depthwise stage is, per 32 pixels, one matrix instruction per filter tap or pair of taps: A
// is the 32 x 16 matrix that holds tap (u,v) of intermediate channel j in column chan_of[j] (one non-zero per
// row, built in registers from a per-lane tap value by byte permutes whose selectors depend only on the row's window
// column; two taps side by side are the 2:4 sparse operand of v_smfmac_f32_32x32x32), B is the 16-channel slice of
// the input tile shifted by (u,v), read straight from LDS.  The 32 x 32 fp32 result is rounded to the
// storage type in the lane that holds it and is, without any data movement, the B operand of the
// pointwise MFMAs (the pointwise weights are packed at plan time in the matching K order).
#pragma once
#include <vector>

#include "common.h"

namespace gdws {

constexpr int kRowBlock = 32;  // intermediate channels per row block
constexpr int kWindow = 16;    // input channels one row block may draw from (K of the depthwise MFMA)

// LDS layout of the input tile: pixel-major, a pixel's stage channels followed by padding, and every tile row followed
// by lds_row_pad dwords.  A window starts at a multiple of four channels, so the depthwise B operand (16 bytes per lane)
// is read as a pair of 8-byte halves.  Measured with a read-only loop (all four waves of a CU reading, 1 KB per
// wave-read): a pixel stride of 4 modulo 32 dwords (16 bytes of padding) serves such a read in 64 cycles, whatever the
// row pad; a stride of 2 modulo 4 dwords (8 bytes of padding) in 32 cycles when the 32 pixels of a block are two rows
// of 16 or one of 32, and with the row pad below also when they are four rows of 8 or eight of 4.  (Aligned 16-byte
// reads reach 20 cycles with a row pad of 56 dwords, but need windows at multiples of eight channels, which costs
// more row blocks than the reads save.)  At stride 2 neighbouring lanes are two pixels apart and no padding does
// better than 64 cycles: those tiles keep 16 bytes of padding (aligned LDS writes).
constexpr int lds_pixel_dwords(int stage_channels, int stride) { return stage_channels / 2 + (stride == 1 ? 2 : 4); }
constexpr int lds_row_pad(int tw, int stride) { return stride == 1 && tw <= 8 ? 28 : 0; }
// Behind everything else in LDS: the table of A-operand selectors of the sparse depthwise stage, 32 entries (window
// column x lane half) of kLutEntry dwords.
constexpr int kLutEntry = 12;
constexpr int kLutBytes = 32 * kLutEntry * 4;

// Record of a row block, per lane: six dwords in two arrays (16-byte and 8-byte loads).
//   a[0..3]  taps 0..7 of the lane's row, two per dword
//   b[0]     tap 8 | select << 16 | own << 20   (own, the same in all lanes, only in the depthwise-only mode:
//                                   bits 0-9 first group of 8 intermediate channels the row block owns, bits 10-11
//                                   number of groups - 1)   select: bits 0-2 = which of the lane's four A dwords holds the row's
//                                   only column (4: none of them), bit 3 = upper half of that dword
//   (this is the form of the two-tap depthwise stage; for the one-tap stage see FusedSchedule::sparse)
//   b[1]     control word, the same in all lanes (see kCtrl*)
constexpr uint32_t kCtrlNewStage = 1u << 12;   // the row block is the first of a stage that uses the other buffer
constexpr uint32_t kCtrlChainNext = 1u << 13;  // the next row block reads the same buffer and waits for no chunk
// bits 0-7: dword offset of the window inside an LDS pixel; bits 8-11: chunk barriers to pass before the row
// block; bits 16-23: window offset of the next row block

struct FusedSchedule {
    bool valid = false;
    bool gdw_only = false;   // depthwise stage alone: row blocks own whole groups of 8 intermediate channels, no
                             // pointwise fragments; only for layers that are a single stage
    bool tap2 = false;       // depthwise stage with two taps of an 8-channel window per MFMA (else one tap of 16 channels)
    bool sparse = false;     // records in the form of the sparse-MFMA depthwise stage (one tap of 16 channels, taps
                             // paired; general and deep-layer kernel): a[i] = taps 2i+1, 2i+2; b[0] = tap 0 | window
                             // column of the row << 16 | own << 20
    int stride = 1;
    bool big = false;        // stage size class: stride 1: 128 (else 64) channels, stride 2: 32 (else 16)
    int stage_channels = 0;  // input channels per LDS stage
    int chunk_channels = 0;  // channels per arrival chunk: 32 (stride 1) or 16 (stride 2)
    int buffers = 1;         // 2: stages alternate between two LDS buffers
    int n_stages = 0, n_rowblocks = 0;
    int n_chunks = 0;        // chunk barriers in all
    int final_waits = 0;     // chunk barriers no row block waits for
    int m_blocks = 0;        // ceil(M / 32)
    int mb_per_wg = 0;       // 32-wide blocks of M per workgroup (2 or 4)
    int m_blocks_pad = 0;    // m_blocks rounded up to a multiple of mb_per_wg
    int record_slots = 0;    // row-block records stored: n_rowblocks plus the all-zero ones the kernels read ahead into
    std::vector<int32_t> stage_tab;  // per non-empty stage: c_begin, c_count
    // (n_rowblocks + 2) x 64 lanes x 4 dwords, then (n_rowblocks + 2) x 64 lanes x 2 dwords (two row blocks of
    // zeros at the end: the records are read two row blocks ahead)
    std::vector<uint32_t> records;
    std::vector<uint16_t> pwfrag;    // per row block (+1 of zeros), K-step, 32-wide block of M, lane: 8 weights
    std::vector<float> bias_pad;     // [m_blocks_pad * 32]: the bias, zero beyond M (all zero without a bias)
    std::vector<uint32_t> group_chan;  // deep schedules: per group of four row blocks, first input channel its windows
                                       // reach | (last + 1) << 16
    // device copies
    int32_t *d_stage_tab = nullptr;
    uint32_t *d_records = nullptr;
    uint16_t *d_pwfrag = nullptr;
    float *d_bias_pad = nullptr;
    uint32_t *d_group_chan = nullptr;
};

// Builds the host tables from the (already rounded) factors.  dw [G][9], pw [M][G], bias [M] or nullptr.
// allow_tap2: the builder may choose the two-tap depthwise stage (kernel instances exist for NHWC).
// deep_stage (0, 256 or 512): the schedule of the deep-layer kernel (kernels_fused_deep.hip) -- all input channels
// are one stage of that many channels, the row blocks are padded with empty ones to a multiple of four and the
// output channels to a multiple of 256.
void build_fused_schedule(FusedSchedule &s, int dtype, int stride, int C, int M, const int32_t *g,
                          const int32_t *offsets, const float *dw, const float *pw, const float *bias,
                          bool gdw_only = false, int deep_stage = 0, bool allow_tap2 = false);

struct FusedArgs {
    const void *x;
    void *y;
    Epilogue ep;
    const FusedSchedule *sched;
    int dtype, layout, stride;
    int pool = 0;               // 1: y = 2 x 2 / stride-2 max-pool of the layer's output, [N][Ho/2][Wo/2][M] (NHWC only)
    int N, C, H, W, M, Ho, Wo;  // depthwise-only schedule: y is T and M its channel stride (G rounded up to 16)
};

// True if a fused kernel instance exists for this kind of layer.
bool fused_shape_supported(int dtype, int layout, int K, int stride, int pad, int C, int M);
// True if, additionally, the tile chosen for this image size fits the LDS (with the fp32 output tile of the
// residual case if `residual`) and x (x_elems elements) is within the loader's addressing range.
bool fused_image_supported(const FusedSchedule &s, int layout, int stride, int C, int Ho, int Wo, bool residual,
                           int64_t x_elems);
int launch_fused(const FusedArgs &a, hipStream_t s);

// The deep-layer kernel: few pixels, many channels (see kernels_fused_deep.hip).  a.sched is a deep schedule.
bool deep_shape_supported(int dtype, int layout, int K, int stride, int pad, int C, int M);
int64_t deep_workgroups(const FusedSchedule &sc, int N, int C, int H, int W, int M, int Ho, int Wo, bool pool);
// Bytes of workspace with which a launch this small is split over runs of row blocks (0: it is not split).
size_t deep_split_workspace_bytes(const FusedSchedule &sc, int N, int C, int H, int W, int M, int Ho, int Wo, bool pool);
int launch_fused_deep(const FusedArgs &a, void *workspace, size_t workspace_bytes, hipStream_t s);

}  // namespace gdws
