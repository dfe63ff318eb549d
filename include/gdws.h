/*
 * libgdws -- forward pass of Generalized Depthwise-Separable (GDWS) convolutions on gfx950.
 *
 * Notation follows the paper (Section 3): a (C,K,M) standard convolution has a
 * weight tensor W [M][C][K][K]; a (C,K,g,M) GDWS convolution is a (C,K,g)
 * generalized depthwise (GDW) stage, in which input channel c is convolved
 * with g[c] K x K filters giving G = sum(g) intermediate channels, followed by a
 * (G,1,M) pointwise (PW) stage.  Intermediate channel j = h[c] + i is the i-th
 * filter of channel c, h = exclusive prefix sum of g (Property 2).
 *
 * Conventions for every entry point
 *   - returns GDWS_OK (0) or a negative gdws_status_t; never throws or aborts;
 *     output handles are written only on success.
 *   - "host" pointers are ordinary CPU memory, read during the call only.
 *     "dev" pointers are HIP device memory owned by the caller; the library
 *     neither allocates nor frees caller tensors.  A plan / network owns the
 *     device copies of its packed weights and tables until it is destroyed.
 *   - forward calls are asynchronous on the given HIP stream (a hipStream_t
 *     passed as void*, NULL = the default stream), allocate nothing and never
 *     synchronise with the host.  A plan is immutable after creation and may be
 *     used from several streams at once.
 *   - activations are N x C x H x W (GDWS_NCHW) or N x H x W x C (GDWS_NHWC),
 *     dense, in the plan's dtype.  The sliding window is a cross-correlation
 *     with zero padding; stride and pad apply to the K x K stage, the pointwise
 *     stage is 1 x 1, stride 1.  Output size H' = (H + 2 pad - K) / stride + 1.
 *   - arithmetic: products and sums are accumulated in fp32 whatever the storage
 *     dtype; in the 16-bit dtypes the G-channel intermediate is rounded to the
 *     storage dtype (nearest even) before the pointwise stage.
 */
#ifndef GDWS_H
#define GDWS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    GDWS_OK = 0,
    GDWS_EINVAL = -1,       /* a size, flag or g entry is out of range */
    GDWS_ENULL = -2,        /* a required pointer is NULL */
    GDWS_EUNSUPPORTED = -3, /* valid request this build has no kernel for */
    GDWS_EWORKSPACE = -4,   /* workspace missing or too small */
    GDWS_EHIP = -5,         /* the HIP runtime reported an error */
    GDWS_ENOMEM = -6        /* a host allocation failed */
} gdws_status_t;

typedef enum { GDWS_F32 = 0, GDWS_F16 = 1, GDWS_BF16 = 2 } gdws_dtype_t;
typedef enum { GDWS_NCHW = 0, GDWS_NHWC = 1 } gdws_layout_t;
typedef enum { GDWS_MODE_AUTO = 0, GDWS_MODE_FUSED = 1, GDWS_MODE_UNFUSED = 2 } gdws_mode_t;

/* One convolution layer.  relu / has_bias / has_residual select the epilogue
 * y = act(conv(x) + bias + residual) that the network workloads need (the paper's
 * convolution itself has none of them). */
typedef struct {
    int32_t C, M, K, stride, pad;
    int32_t dtype;  /* gdws_dtype_t  */
    int32_t layout; /* gdws_layout_t */
    int32_t relu, has_bias, has_residual;
} gdws_layer_desc_t;

typedef struct gdws_plan_s gdws_plan_t;
typedef struct gdws_net_s gdws_net_t;
typedef struct gdws_graph_s gdws_graph_t;

const char *gdws_strerror(int code);

/* ---- construction (host side; Section 3.3) -------------------------------- */

/* Singular values of the C sub-matrices W_c (M x K^2 slices of W, Section 3
 * "2D Convolution as Matrix Multiplication"), descending, R = min(M, K^2) per
 * channel.  W host [M][C][K][K]; sigma host [C][R] out; rank host [C] out (may be
 * NULL) = number of sigma above max(M,K^2) * eps * sigma_1. */
int gdws_singular_values(const float *W, int32_t M, int32_t C, int32_t K, double *sigma, int32_t *rank);

/* The same singular values computed on the device, for a weight that already
 * lives there (the ranking step of Algorithms 1 and 2 over all layers of a
 * network without a round trip to the host).  One wave per channel forms the
 * K^2 x K^2 Gram matrix W_c^T W_c in fp64 and diagonalises it with cyclic
 * Jacobi rotations.  w_dev device fp32 [M][C][K][K]; sigma_dev device fp64
 * [C][R] out, R = min(M, K^2), descending; rank_dev device int32 [C] out or NULL
 * = number of sigma_i^2 above 64 * max(M,K^2) * eps * sigma_1^2 (the Gram matrix
 * resolves singular values down to about sqrt(eps) sigma_1 only, so the
 * threshold is coarser than the host routine's); v_dev device fp64
 * [C][R][K^2] out or NULL = right singular vectors v_i (Lemma 3's depthwise
 * filters), each with its largest-magnitude entry (first on ties) positive.
 * Asynchronous on `stream`; allocates nothing.  GDWS_EUNSUPPORTED for K > 7,
 * GDWS_EINVAL for sizes below 1, GDWS_ENULL for a missing w_dev or sigma_dev. */
int gdws_singular_values_device(const float *w_dev, int32_t M, int32_t C, int32_t K, double *sigma_dev,
                                int32_t *rank_dev, double *v_dev, void *stream);

/* Algorithm 1 (MEGO): greedy channel distribution vector minimising the weighted
 * error of eq. 4 subject to sum(g) <= gamma.  sigma host [C][R] and rank host [C]
 * as returned above; alpha host [C] or NULL (all ones); g host [C] in/out: on entry
 * the starting vector (zeros for the paper's algorithm), on exit the result.
 * cap <= 0 means no cap besides the rank; ties go to the lowest channel index. */
int gdws_mego(const double *sigma, const int32_t *rank, int32_t C, int32_t R, const double *alpha,
              int64_t gamma, int32_t cap, int32_t *g);

/* Algorithm 2 (LEGO): least-complex g with weighted error <= beta.  Filters are
 * dropped, smallest alpha*sigma^2 first, while the bound holds.  compare selects
 * the reading of the bound: GDWS_LEGO_THEOREM follows Theorem 2 and its proof (the
 * sum of dropped squared terms stays <= beta^2); GDWS_LEGO_LISTING takes the
 * algorithm box literally (the running sum is compared with beta itself, strictly)
 * -- the paper's two statements differ and no printed value decides between them.
 * g host [C] out; no channel goes below g_min. */
typedef enum { GDWS_LEGO_THEOREM = 0, GDWS_LEGO_LISTING = 1 } gdws_lego_compare_t;
int gdws_lego(const double *sigma, const int32_t *rank, int32_t C, int32_t R, const double *alpha,
              double beta, int32_t g_min, int32_t compare, int32_t *g);

/* Total multiplier budget for a complexity target (eq. 3 against eq. 2): the
 * largest G with G (K^2 + M) <= rho * C K^2 M, kept within [C, min(K^2, M) * C].
 * This is the gamma handed to gdws_mego when every layer is cut to the same
 * fraction rho of its MACs (Section 4.4, the GDWS-U setting).  Negative
 * gdws_status_t on invalid arguments. */
int64_t gdws_budget_gamma(double rho, int32_t C, int32_t K, int32_t M);

/* Sparse-aware reduction (Appendix B): intermediate channels whose depthwise
 * filter is all zero, or whose pointwise column is all zero, contribute nothing
 * and are removed.  For a pruned W this turns any g >= rank into g_c = rank(W_c).
 * g host [C], dw host [G][K][K], pw host [M][G] in; g_out host [C]; dw_out
 * [G'][K][K], pw_out [M][G'], keep [G'] (index in the original of each kept
 * channel) may be NULL and need room for G entries.  Returns G' >= 0, or a
 * negative gdws_status_t. */
int gdws_compact_factors(int32_t C, int32_t M, int32_t K, const int32_t *g, const float *dw,
                         const float *pw, int32_t *g_out, float *dw_out, float *pw_out, int32_t *keep);

/* Build a layer plan.  g host [C], g[c] >= 0, sum(g) >= 1.  Exactly one of
 *   W  host [M][C][K][K]: the library factorises each W_c by truncated SVD of
 *      rank g[c] (Lemma 3); requires g[c] <= min(M, K^2);
 *   dw host [G][K][K] and pw host [M][G]: factors used as given (any g[c] >= 0).
 * bias host [M] (required iff desc->has_bias).  Weights are rounded once to
 * desc->dtype; bias stays fp32. */
int gdws_plan(const gdws_layer_desc_t *desc, const int32_t *g, const float *W, const float *dw,
              const float *pw, const float *bias, gdws_plan_t **out);
/* gdws_plan followed by the sparse-aware reduction of Appendix B on the rounded
 * factors: the plan's tables (gdws_plan_info) and factors (gdws_plan_factors) are
 * those of the reduced vector g' <= g, and the forward pass does G' (K^2 + M) MACs
 * per pixel.  GDWS_EINVAL if nothing is left. */
int gdws_plan_sparse(const gdws_layer_desc_t *desc, const int32_t *g, const float *W, const float *dw,
                     const float *pw, const float *bias, gdws_plan_t **out);
int gdws_plan_destroy(gdws_plan_t *plan);

/* Tables of a plan (Property 2).  Any output pointer may be NULL.  offsets
 * [C+1] and chan_of [G] point to host memory owned by the plan.
 * macs_per_pixel = G (K^2 + M), eq. 3 without the H'W' factor. */
int gdws_plan_info(const gdws_plan_t *plan, int32_t *G, const int32_t **offsets, const int32_t **chan_of,
                   int64_t *macs_per_pixel);

/* The factors the kernels use, after rounding to the plan's dtype, widened
 * back to fp32: dw_out host [G][K][K], pw_out host [M][G]. */
int gdws_plan_factors(const gdws_plan_t *plan, float *dw_out, float *pw_out);

/* ---- forward (Section 3.1 Definition) -------------------------------------- */

/* Bytes of device workspace gdws_forward uses for this shape and mode: the
 * G-channel intermediate for the unfused path (required).  For the fused path
 * 0, except for small launches of deep layers (a batch of one or two images,
 * more than 128 input channels): there the row blocks are split over
 * workgroups and the fp32 partial sums pass through this much workspace.  That
 * workspace is optional: without it (NULL, or fewer bytes) the same call runs
 * unsplit, slower, with the same results up to the order of the fp32 sums. */
size_t gdws_workspace_bytes(const gdws_plan_t *plan, int32_t N, int32_t H, int32_t W, int mode);

/* y = epilogue(PW(GDW(x))).  x dev [N,C,H,W] / [N,H,W,C]; y dev [N,M,H',W'] /
 * [N,H',W',M]; residual dev, same shape as y (required iff has_residual).
 * mode: GDWS_MODE_FUSED keeps the intermediate on chip (the matrix-core kernel
 * where it covers the shape -- 16-bit storage, K = 3, pad = 1 -- else a kernel on
 * the vector ALUs for any dtype / layout / K; GDWS_EUNSUPPORTED only if a tile's
 * input patch does not fit on chip, i.e. K or stride far beyond those of the
 * networks here), GDWS_MODE_UNFUSED runs the two stages through the workspace,
 * GDWS_MODE_AUTO picks the matrix-core fused kernel where it applies, else the
 * unfused path. */
int gdws_forward(const gdws_plan_t *plan, const void *x, const void *residual, void *y, int32_t N,
                 int32_t H, int32_t W, void *workspace, size_t workspace_bytes, int mode, void *stream);

/* gdws_forward followed by a 2 x 2, stride-2 max-pool without padding (the
 * pooling layers of the VGG-16 of Section 4), as one kernel: the pool runs in
 * the fused kernel's epilogue, so the unpooled activation never reaches HBM.
 * x dev [N,H,W,C]; y dev [N,H'/2,W'/2,M] (floor).  Only where the matrix-core
 * fused kernel applies (NHWC, 16-bit storage, K = 3, pad = 1, M % 8 == 0, no
 * residual): otherwise GDWS_EUNSUPPORTED and nothing is launched -- the caller
 * then runs gdws_forward and a pooling pass.  GDWS_EINVAL if H' or W' < 2, or if
 * x and y overlap in memory (tiles of y are stored while other tiles of x are
 * still being read). */
int gdws_forward_maxpool2(const gdws_plan_t *plan, const void *x, void *y, int32_t N, int32_t H,
                          int32_t W, void *stream);

/* Channels of the intermediate tensor t as the library stores it: G, or, for
 * NHWC with 16-bit storage, G rounded up to a multiple of 16 (the surplus
 * channels are written as zeros, so that every pixel's row is 16-byte aligned
 * for the matrix-core pointwise kernel).  0 if plan is NULL. */
int32_t gdws_intermediate_channels(const gdws_plan_t *plan);

/* For callers that cannot allocate device memory (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): gdws_forward in
 * GDWS_MODE_UNFUSED with the G-channel intermediate held in a device array that
 * is part of the library image (GDWS_STATIC_SCRATCH_BYTES per GPU, resident from
 * the library's load to the end of the process) instead of a caller's workspace.
 * Calls no allocating routine.  GDWS_EWORKSPACE if the intermediate, N x Gt x H'
 * x W' elements of the plan's dtype (Gt = gdws_intermediate_channels), does not
 * fit.  All calls on one GPU share that one array: calls that may overlap in time
 * on a GPU (different streams, different host threads) race and must be ordered
 * by the caller.  Results are those of gdws_forward(..., GDWS_MODE_UNFUSED), bit
 * for bit. */
#define GDWS_STATIC_SCRATCH_BYTES ((size_t)64 << 20)
int gdws_forward_static(const gdws_plan_t *plan, const void *x, const void *residual, void *y, int32_t N,
                        int32_t H, int32_t W, void *stream);

/* The two stages on their own (Section 3.1 Definition: GDW, then PW).  Same
 * layouts; t dev [N,Gt,H',W'] / [N,H',W',Gt] in the plan's dtype with
 * Gt = gdws_intermediate_channels(plan).  gdws_pw_forward applies the plan's
 * epilogue. */
int gdws_gdw_forward(const gdws_plan_t *plan, const void *x, void *t, int32_t N, int32_t H, int32_t W,
                     void *stream);
int gdws_pw_forward(const gdws_plan_t *plan, const void *t, const void *residual, void *y, int32_t N,
                    int32_t Ho, int32_t Wo, void *stream);

/* ---- backward pass (fine-tuning a GDWS network, Section 4) ------------------- */

/* Gradients through the layer's linear part Y = PW(GDW(X)) + bias (the two
 * operators of Section 3.1 Definition; the paper fine-tunes GDWS networks in
 * its ablation but prints no formulas: these are the operators' adjoints).
 * dy = dL/dY at the layer's linear output: a ReLU or residual add that the
 * plan's epilogue applies in the forward pass is the caller's to undo (mask
 * dy with y > 0 first); the desc's relu / has_residual flags are ignored here.
 *   dx     dev, like x (the plan's dtype and layout), out, or NULL
 *   d_dw   dev fp32 [G][K][K] out, or NULL:  dL/dD
 *   d_pw   dev fp32 [M][G]    out, or NULL:  dL/dW_P
 *   d_bias dev fp32 [M]       out, or NULL
 * x dev [N,C,H,W] / [N,H,W,C], dy dev [N,M,H',W'] / [N,H',W',M] in the plan's
 * dtype.  The factors are the plan's (as rounded to its dtype); accumulation is
 * fp32; results are deterministic (no atomics).  workspace: device memory of
 * gdws_backward_workspace_bytes (the intermediate and its gradient in fp32,
 * and the per-slab partial sums of the reductions over pixels),
 * caller-owned; GDWS_EWORKSPACE if missing or too small.  Asynchronous on
 * `stream`, allocates nothing.  General kernels on the vector ALUs for every
 * dtype / layout / K / stride / pad: not tuned. */
size_t gdws_backward_workspace_bytes(const gdws_plan_t *plan, int32_t N, int32_t H, int32_t W);
int gdws_backward(const gdws_plan_t *plan, const void *x, const void *dy, void *dx, float *d_dw, float *d_pw,
                  float *d_bias, int32_t N, int32_t H, int32_t W, void *workspace, size_t workspace_bytes,
                  void *stream);

/* ---- reference point: the standard convolution (eq. 1) ---------------------- */

/* Bytes of device workspace conv_dense_forward needs: room for a copy of w
 * repacked in matrix-core operand order where the implicit-GEMM kernel applies
 * (16-bit storage, NHWC, K = 3, stride 1, pad 1, C a multiple of 16), else 0. */
size_t conv_dense_workspace_bytes(const gdws_layer_desc_t *desc);

/* y = epilogue(W * x).  w dev [M][C][K][K] in desc->dtype, bias dev fp32 [M]
 * (iff has_bias), residual dev shaped like y (iff has_residual).  Where the
 * implicit-GEMM kernel applies the call first repacks w into the workspace
 * (GDWS_EWORKSPACE if it is missing or smaller than conv_dense_workspace_bytes);
 * every other configuration runs on a direct kernel and needs no workspace. */
int conv_dense_forward(const gdws_layer_desc_t *desc, const void *w, const float *bias, const void *x,
                       const void *residual, void *y, int32_t N, int32_t H, int32_t W, void *workspace,
                       size_t workspace_bytes, void *stream);

/* ---- whole networks ---------------------------------------------------------- */

typedef enum { GDWS_LAYER_GDWS = 0, GDWS_LAYER_DENSE = 1, GDWS_LAYER_MAXPOOL = 2 } gdws_layer_kind_t;

/* One node of a feed-forward graph.  src / residual index earlier nodes
 * (-1 = the network input; residual = -2 for none).
 *   GDWS:    plan (borrowed; must outlive the network); its desc supplies the epilogue.
 *   DENSE:   desc, w host fp32 [M][C][K][K], bias host fp32 [M] or NULL.
 *   MAXPOOL: desc.C channels, window desc.K, desc.stride, desc.pad (padding never wins). */
typedef struct {
    int32_t kind; /* gdws_layer_kind_t */
    int32_t src, residual;
    const gdws_plan_t *plan;
    gdws_layer_desc_t desc;
    const float *w;
    const float *bias;
} gdws_net_layer_t;

/* All layers must share one dtype and layout. */
int gdws_net_create(const gdws_net_layer_t *layers, int32_t n_layers, gdws_net_t **out);
int gdws_net_destroy(gdws_net_t *net);

/* Bytes of device workspace for a batch of N inputs of H x W (activation buffers
 * of every node whose output is still needed, plus per-layer scratch).  The
 * buffer assignment for (N, H, W) is worked out here, once, and kept in the
 * network object (host memory); gdws_network_forward reuses it. */
size_t gdws_net_workspace_bytes(const gdws_net_t *net, int32_t N, int32_t H, int32_t W);

/* Runs every node in order on `stream`; y receives the last node's output. */
int gdws_network_forward(const gdws_net_t *net, const void *x, void *y, int32_t N, int32_t H, int32_t W,
                         void *workspace, size_t workspace_bytes, void *stream);

/* ---- launch graphs (Appendix A, the frames-per-second protocol) ------------------ */

/* The paper measures whole-network inference at batch 1 (5000 warm-up and 10000
 * timed forwards between device events).  At that size a forward is a chain of
 * some twenty short kernels and the host's launch calls dominate, so the chain
 * is recorded once and replayed as one launch.
 *
 * gdws_capture_begin puts `stream` (not the default stream) into capture mode:
 * forward calls of this library issued on it from the calling thread are then
 * recorded instead of run.  gdws_capture_end ends the capture and returns the
 * instantiated graph.  Every forward call to be recorded must have run once,
 * eagerly, with the same arguments before (the first launch of a kernel sets a
 * function attribute, which is not a stream operation).  The graph holds the
 * device pointers passed to the recorded calls: the buffers must stay allocated,
 * and a replay reads and writes them where they are.  No memset node is ever
 * recorded: no forward call of this library clears memory through the runtime. */
int gdws_capture_begin(void *stream);
int gdws_capture_end(void *stream, gdws_graph_t **out);
/* Replays the recorded launches on `stream`, in their recorded order. */
int gdws_graph_launch(const gdws_graph_t *graph, void *stream);
int gdws_graph_destroy(gdws_graph_t *graph);

#ifdef __cplusplus
}
#endif
#endif /* GDWS_H */
