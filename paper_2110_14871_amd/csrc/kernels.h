// Launchers of the HIP kernels behind the C ABI.  Every launcher validates nothing: the
// entry points in api.hip check shapes and pointers before calling.
#pragma once
#include <vector>

#include "common.h"

namespace gdws {

struct GdwArgs {
    const void *x;           // activations in `dtype`, `layout`
    void *t;                 // [N,G,Ho,Wo] / [N,Ho,Wo,G] in `dtype`
    const float *dw;         // [G][K*K] fp32 (values already rounded to dtype)
    const int32_t *chan_of;  // [G]
    int dtype, layout;
    int N, C, H, W, G, K, stride, pad, Ho, Wo;
    int Gt;  // channels of T as stored: G, or G padded with zero channels (NHWC, 16-bit)
};

struct PwArgs {
    const void *t;    // [N,G,Ho,Wo] / [N,Ho,Wo,G]
    void *y;          // [N,M,Ho,Wo] / [N,Ho,Wo,M]
    const float *pw;  // [M][G] fp32 (values already rounded to dtype)
    Epilogue ep;
    int dtype, layout;
    int N, G, M, Ho, Wo;
    int Gt;  // channels of T as stored
};

struct DenseArgs {
    const void *x;
    void *y;
    const void *w;  // [M][C][K][K] in `dtype`
    Epilogue ep;
    int dtype, layout;
    int N, C, H, W, M, K, stride, pad, Ho, Wo;
};

struct PoolArgs {
    const void *x;
    void *y;
    int dtype, layout;
    int N, C, H, W, K, stride, pad, Ho, Wo;
};

// Pointwise stage on the matrix cores (16-bit, NHWC; T stored with a channel stride that is a multiple of 16).
struct PwMfmaTables {
    bool valid = false;
    int Gp = 0, ksteps = 0, mb_per_wg = 0, m_blocks_pad = 0;
    std::vector<uint16_t> frag;   // [ksteps][m_blocks_pad][64 lanes][8]: weights in A-operand order
    std::vector<float> bias_pad;  // [m_blocks_pad * 32]
    uint16_t *d_frag = nullptr;
    float *d_bias_pad = nullptr;
};
struct PwMfmaArgs {
    const void *t;
    void *y;
    Epilogue ep;          // the bias is taken from the tables
    const PwMfmaTables *tables;
    int dtype, M;
    int64_t P;            // output pixels: N * Ho * Wo
    // stride 1 (default): T has P pixels.  stride > 1 (a strided 1 x 1 convolution): output pixel (n, oy, ox) reads
    // pixel (n, oy*stride, ox*stride) of an input with H x W pixels per image
    int stride = 1, Ho = 0, Wo = 0, H = 0, W = 0;
};
void build_pw_mfma_tables(PwMfmaTables &tb, int dtype, int G, int M, const float *pw, const float *bias);
int launch_pw_mfma(const PwMfmaArgs &a, hipStream_t s);
// fp32 pointwise stage on v_mfma_f32_32x32x2_f32, NCHW or NHWC (the arguments of the direct kernel).
int launch_pw_mfma_f32(const PwArgs &a, hipStream_t s);

// Generalized depthwise stage with the input tile and halo staged in LDS (16-bit, NHWC, K = 3, pad = 1).
struct GdwLdsTables {
    bool valid = false;
    int n_chunks = 0, out_stride = 0;
    std::vector<int32_t> chunks;  // per 64-channel chunk: c0, c_count, j0, j_count
    int32_t *d_chunks = nullptr;
};
struct GdwLdsArgs {
    const void *x;
    void *t;
    const float *dw;          // [G][9] fp32, device
    const int32_t *chan_of;   // [G], device
    const GdwLdsTables *tables;
    int dtype, stride;
    int N, C, H, W, G, Gp, Ho, Wo;
};
void build_gdw_lds_tables(GdwLdsTables &tb, int C, const int32_t *offsets);
bool gdw_lds_supported(const GdwLdsTables &tb, int dtype, int layout, int K, int stride, int pad, int C, int64_t x_elems);
int launch_gdw_lds(const GdwLdsArgs &a, hipStream_t s);

// Shape-agnostic direct kernels (one thread per output element).
int launch_gdw_direct(const GdwArgs &a, hipStream_t s);
int launch_pw_direct(const PwArgs &a, hipStream_t s);
int launch_dense_direct(const DenseArgs &a, hipStream_t s);
int launch_maxpool(const PoolArgs &a, hipStream_t s);

// Standard 3 x 3 convolution as an implicit GEMM on the matrix cores (16-bit NHWC, stride 1, pad 1, C a multiple of 16).
// The workspace receives the weights repacked in operand order (conv_mfma_workspace_bytes).
bool conv_mfma_supported(int dtype, int layout, int K, int stride, int pad, int C, int64_t x_elems);
size_t conv_mfma_workspace_bytes(int C, int M);
int launch_conv_mfma(const DenseArgs &a, void *workspace, hipStream_t s);

// Backward pass through the layer's linear part (kernels_backward.hip).  Gradient outputs that are nullptr are skipped.
struct BackwardArgs {
    const void *x, *dy;        // activations in the layer's storage type and layout
    void *dx;                  // like x, or nullptr
    float *g_dw, *g_pw, *g_bias;  // fp32 [G][K][K], [M][G], [M], or nullptr
    const float *dw, *pw;      // the plan's factors (fp32 copies of the rounded values)
    const int32_t *offsets, *chan_of;
    void *workspace;           // backward_workspace_bytes
    int dtype, layout;
    int N, C, H, W, M, G, K, stride, pad, Ho, Wo;
};
size_t backward_workspace_bytes(int N, int M, int G, int K, int Ho, int Wo);
int launch_backward(const BackwardArgs &a, hipStream_t s);

// Singular values (descending), numerical rank and, optionally, right singular vectors of the C slices W_c (M x K^2)
// of a weight [M][C][K][K] in device memory: one wave per slice, Jacobi on the Gram matrix in fp64.  K <= 7.
int launch_svd_device(const float *w, int M, int C, int K, double *sigma, int32_t *rank, double *v, hipStream_t s);

// Fused GDWS forward on the vector ALUs for the shapes the matrix-core kernel does not take (any dtype / layout / K).
struct FusedGenericArgs {
    const void *x;
    void *y;
    const float *dw;           // [G][K*K], values representable in `dtype`
    const float *pw;           // [M][G]
    const int32_t *offsets;    // [C + 1]
    const int32_t *chan_of;    // [G]
    Epilogue ep;
    int dtype, layout;
    int N, C, H, W, M, G, K, stride, pad, Ho, Wo;
};
bool fused_generic_supported(int K, int stride);
int launch_fused_generic(const FusedGenericArgs &a, hipStream_t s);

// Standard convolution with 3 input channels on the matrix cores (16-bit NHWC; 7 x 7 stride 2 or 3 x 3 stride 1).
struct DenseMfmaTables {
    bool valid = false;
    int ksteps = 0, m_blocks_pad = 0;
    std::vector<uint16_t> frag;   // [ksteps][m_blocks_pad][64 lanes][8]: weights in A-operand order
    std::vector<float> bias_pad;  // [m_blocks_pad * 32]
    uint16_t *d_frag = nullptr;
    float *d_bias_pad = nullptr;
};
struct DenseMfmaArgs {
    const void *x;
    void *y;
    const DenseMfmaTables *tables;  // the bias is taken from the tables
    int dtype, relu;
    int N, C, H, W, M, K, stride, pad, Ho, Wo;
};
bool dense_mfma_supported(int dtype, int layout, int K, int C, int stride, bool residual);
// True if x (x_elems elements) is within the kernel's addressing range (and not smaller than one 16-byte load).
bool dense_mfma_image_supported(int64_t x_elems);
// w: [M][C][K][K], already rounded to the storage type; bias [M] or nullptr
void build_dense_mfma_tables(DenseMfmaTables &tb, int dtype, int K, int C, int M, const float *w, const float *bias);
int launch_dense_mfma(const DenseMfmaArgs &a, hipStream_t s);

}  // namespace gdws
