// C ABI of libgdws: argument validation, plan / network objects, kernel dispatch.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <memory>
#include <mutex>
#include <new>
#include <vector>

#include "fused.h"
#include "kernels.h"
#include "planner.h"

using namespace gdws;

// No exception crosses the C boundary: host allocation failures inside an entry point become a status.
#define GDWS_TRY try {
#define GDWS_CATCH                                   \
    }                                                \
    catch (const std::bad_alloc &) { return GDWS_ENOMEM; } \
    catch (...) { return GDWS_EHIP; }

// ---------------------------------------------------------------------------------
// objects
// ---------------------------------------------------------------------------------

struct gdws_plan_s {
    gdws_layer_desc_t desc{};
    int G = 0;
    std::vector<int32_t> g, offsets, chan_of;  // host tables (Property 2)
    std::vector<float> dw, pw, bias;           // host factors after rounding to desc.dtype
    // device copies
    int32_t *d_chan_of = nullptr;
    int32_t *d_offsets = nullptr;
    float *d_dw = nullptr;    // [G][K*K] fp32
    float *d_pw = nullptr;    // [M][G]   fp32
    float *d_bias = nullptr;  // [M]
    FusedSchedule fused;      // tables of the fused kernel (valid only for the shapes it covers)
    FusedSchedule gdwm;       // tables of its depthwise-only mode (16-bit NHWC, single-stage layers)
    FusedSchedule deep;       // tables of the deep-layer fused kernel (16-bit NHWC, 128 < C <= 512, M >= 256)
    PwMfmaTables pwm;         // tables of the MFMA pointwise kernel (16-bit NHWC)
    DenseMfmaTables gdm;      // depthwise stage of a 3-channel layer as an implicit GEMM (16-bit NHWC)
    GdwLdsTables gdl;         // tables of the LDS-tiled depthwise kernel (16-bit NHWC, K = 3)
    int Gt = 0;               // channels of the intermediate as stored (G, or G rounded up to 16: NHWC 16-bit)
    ~gdws_plan_s()
    {
        (void)hipFree(d_chan_of); (void)hipFree(d_offsets); (void)hipFree(d_dw); (void)hipFree(d_pw);
        (void)hipFree(d_bias);
        (void)hipFree(fused.d_stage_tab); (void)hipFree(fused.d_records);
        (void)hipFree(fused.d_pwfrag); (void)hipFree(fused.d_bias_pad);
        (void)hipFree(gdwm.d_stage_tab); (void)hipFree(gdwm.d_records); (void)hipFree(gdwm.d_bias_pad);
        (void)hipFree(deep.d_stage_tab); (void)hipFree(deep.d_records); (void)hipFree(deep.d_pwfrag);
        (void)hipFree(deep.d_bias_pad); (void)hipFree(deep.d_group_chan);
        (void)hipFree(pwm.d_frag); (void)hipFree(pwm.d_bias_pad); (void)hipFree(gdl.d_chunks);
        (void)hipFree(gdm.d_frag); (void)hipFree(gdm.d_bias_pad);
    }
};

namespace {

struct NetNode {
    gdws_net_layer_t l{};
    void *d_w = nullptr;     // dense: [M][C][K][K] in dtype
    float *d_bias = nullptr; // dense: [M]
    PwMfmaTables pwm;        // dense 1 x 1, 16-bit NHWC, C a multiple of 16: the matrix-core pointwise kernel
    DenseMfmaTables dm;      // dense with 3 input channels, 16-bit NHWC: the implicit-GEMM kernel
};

struct NodeShape {
    int C, H, W;      // output channels / size
    size_t bytes;     // of the output tensor
    size_t scratch;   // per-layer scratch
    size_t offset;    // of the output buffer inside the workspace (SIZE_MAX = writes to y)
};

// Buffer assignment of a network for one input size.
struct NetLayout {
    int N = 0, H = 0, W = 0;
    std::vector<NodeShape> sh;
    size_t act_top = 0;  // end of the activation buffers = start of the per-layer scratch
    size_t total = 0;
};

}  // namespace

struct gdws_net_s {
    std::vector<NetNode> nodes;
    int dtype = 0, layout = 0;
    // layouts worked out so far, one per input size seen (append-only, guarded by mu; entries are never moved)
    mutable std::mutex mu;
    mutable std::vector<std::unique_ptr<NetLayout>> layouts;
    ~gdws_net_s()
    {
        for (auto &n : nodes) {
            (void)hipFree(n.d_w); (void)hipFree(n.d_bias); (void)hipFree(n.pwm.d_frag); (void)hipFree(n.pwm.d_bias_pad);
            (void)hipFree(n.dm.d_frag); (void)hipFree(n.dm.d_bias_pad);
        }
    }
};

namespace {

float round_to_dtype(float v, int dtype)
{
    if (dtype == GDWS_BF16) return bf16_to_float(float_to_bf16(v));
    if (dtype == GDWS_F16) return (float)(_Float16)v;
    return v;
}

int check_desc(const gdws_layer_desc_t *d)
{
    if (!d) return GDWS_ENULL;
    if (d->C < 1 || d->M < 1 || d->K < 1 || d->stride < 1 || d->pad < 0) return GDWS_EINVAL;
    if (d->dtype < GDWS_F32 || d->dtype > GDWS_BF16) return GDWS_EINVAL;
    if (d->layout != GDWS_NCHW && d->layout != GDWS_NHWC) return GDWS_EINVAL;
    return GDWS_OK;
}

int check_image(const gdws_layer_desc_t &d, int N, int H, int W, int *Ho, int *Wo)
{
    if (N < 1 || H < 1 || W < 1) return GDWS_EINVAL;
    if (H + 2 * d.pad < d.K || W + 2 * d.pad < d.K) return GDWS_EINVAL;
    *Ho = out_size(H, d.K, d.stride, d.pad);
    *Wo = out_size(W, d.K, d.stride, d.pad);
    return GDWS_OK;
}

template <typename T>
int upload(T **dst, const std::vector<T> &src)
{
    if (src.empty()) { *dst = nullptr; return GDWS_OK; }
    GDWS_HIP_CHECK(hipMalloc((void **)dst, src.size() * sizeof(T)));
    GDWS_HIP_CHECK(hipMemcpy(*dst, src.data(), src.size() * sizeof(T), hipMemcpyHostToDevice));
    return GDWS_OK;
}

// Host fp32 -> device buffer in `dtype`.
int upload_as_dtype(void **dst, const float *src, size_t count, int dtype)
{
    if (dtype == GDWS_F32) {
        GDWS_HIP_CHECK(hipMalloc(dst, count * 4));
        GDWS_HIP_CHECK(hipMemcpy(*dst, src, count * 4, hipMemcpyHostToDevice));
        return GDWS_OK;
    }
    std::vector<uint16_t> tmp(count);
    for (size_t i = 0; i < count; ++i) {
        if (dtype == GDWS_BF16) tmp[i] = float_to_bf16(src[i]);
        else { _Float16 h = (_Float16)src[i]; std::memcpy(&tmp[i], &h, 2); }
    }
    GDWS_HIP_CHECK(hipMalloc(dst, count * 2));
    GDWS_HIP_CHECK(hipMemcpy(*dst, tmp.data(), count * 2, hipMemcpyHostToDevice));
    return GDWS_OK;
}

bool ranges_overlap(const void *a, size_t na, const void *b, size_t nb)
{
    const char *pa = (const char *)a, *pb = (const char *)b;
    return pa < pb + nb && pb < pa + na;
}

Epilogue plan_epilogue(const gdws_plan_t *p, const void *residual)
{
    Epilogue e;
    e.bias = p->desc.has_bias ? p->d_bias : nullptr;
    e.residual = p->desc.has_residual ? residual : nullptr;
    e.relu = p->desc.relu;
    return e;
}

int run_gdw(const gdws_plan_t *p, const void *x, void *t, int N, int H, int W, int Ho, int Wo, hipStream_t s)
{
    GdwArgs a;
    a.x = x; a.t = t; a.dw = p->d_dw; a.chan_of = p->d_chan_of;
    a.dtype = p->desc.dtype; a.layout = p->desc.layout;
    a.N = N; a.C = p->desc.C; a.H = H; a.W = W; a.G = p->G; a.K = p->desc.K;
    a.stride = p->desc.stride; a.pad = p->desc.pad; a.Ho = Ho; a.Wo = Wo; a.Gt = p->Gt;
    const gdws_layer_desc_t &d = p->desc;
    if (p->gdwm.valid && fused_image_supported(p->gdwm, d.layout, d.stride, d.C, Ho, Wo, false, (int64_t)N * d.C * H * W)) {
        FusedArgs f;
        f.x = x; f.y = t; f.ep = Epilogue{nullptr, nullptr, 0}; f.sched = &p->gdwm;
        f.dtype = d.dtype; f.layout = d.layout; f.stride = d.stride;
        f.N = N; f.C = d.C; f.H = H; f.W = W; f.M = p->Gt; f.Ho = Ho; f.Wo = Wo;
        const int rc = launch_fused(f, s);
        if (rc != GDWS_EUNSUPPORTED) return rc;
    }
    if (p->gdm.valid && dense_mfma_image_supported((int64_t)N * d.C * H * W)) {
        DenseMfmaArgs m;
        m.x = x; m.y = t; m.tables = &p->gdm; m.dtype = d.dtype; m.relu = 0;
        m.N = N; m.C = d.C; m.H = H; m.W = W; m.M = p->Gt; m.K = d.K; m.stride = d.stride; m.pad = d.pad;
        m.Ho = Ho; m.Wo = Wo;
        return launch_dense_mfma(m, s);
    }
    if (gdw_lds_supported(p->gdl, d.dtype, d.layout, d.K, d.stride, d.pad, d.C, (int64_t)N * d.C * H * W)) {
        GdwLdsArgs g;
        g.x = x; g.t = t; g.dw = p->d_dw; g.chan_of = p->d_chan_of; g.tables = &p->gdl;
        g.dtype = d.dtype; g.stride = d.stride;
        g.N = N; g.C = d.C; g.H = H; g.W = W; g.G = p->G; g.Gp = p->Gt; g.Ho = Ho; g.Wo = Wo;
        return launch_gdw_lds(g, s);
    }
    return launch_gdw_direct(a, s);
}

int run_pw(const gdws_plan_t *p, const void *t, const void *residual, void *y, int N, int Ho, int Wo, hipStream_t s)
{
    PwArgs a;
    a.t = t; a.y = y; a.pw = p->d_pw; a.ep = plan_epilogue(p, residual);
    a.dtype = p->desc.dtype; a.layout = p->desc.layout;
    a.N = N; a.G = p->G; a.M = p->desc.M; a.Ho = Ho; a.Wo = Wo; a.Gt = p->Gt;
    if (p->pwm.valid) {
        PwMfmaArgs m;
        m.t = t; m.y = y; m.ep = a.ep; m.tables = &p->pwm; m.dtype = p->desc.dtype; m.M = p->desc.M;
        m.P = (int64_t)N * Ho * Wo;
        return launch_pw_mfma(m, s);
    }
    if (p->desc.dtype == GDWS_F32) return launch_pw_mfma_f32(a, s);
    return launch_pw_direct(a, s);
}

size_t intermediate_bytes(const gdws_plan_t *p, int N, int Ho, int Wo)
{
    return (size_t)N * p->Gt * Ho * Wo * dtype_bytes(p->desc.dtype);
}

bool fused_supported(const gdws_plan_t *p, int N, int H, int W)
{
    const gdws_layer_desc_t &d = p->desc;
    return p->fused.valid && fused_image_supported(p->fused, d.layout, d.stride, d.C, out_size(H, d.K, d.stride, d.pad),
                                                   out_size(W, d.K, d.stride, d.pad), d.has_residual != 0,
                                                   (int64_t)N * d.C * H * W);
}

constexpr int64_t kDeepMinWorkgroups = 64;
// Output pixels of the batch above which the general kernel's tiles fill the chip and it is the faster one
// (measured on the network shapes: 512 channels: 4,096 and 6,272 pixels gain 10 to 30 %, 8,192 lose 2 %; 256
// channels: 16,384 pixels still gain).
inline int64_t deep_max_pixels(int C) { return C <= 256 ? 16384 : 6400; }

// Workspace with which the fused path splits a small launch of a deep layer (0: no such split for this call).
size_t fused_split_bytes(const gdws_plan_t *p, int N, int H, int W, int Ho, int Wo, bool pool)
{
    if (!p->deep.valid || (int64_t)N * Ho * Wo > deep_max_pixels(p->desc.C)) return 0;
    return deep_split_workspace_bytes(p->deep, N, p->desc.C, H, W, p->desc.M, Ho, Wo, pool);
}

int run_fused(const gdws_plan_t *p, const void *x, const void *residual, void *y, int N, int H, int W, int Ho, int Wo,
              hipStream_t s, int pool = 0, void *ws = nullptr, size_t ws_bytes = 0)
{
    FusedArgs a;
    a.pool = pool;
    a.x = x; a.y = y; a.ep = plan_epilogue(p, residual); a.sched = &p->fused;
    a.dtype = p->desc.dtype; a.layout = p->desc.layout; a.stride = p->desc.stride;
    a.N = N; a.C = p->desc.C; a.H = H; a.W = W; a.M = p->desc.M; a.Ho = Ho; a.Wo = Wo;
    // Few pixels and many channels: the kernel whose waves split the output channels of one 32-pixel block, when its
    // grid gives the chip enough workgroups -- or, for the smallest launches, when the caller's workspace lets it
    // split the row blocks over workgroups as well.
    const int64_t dwg = deep_workgroups(p->deep, N, a.C, H, W, a.M, Ho, Wo, pool != 0);
    if (dwg > 0 && (int64_t)N * Ho * Wo <= deep_max_pixels(a.C) && !(pool && a.ep.residual)) {
        const size_t split = fused_split_bytes(p, N, H, W, Ho, Wo, pool != 0);
        const bool can_split = split > 0 && ws && ws_bytes >= split;
        if (dwg >= kDeepMinWorkgroups || can_split) {
            FusedArgs d = a;
            d.sched = &p->deep;
            const int rc = launch_fused_deep(d, can_split ? ws : nullptr, can_split ? ws_bytes : 0, s);
            if (rc != GDWS_EUNSUPPORTED) return rc;
        }
    }
    return launch_fused(a, s);
}

// the fused path for the shapes the matrix-core kernel does not take
int run_fused_generic(const gdws_plan_t *p, const void *x, const void *residual, void *y, int N, int H, int W, int Ho,
                      int Wo, hipStream_t s)
{
    FusedGenericArgs a;
    a.x = x; a.y = y; a.dw = p->d_dw; a.pw = p->d_pw; a.offsets = p->d_offsets; a.chan_of = p->d_chan_of;
    a.ep = plan_epilogue(p, residual);
    a.dtype = p->desc.dtype; a.layout = p->desc.layout;
    a.N = N; a.C = p->desc.C; a.H = H; a.W = W; a.M = p->desc.M; a.G = p->G; a.K = p->desc.K;
    a.stride = p->desc.stride; a.pad = p->desc.pad; a.Ho = Ho; a.Wo = Wo;
    return launch_fused_generic(a, s);
}

}  // namespace

// ---------------------------------------------------------------------------------
// entry points
// ---------------------------------------------------------------------------------

extern "C" {

const char *gdws_strerror(int code)
{
    switch (code) {
        case GDWS_OK: return "ok";
        case GDWS_EINVAL: return "invalid argument";
        case GDWS_ENULL: return "required pointer is NULL";
        case GDWS_EUNSUPPORTED: return "unsupported configuration";
        case GDWS_EWORKSPACE: return "workspace missing or too small";
        case GDWS_EHIP: return "HIP runtime error";
        case GDWS_ENOMEM: return "host memory allocation failed";
        default: return "unknown status";
    }
}

int gdws_singular_values(const float *W, int32_t M, int32_t C, int32_t K, double *sigma, int32_t *rank)
{
    GDWS_TRY
    if (!W || !sigma) return GDWS_ENULL;
    if (M < 1 || C < 1 || K < 1) return GDWS_EINVAL;
    const int KK = K * K, R = std::min(M, KK);
    std::vector<double> Wc;
    SliceSvd svd;
    for (int c = 0; c < C; ++c) {
        slice_of(W, M, C, KK, c, Wc);
        svd.compute(Wc.data(), M, KK);
        for (int i = 0; i < R; ++i) sigma[(size_t)c * R + i] = svd.sigma[i];
        if (rank) rank[c] = svd.rank;
    }
    return GDWS_OK;
    GDWS_CATCH
}

int gdws_singular_values_device(const float *w_dev, int32_t M, int32_t C, int32_t K, double *sigma_dev,
                                int32_t *rank_dev, double *v_dev, void *stream)
{
    if (!w_dev || !sigma_dev) return GDWS_ENULL;
    if (M < 1 || C < 1 || K < 1) return GDWS_EINVAL;
    return launch_svd_device(w_dev, M, C, K, sigma_dev, rank_dev, v_dev, (hipStream_t)stream);
}

int gdws_mego(const double *sigma, const int32_t *rank, int32_t C, int32_t R, const double *alpha, int64_t gamma,
              int32_t cap, int32_t *g)
{
    if (!sigma || !rank || !g) return GDWS_ENULL;
    if (C < 1 || R < 1 || gamma < 0) return GDWS_EINVAL;
    for (int c = 0; c < C; ++c)
        if (g[c] < 0 || g[c] > R || (alpha && !(alpha[c] > 0))) return GDWS_EINVAL;
    mego(sigma, rank, C, R, alpha, gamma, cap, g);
    return GDWS_OK;
}

int gdws_lego(const double *sigma, const int32_t *rank, int32_t C, int32_t R, const double *alpha, double beta,
              int32_t g_min, int32_t compare, int32_t *g)
{
    if (!sigma || !rank || !g) return GDWS_ENULL;
    if (C < 1 || R < 1 || !(beta >= 0) || g_min < 0) return GDWS_EINVAL;
    if (compare != GDWS_LEGO_THEOREM && compare != GDWS_LEGO_LISTING) return GDWS_EINVAL;
    for (int c = 0; c < C; ++c)
        if (alpha && !(alpha[c] > 0)) return GDWS_EINVAL;
    lego(sigma, rank, C, R, alpha, beta, g_min, compare == GDWS_LEGO_LISTING, g);
    return GDWS_OK;
}

int64_t gdws_budget_gamma(double rho, int32_t C, int32_t K, int32_t M)
{
    if (!(rho >= 0) || C < 1 || K < 1 || M < 1) return GDWS_EINVAL;
    return budget_gamma(rho, C, K, M);
}

int gdws_compact_factors(int32_t C, int32_t M, int32_t K, const int32_t *g, const float *dw, const float *pw,
                         int32_t *g_out, float *dw_out, float *pw_out, int32_t *keep)
{
    GDWS_TRY
    if (!g || !dw || !pw || !g_out) return GDWS_ENULL;
    if (C < 1 || M < 1 || K < 1) return GDWS_EINVAL;
    for (int c = 0; c < C; ++c)
        if (g[c] < 0) return GDWS_EINVAL;
    std::vector<int32_t> go, kp;
    std::vector<float> d, p;
    compact_factors(C, M, K * K, g, dw, pw, go, d, p, kp);
    std::copy(go.begin(), go.end(), g_out);
    if (dw_out) std::copy(d.begin(), d.end(), dw_out);
    if (pw_out) std::copy(p.begin(), p.end(), pw_out);
    if (keep) std::copy(kp.begin(), kp.end(), keep);
    return (int)kp.size();
    GDWS_CATCH
}

}  // extern "C"

namespace {

int plan_impl(const gdws_layer_desc_t *desc, const int32_t *g, const float *W, const float *dw, const float *pw,
              const float *bias, bool compact, gdws_plan_t **out)
{
    GDWS_TRY
    if (!out || !g) return GDWS_ENULL;
    int rc = check_desc(desc);
    if (rc) return rc;
    const bool from_w = W != nullptr;
    if (from_w == (dw != nullptr || pw != nullptr)) return GDWS_EINVAL;  // exactly one source of weights
    if (!from_w && (!dw || !pw)) return GDWS_ENULL;
    if (desc->has_bias && !bias) return GDWS_ENULL;
    const int C = desc->C, M = desc->M, KK = desc->K * desc->K;
    int64_t G = 0;
    for (int c = 0; c < C; ++c) {
        if (g[c] < 0) return GDWS_EINVAL;
        if (from_w && g[c] > std::min(M, KK)) return GDWS_EINVAL;
        G += g[c];
    }
    if (G < 1 || G > (1 << 24)) return GDWS_EINVAL;

    std::unique_ptr<gdws_plan_t> holder(new gdws_plan_t);
    gdws_plan_t *p = holder.get();
    p->desc = *desc;
    p->G = (int)G;
    p->g.assign(g, g + C);
    build_tables(g, C, p->offsets, p->chan_of);
    if (from_w) {
        factorise(W, M, C, desc->K, g, p->offsets, p->dw, p->pw);
    } else {
        p->dw.assign(dw, dw + (size_t)G * KK);
        p->pw.assign(pw, pw + (size_t)M * G);
    }
    for (auto &v : p->dw) v = round_to_dtype(v, desc->dtype);
    for (auto &v : p->pw) v = round_to_dtype(v, desc->dtype);
    if (compact) {
        // Appendix B: filters past a pruned slice's rank (and any other zero filter or zero column) are dropped;
        // the tables are those of the reduced vector g
        std::vector<int32_t> gk, keep;
        std::vector<float> dk, pk;
        compact_factors(C, M, KK, g, p->dw.data(), p->pw.data(), gk, dk, pk, keep);
        if (keep.empty()) return GDWS_EINVAL;  // the layer's output would be its bias
        p->g = gk; p->dw = dk; p->pw = pk;
        G = (int64_t)keep.size();
        p->G = (int)G;
        build_tables(p->g.data(), C, p->offsets, p->chan_of);
        g = p->g.data();
    }
    if (desc->has_bias) p->bias.assign(bias, bias + M);

    rc = upload(&p->d_chan_of, p->chan_of);
    if (!rc) rc = upload(&p->d_offsets, p->offsets);
    if (!rc) rc = upload(&p->d_dw, p->dw);
    if (!rc) rc = upload(&p->d_pw, p->pw);
    if (!rc) rc = upload(&p->d_bias, p->bias);
    if (!rc && fused_shape_supported(desc->dtype, desc->layout, desc->K, desc->stride, desc->pad, C, M)) {
        build_fused_schedule(p->fused, desc->dtype, desc->stride, C, M, g, p->offsets.data(), p->dw.data(),
                             p->pw.data(), desc->has_bias ? p->bias.data() : nullptr, false, 0,
                             desc->layout == GDWS_NHWC);
        rc = upload(&p->fused.d_stage_tab, p->fused.stage_tab);
        if (!rc) rc = upload(&p->fused.d_records, p->fused.records);
        if (!rc) rc = upload(&p->fused.d_pwfrag, p->fused.pwfrag);
        if (!rc) rc = upload(&p->fused.d_bias_pad, p->fused.bias_pad);
    }
    if (!rc && deep_shape_supported(desc->dtype, desc->layout, desc->K, desc->stride, desc->pad, C, M)) {
        build_fused_schedule(p->deep, desc->dtype, desc->stride, C, M, g, p->offsets.data(), p->dw.data(),
                             p->pw.data(), desc->has_bias ? p->bias.data() : nullptr, false, C <= 256 ? 256 : 512);
        if (p->deep.valid) {
            rc = upload(&p->deep.d_records, p->deep.records);
            if (!rc) rc = upload(&p->deep.d_pwfrag, p->deep.pwfrag);
            if (!rc) rc = upload(&p->deep.d_bias_pad, p->deep.bias_pad);
            if (!rc) rc = upload(&p->deep.d_group_chan, p->deep.group_chan);
        }
    }
    p->Gt = G;
    if (!rc && desc->layout == GDWS_NHWC && desc->dtype != GDWS_F32) {
        // unfused path: T is stored with a channel stride that is a multiple of 16 (zero channels at the end)
        p->Gt = (G + 15) & ~15;
        build_pw_mfma_tables(p->pwm, desc->dtype, G, M, p->pw.data(), desc->has_bias ? p->bias.data() : nullptr);
        rc = upload(&p->pwm.d_frag, p->pwm.frag);
        if (!rc) rc = upload(&p->pwm.d_bias_pad, p->pwm.bias_pad);
        build_gdw_lds_tables(p->gdl, C, p->offsets.data());
        if (!rc) rc = upload(&p->gdl.d_chunks, p->gdl.chunks);
        if (!rc && dense_mfma_supported(desc->dtype, desc->layout, desc->K, C, desc->stride, false)) {
            // 3 input channels: the depthwise stage is a standard convolution from 3 to Gt channels whose filter for
            // intermediate channel j is D[j] on input channel chan_of[j] and zero on the others (Gt - G zero filters
            // at the end write the padding channels of T)
            std::vector<float> wd((size_t)p->Gt * C * KK, 0.f);
            for (int64_t j = 0; j < G; ++j)
                std::copy(p->dw.begin() + j * KK, p->dw.begin() + (j + 1) * KK, wd.begin() + (j * C + p->chan_of[j]) * KK);
            build_dense_mfma_tables(p->gdm, desc->dtype, desc->K, C, p->Gt, wd.data(), nullptr);
            rc = upload(&p->gdm.d_frag, p->gdm.frag);
            if (!rc) rc = upload(&p->gdm.d_bias_pad, p->gdm.bias_pad);
        }
        if (!rc && fused_shape_supported(desc->dtype, desc->layout, desc->K, desc->stride, desc->pad, C, M)) {
            build_fused_schedule(p->gdwm, desc->dtype, desc->stride, C, M, g, p->offsets.data(), p->dw.data(),
                                 p->pw.data(), nullptr, true);
            if (p->gdwm.valid) {
                rc = upload(&p->gdwm.d_stage_tab, p->gdwm.stage_tab);
                if (!rc) rc = upload(&p->gdwm.d_records, p->gdwm.records);
                if (!rc) rc = upload(&p->gdwm.d_bias_pad, p->gdwm.bias_pad);
            }
        }
    }
    if (rc) return rc;
    *out = holder.release();
    return GDWS_OK;
    GDWS_CATCH
}

}  // namespace

extern "C" {

int gdws_plan(const gdws_layer_desc_t *desc, const int32_t *g, const float *W, const float *dw, const float *pw,
              const float *bias, gdws_plan_t **out)
{
    return plan_impl(desc, g, W, dw, pw, bias, false, out);
}

int gdws_plan_sparse(const gdws_layer_desc_t *desc, const int32_t *g, const float *W, const float *dw, const float *pw,
                     const float *bias, gdws_plan_t **out)
{
    return plan_impl(desc, g, W, dw, pw, bias, true, out);
}

int gdws_plan_destroy(gdws_plan_t *plan)
{
    delete plan;
    return GDWS_OK;
}

int gdws_plan_info(const gdws_plan_t *plan, int32_t *G, const int32_t **offsets, const int32_t **chan_of,
                   int64_t *macs_per_pixel)
{
    if (!plan) return GDWS_ENULL;
    if (G) *G = plan->G;
    if (offsets) *offsets = plan->offsets.data();
    if (chan_of) *chan_of = plan->chan_of.data();
    if (macs_per_pixel) *macs_per_pixel = (int64_t)plan->G * (plan->desc.K * plan->desc.K + plan->desc.M);
    return GDWS_OK;
}

int gdws_plan_factors(const gdws_plan_t *plan, float *dw_out, float *pw_out)
{
    if (!plan) return GDWS_ENULL;
    if (dw_out) std::memcpy(dw_out, plan->dw.data(), plan->dw.size() * sizeof(float));
    if (pw_out) std::memcpy(pw_out, plan->pw.data(), plan->pw.size() * sizeof(float));
    return GDWS_OK;
}

int32_t gdws_intermediate_channels(const gdws_plan_t *plan) { return plan ? plan->Gt : 0; }

size_t gdws_workspace_bytes(const gdws_plan_t *plan, int32_t N, int32_t H, int32_t W, int mode)
{
    if (!plan) return 0;
    int Ho, Wo;
    if (check_image(plan->desc, N, H, W, &Ho, &Wo)) return 0;
    if (mode != GDWS_MODE_UNFUSED && fused_supported(plan, N, H, W))  // (with or without a pooled epilogue)
        return std::max(fused_split_bytes(plan, N, H, W, Ho, Wo, false), fused_split_bytes(plan, N, H, W, Ho, Wo, true));
    if (mode == GDWS_MODE_FUSED) return 0;
    return intermediate_bytes(plan, N, Ho, Wo);
}

int gdws_forward(const gdws_plan_t *plan, const void *x, const void *residual, void *y, int32_t N, int32_t H,
                 int32_t W, void *workspace, size_t workspace_bytes, int mode, void *stream)
{
    if (!plan || !x || !y) return GDWS_ENULL;
    if (plan->desc.has_residual && !residual) return GDWS_ENULL;
    if (mode < GDWS_MODE_AUTO || mode > GDWS_MODE_UNFUSED) return GDWS_EINVAL;
    int Ho, Wo;
    int rc = check_image(plan->desc, N, H, W, &Ho, &Wo);
    if (rc) return rc;
    hipStream_t s = (hipStream_t)stream;
    const bool fused_ok = fused_supported(plan, N, H, W);
    if (mode != GDWS_MODE_UNFUSED && fused_ok) {
        rc = run_fused(plan, x, residual, y, N, H, W, Ho, Wo, s, 0, workspace, workspace_bytes);
        if (rc != GDWS_EUNSUPPORTED) return rc;
    }
    // asked for the fused path on a shape the matrix-core kernel does not take: the vector-ALU fused kernel
    if (mode == GDWS_MODE_FUSED) return run_fused_generic(plan, x, residual, y, N, H, W, Ho, Wo, s);
    if (!workspace || workspace_bytes < intermediate_bytes(plan, N, Ho, Wo)) return GDWS_EWORKSPACE;
    rc = run_gdw(plan, x, workspace, N, H, W, Ho, Wo, s);
    if (rc) return rc;
    return run_pw(plan, workspace, residual, y, N, Ho, Wo, s);
}

size_t gdws_backward_workspace_bytes(const gdws_plan_t *plan, int32_t N, int32_t H, int32_t W)
{
    if (!plan) return 0;
    int Ho, Wo;
    if (check_image(plan->desc, N, H, W, &Ho, &Wo)) return 0;
    return backward_workspace_bytes(N, plan->desc.M, plan->G, plan->desc.K, Ho, Wo);
}

int gdws_backward(const gdws_plan_t *plan, const void *x, const void *dy, void *dx, float *d_dw, float *d_pw,
                  float *d_bias, int32_t N, int32_t H, int32_t W, void *workspace, size_t workspace_bytes,
                  void *stream)
{
    if (!plan || !x || !dy) return GDWS_ENULL;
    int Ho, Wo;
    const int rc = check_image(plan->desc, N, H, W, &Ho, &Wo);
    if (rc) return rc;
    if (!workspace || workspace_bytes < backward_workspace_bytes(N, plan->desc.M, plan->G, plan->desc.K, Ho, Wo))
        return GDWS_EWORKSPACE;
    const gdws_layer_desc_t &d = plan->desc;
    BackwardArgs a;
    a.x = x; a.dy = dy; a.dx = dx; a.g_dw = d_dw; a.g_pw = d_pw; a.g_bias = d_bias;
    a.dw = plan->d_dw; a.pw = plan->d_pw; a.offsets = plan->d_offsets; a.chan_of = plan->d_chan_of;
    a.workspace = workspace; a.dtype = d.dtype; a.layout = d.layout;
    a.N = N; a.C = d.C; a.H = H; a.W = W; a.M = d.M; a.G = plan->G; a.K = d.K; a.stride = d.stride; a.pad = d.pad;
    a.Ho = Ho; a.Wo = Wo;
    return launch_backward(a, (hipStream_t)stream);
}

}  // extern "C"

namespace {

int forward_maxpool2(const gdws_plan_t *plan, const void *x, void *y, int32_t N, int32_t H, int32_t W, void *ws,
                     size_t ws_bytes, void *stream)
{
    if (!plan || !x || !y) return GDWS_ENULL;
    int Ho, Wo;
    int rc = check_image(plan->desc, N, H, W, &Ho, &Wo);
    if (rc) return rc;
    if (plan->desc.has_residual || plan->desc.layout != GDWS_NHWC || !fused_supported(plan, N, H, W))
        return GDWS_EUNSUPPORTED;
    if (Ho < 2 || Wo < 2) return GDWS_EINVAL;  // the pooled tensor would be empty
    // workgroups store pooled rows while others still read x: the two tensors must not share memory
    if (ranges_overlap(x, (size_t)N * plan->desc.C * H * W * 2, y, (size_t)N * plan->desc.M * (Ho / 2) * (Wo / 2) * 2))
        return GDWS_EINVAL;
    return run_fused(plan, x, nullptr, y, N, H, W, Ho, Wo, (hipStream_t)stream, 1, ws, ws_bytes);
}

}  // namespace

extern "C" {

int gdws_forward_maxpool2(const gdws_plan_t *plan, const void *x, void *y, int32_t N, int32_t H, int32_t W,
                          void *stream)
{
    return forward_maxpool2(plan, x, y, N, H, W, nullptr, 0, stream);
}

int gdws_gdw_forward(const gdws_plan_t *plan, const void *x, void *t, int32_t N, int32_t H, int32_t W, void *stream)
{
    if (!plan || !x || !t) return GDWS_ENULL;
    int Ho, Wo;
    int rc = check_image(plan->desc, N, H, W, &Ho, &Wo);
    if (rc) return rc;
    return run_gdw(plan, x, t, N, H, W, Ho, Wo, (hipStream_t)stream);
}

int gdws_pw_forward(const gdws_plan_t *plan, const void *t, const void *residual, void *y, int32_t N, int32_t Ho,
                    int32_t Wo, void *stream)
{
    if (!plan || !t || !y) return GDWS_ENULL;
    if (plan->desc.has_residual && !residual) return GDWS_ENULL;
    if (N < 1 || Ho < 1 || Wo < 1) return GDWS_EINVAL;
    return run_pw(plan, t, residual, y, N, Ho, Wo, (hipStream_t)stream);
}

size_t conv_dense_workspace_bytes(const gdws_layer_desc_t *desc)
{
    if (check_desc(desc)) return 0;
    // (the image size is not known here: the kernel's addressing limit is checked by the forward call)
    if (conv_mfma_supported(desc->dtype, desc->layout, desc->K, desc->stride, desc->pad, desc->C, 0))
        return conv_mfma_workspace_bytes(desc->C, desc->M);
    return 0;
}

int conv_dense_forward(const gdws_layer_desc_t *desc, const void *w, const float *bias, const void *x,
                       const void *residual, void *y, int32_t N, int32_t H, int32_t W, void *workspace,
                       size_t workspace_bytes, void *stream)
{
    int rc = check_desc(desc);
    if (rc) return rc;
    if (!w || !x || !y) return GDWS_ENULL;
    if ((desc->has_bias && !bias) || (desc->has_residual && !residual)) return GDWS_ENULL;
    int Ho, Wo;
    rc = check_image(*desc, N, H, W, &Ho, &Wo);
    if (rc) return rc;
    DenseArgs a;
    a.x = x; a.y = y; a.w = w;
    a.ep.bias = desc->has_bias ? bias : nullptr;
    a.ep.residual = desc->has_residual ? residual : nullptr;
    a.ep.relu = desc->relu;
    a.dtype = desc->dtype; a.layout = desc->layout;
    a.N = N; a.C = desc->C; a.H = H; a.W = W; a.M = desc->M; a.K = desc->K;
    a.stride = desc->stride; a.pad = desc->pad; a.Ho = Ho; a.Wo = Wo;
    if (conv_mfma_supported(desc->dtype, desc->layout, desc->K, desc->stride, desc->pad, desc->C,
                            (int64_t)N * desc->C * H * W)) {
        if (!workspace || workspace_bytes < conv_mfma_workspace_bytes(desc->C, desc->M)) return GDWS_EWORKSPACE;
        return launch_conv_mfma(a, workspace, (hipStream_t)stream);
    }
    return launch_dense_direct(a, (hipStream_t)stream);
}

}  // extern "C"

// ---------------------------------------------------------------------------------
// networks
// ---------------------------------------------------------------------------------

namespace {

const gdws_layer_desc_t &node_desc(const NetNode &n)
{
    return n.l.kind == GDWS_LAYER_GDWS ? n.l.plan->desc : n.l.desc;
}

// True if node i + 1 is a 2 x 2 / stride-2 max-pool without padding whose input is node i, and nothing else reads
// node i: the pair can then run as one kernel.
bool pooled_by_next(const gdws_net_t *net, int i)
{
    const int L = (int)net->nodes.size();
    if (i + 1 >= L || net->nodes[i].l.kind != GDWS_LAYER_GDWS) return false;
    const auto &q = net->nodes[i + 1].l;
    if (q.kind != GDWS_LAYER_MAXPOOL || q.src != i || q.desc.K != 2 || q.desc.stride != 2 || q.desc.pad != 0) return false;
    for (int k = i + 2; k < L; ++k)
        if (net->nodes[k].l.src == i || net->nodes[k].l.residual == i) return false;
    return true;
}

// Shapes and workspace offsets of every node for one input size.  Buffers are handed out best-fit from a free
// list; a buffer returns to the list once the output of its last reader has been placed, so no node writes
// into a tensor it reads.  A layer that may run as one kernel with the max-pool behind it (pooled_by_next) reads its
// input while that kernel writes the pool's output: its inputs are therefore released only after the pool's
// output has been placed.
int layout_buffers(const gdws_net_t *net, int N, int H, int W, NetLayout &lay)
{
    const int L = (int)net->nodes.size();
    std::vector<NodeShape> &sh = lay.sh;
    sh.assign(L, NodeShape{});
    std::vector<int> release_at(L, -1);  // node after whose output placement a node's buffer is free again
    for (int i = 0; i < L; ++i) {
        const auto &l = net->nodes[i].l;
        if (l.src >= 0) release_at[l.src] = i;
        if (l.residual >= 0) release_at[l.residual] = std::max(release_at[l.residual], i);
    }
    std::vector<int> last_use = release_at;
    for (int j = 0; j < L; ++j)
        if (release_at[j] >= 0 && pooled_by_next(net, release_at[j])) ++release_at[j];
    struct Block { size_t off, size; bool free; };
    std::vector<Block> blocks;
    std::vector<int> block_of(L, -1);
    size_t top = 0, scratch = 0;
    const size_t eb = dtype_bytes(net->dtype);
    for (int i = 0; i < L; ++i) {
        const auto &n = net->nodes[i];
        const gdws_layer_desc_t &d = node_desc(n);
        int ic, ih, iw;
        if (n.l.src < 0) { ic = d.C; ih = H; iw = W; }
        else { ic = sh[n.l.src].C; ih = sh[n.l.src].H; iw = sh[n.l.src].W; }
        if (ic != d.C) return GDWS_EINVAL;
        int Ho, Wo;
        int rc = check_image(d, N, ih, iw, &Ho, &Wo);
        if (rc) return rc;
        sh[i].C = n.l.kind == GDWS_LAYER_MAXPOOL ? d.C : d.M;
        sh[i].H = Ho; sh[i].W = Wo;
        sh[i].bytes = (size_t)N * sh[i].C * Ho * Wo * eb;
        if (n.l.residual >= 0) {
            const NodeShape &r = sh[n.l.residual];
            if (r.C != sh[i].C || r.H != Ho || r.W != Wo) return GDWS_EINVAL;
        }
        sh[i].scratch = n.l.kind == GDWS_LAYER_GDWS    ? gdws_workspace_bytes(n.l.plan, N, ih, iw, GDWS_MODE_AUTO)
                        : n.l.kind == GDWS_LAYER_DENSE ? conv_dense_workspace_bytes(&n.l.desc)
                                                       : 0;
        scratch = std::max(scratch, sh[i].scratch);
        if (i == L - 1) { sh[i].offset = SIZE_MAX; break; }
        const size_t need = (sh[i].bytes + 255) & ~(size_t)255;
        int pick = -1;
        for (int b = 0; b < (int)blocks.size(); ++b)
            if (blocks[b].free && blocks[b].size >= need && (pick < 0 || blocks[b].size < blocks[pick].size)) pick = b;
        if (pick < 0) { blocks.push_back(Block{top, need, false}); pick = (int)blocks.size() - 1; top += need; }
        blocks[pick].free = false;
        block_of[i] = pick;
        sh[i].offset = blocks[pick].off;
        for (int j = 0; j < i; ++j)
            if (release_at[j] == i && block_of[j] >= 0) blocks[block_of[j]].free = true;
        if (last_use[i] < 0) blocks[pick].free = true;  // dead output
    }
    lay.N = N; lay.H = H; lay.W = W;
    lay.act_top = top;                                    // scratch sits after the activation buffers
    lay.total = top + ((scratch + 255) & ~(size_t)255);
    return GDWS_OK;
}

// The layout for this input size: worked out at the first request (gdws_net_workspace_bytes, which a caller needs
// before its first forward anyway) and kept, so that a forward call neither allocates nor plans.
int cached_layout(const gdws_net_t *net, int N, int H, int W, const NetLayout **out)
{
    std::lock_guard<std::mutex> lock(net->mu);
    for (const auto &l : net->layouts)
        if (l->N == N && l->H == H && l->W == W) { *out = l.get(); return GDWS_OK; }
    std::unique_ptr<NetLayout> lay(new NetLayout);
    const int rc = layout_buffers(net, N, H, W, *lay);
    if (rc) return rc;
    net->layouts.push_back(std::move(lay));
    *out = net->layouts.back().get();
    return GDWS_OK;
}

int run_network(const gdws_net_t *net, const NetLayout &lay, const void *x, void *y, int N, int H, int W, void *workspace,
                void *stream)
{
    const std::vector<NodeShape> &sh = lay.sh;
    char *ws = (char *)workspace;
    void *scratch = ws ? ws + lay.act_top : nullptr;
    const size_t scratch_bytes = lay.total - lay.act_top;
    const int L = (int)net->nodes.size();
    int rc = GDWS_OK;
    for (int i = 0; i < L; ++i) {
        const NetNode &n = net->nodes[i];
        const void *in = n.l.src < 0 ? x : ws + sh[n.l.src].offset;
        const int ih = n.l.src < 0 ? H : sh[n.l.src].H, iw = n.l.src < 0 ? W : sh[n.l.src].W;
        const void *res = n.l.residual >= 0 ? ws + sh[n.l.residual].offset : nullptr;
        void *outp = sh[i].offset == SIZE_MAX ? y : ws + sh[i].offset;
        if (n.l.kind == GDWS_LAYER_GDWS && pooled_by_next(net, i)) {
            // the 2 x 2 max-pool that is this layer's only reader runs in its epilogue when the kernel can
            void *pout = sh[i + 1].offset == SIZE_MAX ? y : ws + sh[i + 1].offset;
            rc = forward_maxpool2(n.l.plan, in, pout, N, ih, iw, scratch, scratch_bytes, stream);
            if (rc == GDWS_OK) { ++i; continue; }
            if (rc != GDWS_EUNSUPPORTED && rc != GDWS_EINVAL) return rc;
            rc = gdws_forward(n.l.plan, in, res, outp, N, ih, iw, scratch, scratch_bytes, GDWS_MODE_AUTO, stream);
        } else if (n.l.kind == GDWS_LAYER_GDWS) {
            rc = gdws_forward(n.l.plan, in, res, outp, N, ih, iw, scratch, scratch_bytes, GDWS_MODE_AUTO, stream);
        } else if (n.l.kind == GDWS_LAYER_DENSE && n.pwm.valid) {
            PwMfmaArgs m;
            m.t = in; m.y = outp; m.tables = &n.pwm; m.dtype = n.l.desc.dtype; m.M = n.l.desc.M;
            m.ep.bias = nullptr; m.ep.residual = n.l.desc.has_residual ? res : nullptr; m.ep.relu = n.l.desc.relu;
            m.P = (int64_t)N * sh[i].H * sh[i].W;
            m.stride = n.l.desc.stride; m.Ho = sh[i].H; m.Wo = sh[i].W; m.H = ih; m.W = iw;
            rc = launch_pw_mfma(m, (hipStream_t)stream);
        } else if (n.l.kind == GDWS_LAYER_DENSE && n.dm.valid &&
                   dense_mfma_image_supported((int64_t)N * n.l.desc.C * ih * iw)) {
            DenseMfmaArgs m;
            m.x = in; m.y = outp; m.tables = &n.dm; m.dtype = n.l.desc.dtype; m.relu = n.l.desc.relu;
            m.N = N; m.C = n.l.desc.C; m.H = ih; m.W = iw; m.M = n.l.desc.M; m.K = n.l.desc.K;
            m.stride = n.l.desc.stride; m.pad = n.l.desc.pad; m.Ho = sh[i].H; m.Wo = sh[i].W;
            rc = launch_dense_mfma(m, (hipStream_t)stream);
        } else if (n.l.kind == GDWS_LAYER_DENSE) {
            rc = conv_dense_forward(&n.l.desc, n.d_w, n.d_bias, in, res, outp, N, ih, iw, scratch, scratch_bytes,
                                    stream);
        } else {
            PoolArgs a;
            a.x = in; a.y = outp; a.dtype = net->dtype; a.layout = net->layout;
            a.N = N; a.C = n.l.desc.C; a.H = ih; a.W = iw; a.K = n.l.desc.K; a.stride = n.l.desc.stride;
            a.pad = n.l.desc.pad; a.Ho = sh[i].H; a.Wo = sh[i].W;
            rc = launch_maxpool(a, (hipStream_t)stream);
        }
        if (rc) return rc;
    }
    return GDWS_OK;
}

}  // namespace

extern "C" {

int gdws_net_create(const gdws_net_layer_t *layers, int32_t n_layers, gdws_net_t **out)
{
    GDWS_TRY
    if (!layers || !out) return GDWS_ENULL;
    if (n_layers < 1) return GDWS_EINVAL;
    gdws_net_t *net = new (std::nothrow) gdws_net_t;
    if (!net) return GDWS_ENOMEM;
    std::unique_ptr<gdws_net_t> guard(net);
    net->nodes.resize(n_layers);
    for (int i = 0; i < n_layers; ++i) {
        const gdws_net_layer_t &l = layers[i];
        int rc = GDWS_OK;
        if (l.kind < GDWS_LAYER_GDWS || l.kind > GDWS_LAYER_MAXPOOL) rc = GDWS_EINVAL;
        else if (l.src < -1 || l.src >= i || l.residual < -2 || l.residual >= i || l.residual == -1) rc = GDWS_EINVAL;
        else if (l.kind == GDWS_LAYER_GDWS && !l.plan) rc = GDWS_ENULL;
        else if (l.kind != GDWS_LAYER_GDWS) rc = check_desc(&l.desc);
        if (!rc && l.kind == GDWS_LAYER_DENSE && (!l.w || (l.desc.has_bias && !l.bias))) rc = GDWS_ENULL;
        if (!rc) {
            const gdws_layer_desc_t &d = l.kind == GDWS_LAYER_GDWS ? l.plan->desc : l.desc;
            if (i == 0) { net->dtype = d.dtype; net->layout = d.layout; }
            else if (d.dtype != net->dtype || d.layout != net->layout) rc = GDWS_EINVAL;
            if (!rc && (d.has_residual != 0) != (l.residual >= 0) && l.kind != GDWS_LAYER_MAXPOOL) rc = GDWS_EINVAL;
            if (!rc && l.kind == GDWS_LAYER_MAXPOOL && l.residual >= 0) rc = GDWS_EINVAL;
        }
        if (!rc) {
            net->nodes[i].l = l;
            if (l.kind == GDWS_LAYER_DENSE) {
                const size_t cnt = (size_t)l.desc.M * l.desc.C * l.desc.K * l.desc.K;
                rc = upload_as_dtype(&net->nodes[i].d_w, l.w, cnt, l.desc.dtype);
                if (!rc && l.desc.has_bias) {
                    std::vector<float> b(l.bias, l.bias + l.desc.M);
                    rc = upload(&net->nodes[i].d_bias, b);
                }
                const gdws_layer_desc_t &dd = l.desc;
                if (!rc && dd.K == 1 && dd.pad == 0 && dd.layout == GDWS_NHWC && dd.dtype != GDWS_F32 &&
                    dd.C % 16 == 0) {
                    // a 1 x 1 convolution is the pointwise stage with G = C; the kernel takes rounded weights
                    std::vector<float> wq(l.w, l.w + cnt);
                    for (auto &v : wq) v = round_to_dtype(v, dd.dtype);
                    build_pw_mfma_tables(net->nodes[i].pwm, dd.dtype, dd.C, dd.M, wq.data(), dd.has_bias ? l.bias : nullptr);
                    rc = upload(&net->nodes[i].pwm.d_frag, net->nodes[i].pwm.frag);
                    if (!rc) rc = upload(&net->nodes[i].pwm.d_bias_pad, net->nodes[i].pwm.bias_pad);
                }
                if (!rc && dense_mfma_supported(dd.dtype, dd.layout, dd.K, dd.C, dd.stride, dd.has_residual != 0)) {
                    std::vector<float> wq(l.w, l.w + cnt);
                    for (auto &v : wq) v = round_to_dtype(v, dd.dtype);
                    build_dense_mfma_tables(net->nodes[i].dm, dd.dtype, dd.K, dd.C, dd.M, wq.data(), dd.has_bias ? l.bias : nullptr);
                    rc = upload(&net->nodes[i].dm.d_frag, net->nodes[i].dm.frag);
                    if (!rc) rc = upload(&net->nodes[i].dm.d_bias_pad, net->nodes[i].dm.bias_pad);
                }
                net->nodes[i].l.w = nullptr;  // host pointers are not kept
                net->nodes[i].l.bias = nullptr;
            }
        }
        if (rc) return rc;
    }
    *out = guard.release();
    return GDWS_OK;
    GDWS_CATCH
}

int gdws_net_destroy(gdws_net_t *net)
{
    delete net;
    return GDWS_OK;
}

size_t gdws_net_workspace_bytes(const gdws_net_t *net, int32_t N, int32_t H, int32_t W)
{
    if (!net) return 0;
    try {
        const NetLayout *lay = nullptr;
        if (cached_layout(net, N, H, W, &lay)) return 0;
        return lay->total;
    } catch (...) {
        return 0;
    }
}

int gdws_network_forward(const gdws_net_t *net, const void *x, void *y, int32_t N, int32_t H, int32_t W,
                         void *workspace, size_t workspace_bytes, void *stream)
{
    GDWS_TRY
    if (!net || !x || !y) return GDWS_ENULL;
    const NetLayout *lay = nullptr;
    int rc = cached_layout(net, N, H, W, &lay);
    if (rc) return rc;
    if (lay->total > 0 && (!workspace || workspace_bytes < lay->total)) return GDWS_EWORKSPACE;
    return run_network(net, *lay, x, y, N, H, W, workspace, stream);
    GDWS_CATCH
}

}  // extern "C"

// ---------------------------------------------------------------------------------
// launch graphs (the batch-1 protocol of Appendix A: a whole forward replayed as one graph launch)
// ---------------------------------------------------------------------------------

struct gdws_graph_s {
    hipGraph_t graph = nullptr;
    hipGraphExec_t exec = nullptr;
    ~gdws_graph_s()
    {
        if (exec) (void)hipGraphExecDestroy(exec);
        if (graph) (void)hipGraphDestroy(graph);
    }
};

extern "C" {

int gdws_capture_begin(void *stream)
{
    if (!stream) return GDWS_EINVAL;  // the default stream cannot be captured
    GDWS_HIP_CHECK(hipStreamBeginCapture((hipStream_t)stream, hipStreamCaptureModeThreadLocal));
    return GDWS_OK;
}

int gdws_capture_end(void *stream, gdws_graph_t **out)
{
    GDWS_TRY
    if (!stream) return GDWS_EINVAL;
    hipGraph_t graph = nullptr;
    const hipError_t e = hipStreamEndCapture((hipStream_t)stream, &graph);  // (always ends the capture)
    if (!out) { if (graph) (void)hipGraphDestroy(graph); return GDWS_ENULL; }
    if (e != hipSuccess || !graph) return GDWS_EHIP;
    std::unique_ptr<gdws_graph_t> g(new gdws_graph_t);
    g->graph = graph;
    GDWS_HIP_CHECK(hipGraphInstantiate(&g->exec, graph, nullptr, nullptr, 0));
    *out = g.release();
    return GDWS_OK;
    GDWS_CATCH
}

int gdws_graph_launch(const gdws_graph_t *graph, void *stream)
{
    if (!graph) return GDWS_ENULL;
    GDWS_HIP_CHECK(hipGraphLaunch(graph->exec, (hipStream_t)stream));
    return GDWS_OK;
}

int gdws_graph_destroy(gdws_graph_t *graph)
{
    delete graph;
    return GDWS_OK;
}

}  // extern "C"

// ---------------------------------------------------------------------------------
// the forward pass for callers that cannot allocate: the intermediate lives in a static device array
// ---------------------------------------------------------------------------------

namespace {

constexpr size_t kStaticScratchBytes = GDWS_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices] = {};  // device address of `scratch` on each GPU (every GPU holds its own copy)
std::mutex g_scratch_mu;

// The array's address on the current device, looked up once per device.  (In host code `scratch` itself is only
// a handle for this lookup, never a device address.)
int static_scratch(void **out)
{
    int dev = -1;
    GDWS_HIP_CHECK(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return GDWS_EUNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        GDWS_HIP_CHECK(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) return GDWS_EHIP;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return GDWS_OK;
}

}  // namespace

extern "C" int gdws_forward_static(const gdws_plan_t *plan, const void *x, const void *residual, void *y, int32_t N,
                                   int32_t H, int32_t W, void *stream)
{
    if (!plan || !x || !y) return GDWS_ENULL;
    if (plan->desc.has_residual && !residual) return GDWS_ENULL;
    int Ho, Wo;
    int rc = check_image(plan->desc, N, H, W, &Ho, &Wo);
    if (rc) return rc;
    if (intermediate_bytes(plan, N, Ho, Wo) > kStaticScratchBytes) return GDWS_EWORKSPACE;
    void *t = nullptr;
    rc = static_scratch(&t);
    if (rc) return rc;
    // every element of the intermediate (its zero padding channels included) is written by the depthwise stage
    // before the pointwise stage reads it: nothing of an earlier call's contents has to be cleared
    rc = run_gdw(plan, x, t, N, H, W, Ho, Wo, (hipStream_t)stream);
    if (rc) return rc;
    return run_pw(plan, t, residual, y, N, Ho, Wo, (hipStream_t)stream);
}
