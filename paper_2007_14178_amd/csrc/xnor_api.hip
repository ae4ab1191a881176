// Host side of the C ABI declared in xnor.h: argument validation, geometry, kernel choice.
// Nothing here allocates or synchronises; every call enqueues on the caller's stream.
#include <atomic>
#include <stdio.h>
#include <string.h>

#include "xnor_internal.hpp"

namespace {

thread_local char g_hip_err[256] = "";

int hip_status(hipError_t e)
{
    if (e == hipSuccess) return XNOR_OK;
    snprintf(g_hip_err, sizeof g_hip_err, "%s: %s", hipGetErrorName(e), hipGetErrorString(e));
    return XNOR_E_HIP;
}

constexpr long long kMaxIndex = 0x7fffffffLL;

bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

// Validates a layer and fills the derived geometry.
int make_geom(const xnor_shape *s, xnor::Geom *g)
{
    if (!s) return XNOR_E_NULL;
    if (s->N <= 0 || s->C <= 0 || s->H <= 0 || s->W <= 0 || s->F <= 0 || s->kh <= 0 ||
        s->kw <= 0 || s->sh <= 0 || s->sw <= 0 || s->ph < 0 || s->pw < 0)
        return XNOR_E_SHAPE;
    const long long eh = (long long)s->H + 2LL * s->ph - s->kh;
    const long long ew = (long long)s->W + 2LL * s->pw - s->kw;
    if (eh < 0 || ew < 0) return XNOR_E_SHAPE;
    const long long OH = eh / s->sh + 1, OW = ew / s->sw + 1;
    const long long Cw = ((long long)s->C + 31) / 32;
    if ((long long)s->N * s->H * s->W > kMaxIndex || (long long)s->N * OH * OW > kMaxIndex ||
        (long long)s->H * s->W * Cw > kMaxIndex || (long long)s->F * s->kh * s->kw * Cw > kMaxIndex ||
        (long long)s->kh * s->kw * s->C > kMaxIndex ||
        ((long long)s->N * OH * OW) > (kMaxIndex * 256) / s->F ||
        (long long)s->H + 2LL * s->ph > kMaxIndex || (long long)s->W + 2LL * s->pw > kMaxIndex)
        return XNOR_E_SHAPE;
    *g = xnor::Geom{s->N, s->C, s->H, s->W, s->F, s->kh, s->kw, s->sh, s->sw, s->ph, s->pw,
                    (int)OH, (int)OW, (int)Cw};
    return XNOR_OK;
}

int pick_algo(const xnor::Geom &g, size_t workspace_bytes)
{
    const size_t need = xnor::conv_mfma_workspace_bytes(g);
    if (need > 0 && workspace_bytes >= need) return XNOR_ALGO_MFMA;
    if (xnor::conv_tiled_supports(g)) return XNOR_ALGO_TILED;
    return XNOR_ALGO_DIRECT;
}

// The expanded filters of xnor_conv2d_fwd_static live here instead of in a caller's workspace.
// One copy per GPU, held until the process ends.  In host code the name is only a handle: the
// memory's address on the current device comes from hipGetSymbolAddress, once per device.
constexpr size_t kStaticScratchBytes = (size_t)XNOR_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::atomic<void *> g_scratch_ptr[kMaxDevices];

hipError_t static_scratch(void **ptr)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev].store(p, std::memory_order_release);   // (racing first calls store the same address)
    }
    *ptr = p;
    return hipSuccess;
}

}  // namespace

extern "C" {

int xnor_out_dim(const xnor_shape *s, int *OH, int *OW)
{
    if (!s || !OH || !OW) return XNOR_E_NULL;
    xnor::Geom g;
    const int rc = make_geom(s, &g);
    if (rc) return rc;
    *OH = g.OH;
    *OW = g.OW;
    return XNOR_OK;
}

int xnor_packed_words(int C) { return C <= 0 ? XNOR_E_SHAPE : (int)(((long long)C + 31) / 32); }

const char *xnor_strerror(int status)
{
    switch (status) {
        case XNOR_OK: return "ok";
        case XNOR_E_NULL: return "a required pointer is NULL";
        case XNOR_E_SHAPE: return "bad shape (non-positive dimension, empty output or tensor too large)";
        case XNOR_E_ALIGN: return "pointer not aligned as required";
        case XNOR_E_HIP: return "HIP launch failed (see xnor_last_hip_error)";
        case XNOR_E_UNSUPPORTED: return "the requested algorithm does not support this shape";
        case XNOR_E_WORKSPACE: return "the requested algorithm needs a larger workspace";
        default: return "unknown status";
    }
}

const char *xnor_last_hip_error(void) { return g_hip_err; }

int xnor_binarize_pack(const float *x, int N, int C, int H, int W, uint32_t *packed, void *stream)
{
    if (!x || !packed) return XNOR_E_NULL;
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0) return XNOR_E_SHAPE;
    const long long Cw = ((long long)C + 31) / 32;
    if ((long long)N * H * W > kMaxIndex || Cw > 65535 || (long long)H * W > kMaxIndex / Cw)
        return XNOR_E_SHAPE;
    if (!aligned(x, 4) || !aligned(packed, 4)) return XNOR_E_ALIGN;
    return hip_status(xnor::launch_binarize_pack(x, N, C, H, W, packed, (hipStream_t)stream));
}

int xnor_scale_K(const float *I, const xnor_shape *s, float *A_work, float *K, void *stream)
{
    if (!I || !s || !A_work || !K) return XNOR_E_NULL;
    xnor::Geom g;
    const int rc = make_geom(s, &g);
    if (rc) return rc;
    if (!aligned(I, 4) || !aligned(A_work, 4) || !aligned(K, 4)) return XNOR_E_ALIGN;
    hipStream_t st = (hipStream_t)stream;
    hipError_t e = xnor::launch_channel_mean_abs(I, g.N, g.C, g.H, g.W, A_work, st);
    if (e != hipSuccess || !K) return hip_status(e);
    return hip_status(xnor::launch_box_filter_K(A_work, g, K, st));
}

int xnor_alpha(const float *Wt, int F, int C, int kh, int kw, float *alpha, void *stream)
{
    if (!Wt || !alpha) return XNOR_E_NULL;
    if (F <= 0 || C <= 0 || kh <= 0 || kw <= 0) return XNOR_E_SHAPE;
    const long long n_red = (long long)C * kh * kw;
    if (n_red > kMaxIndex) return XNOR_E_SHAPE;
    if (!aligned(Wt, 4) || !aligned(alpha, 4)) return XNOR_E_ALIGN;
    return hip_status(xnor::launch_alpha(Wt, F, n_red, alpha, (hipStream_t)stream));
}

int xnor_input_prepare(const float *I, const xnor_shape *s, uint32_t *Ipk, float *A_work, float *K,
                       void *stream)
{
    if (!I || !s || !Ipk || !A_work) return XNOR_E_NULL;   // K may be NULL: then only Ipk and A are produced
    xnor::Geom g;
    const int rc = make_geom(s, &g);
    if (rc) return rc;
    if (!aligned(I, 4) || !aligned(Ipk, 4) || !aligned(A_work, 4) || (K && !aligned(K, 4))) return XNOR_E_ALIGN;
    hipStream_t st = (hipStream_t)stream;
    hipError_t e;
    if (xnor::pack_and_mean_supports(g.C)) {
        e = xnor::launch_pack_and_mean(I, g.N, g.C, g.H, g.W, Ipk, A_work, st);
    } else {   // more channel words than one block's LDS holds: two passes
        e = xnor::launch_binarize_pack(I, g.N, g.C, g.H, g.W, Ipk, st);
        if (e == hipSuccess) e = xnor::launch_channel_mean_abs(I, g.N, g.C, g.H, g.W, A_work, st);
    }
    if (e != hipSuccess || !K) return hip_status(e);
    return hip_status(xnor::launch_box_filter_K(A_work, g, K, st));
}

int xnor_prepare(const float *I, const float *Wt, const xnor_shape *s, uint32_t *Ipk, float *A_work,
                 float *K, uint32_t *Wpk, float *M_work, float *alpha, void *workspace,
                 size_t workspace_bytes, void *stream)
{
    if (!I || !Wt || !s || !Ipk || !A_work || !Wpk || !M_work || !alpha) return XNOR_E_NULL;
    xnor::Geom g;
    const int rc = make_geom(s, &g);
    if (rc) return rc;
    if (!aligned(I, 4) || !aligned(Wt, 4) || !aligned(Ipk, 4) || !aligned(A_work, 4) || (K && !aligned(K, 4)) ||
        !aligned(Wpk, 4) || !aligned(M_work, 4) || !aligned(alpha, 4) || (workspace && !aligned(workspace, 16)))
        return XNOR_E_ALIGN;
    xnor::ExpandLayout L{};
    if (workspace) {
        L = xnor::conv_mfma_expand_layout(g);
        if (!L.ok) return XNOR_E_UNSUPPORTED;
        if (workspace_bytes < L.ws_bytes) return XNOR_E_WORKSPACE;
    }
    hipStream_t st = (hipStream_t)stream;
    const int taps = g.kh * g.kw;
    if (!xnor::prepare_both_supports(I, g.N, g.C, g.H, g.W, taps)) {
        int r = xnor_input_prepare(I, s, Ipk, A_work, K, stream);
        if (!r) r = xnor_filter_prepare(Wt, g.F, g.C, g.kh, g.kw, Wpk, M_work, alpha, stream);
        if (!r && workspace) r = hip_status(xnor::launch_expand_filters(Wpk, g, workspace, st));
        return r;
    }
    const bool expand_here = workspace && xnor::prepare_both_can_expand(g.C, taps);
    hipError_t e = xnor::launch_prepare_both(I, g.N, g.C, g.H, g.W, Ipk, A_work, Wt, g.F, taps, Wpk, M_work, alpha,
                                             expand_here ? workspace : nullptr, L, st);
    if (e == hipSuccess && workspace && !expand_here) e = xnor::launch_expand_filters(Wpk, g, workspace, st);
    if (e != hipSuccess || !K) return hip_status(e);
    return hip_status(xnor::launch_box_filter_K(A_work, g, K, st));
}

int xnor_filter_prepare(const float *Wt, int F, int C, int kh, int kw, uint32_t *Wpk, float *M_work,
                        float *alpha, void *stream)
{
    if (!Wt || !Wpk || !M_work || !alpha) return XNOR_E_NULL;
    if (F <= 0 || C <= 0 || kh <= 0 || kw <= 0) return XNOR_E_SHAPE;
    const long long Cw = ((long long)C + 31) / 32;
    if ((long long)F * kh * kw > kMaxIndex || (long long)C * kh * kw > kMaxIndex || Cw > 65535 ||
        (long long)F * kh * kw > kMaxIndex / Cw)
        return XNOR_E_SHAPE;
    if (!aligned(Wt, 4) || !aligned(Wpk, 4) || !aligned(M_work, 4) || !aligned(alpha, 4)) return XNOR_E_ALIGN;
    hipStream_t st = (hipStream_t)stream;
    hipError_t e;
    if (xnor::filter_pack_mean_supports(kh * kw)) {
        e = xnor::launch_filter_pack_mean(Wt, F, C, kh * kw, Wpk, M_work, alpha, st);
    } else if (xnor::pack_and_mean_supports(C)) {
        e = xnor::launch_pack_and_mean(Wt, F, C, kh, kw, Wpk, M_work, st);
        if (e == hipSuccess) e = xnor::launch_alpha_from_tap_means(M_work, F, kh * kw, alpha, st);
    } else {
        e = xnor::launch_binarize_pack(Wt, F, C, kh, kw, Wpk, st);
        if (e == hipSuccess) e = xnor::launch_alpha(Wt, F, (long long)C * kh * kw, alpha, st);
    }
    return hip_status(e);
}

int xnor_conv2d_pick_algo(const xnor_shape *s, size_t workspace_bytes)
{
    xnor::Geom g;
    const int rc = make_geom(s, &g);
    return rc ? rc : pick_algo(g, workspace_bytes);
}

int xnor_conv2d_workspace_bytes(const xnor_shape *s, size_t *bytes)
{
    if (!s || !bytes) return XNOR_E_NULL;
    xnor::Geom g;
    const int rc = make_geom(s, &g);
    if (rc) return rc;
    *bytes = xnor::conv_mfma_workspace_bytes(g);
    return XNOR_OK;
}

int xnor_conv2d_fwd_algo(const uint32_t *Ipk, const uint32_t *Wpk, const float *K,
                         const float *alpha, const xnor_shape *s, float *out, int32_t *dot,
                         void *workspace, size_t workspace_bytes, int algo, void *stream)
{
    if (!Ipk || !Wpk || !K || !alpha || !s || !out) return XNOR_E_NULL;
    xnor::Geom g;
    const int rc = make_geom(s, &g);
    if (rc) return rc;
    if (!aligned(Ipk, 4) || !aligned(Wpk, 4) || !aligned(K, 4) || !aligned(alpha, 4) ||
        !aligned(out, 4) || (dot && !aligned(dot, 4)) || (workspace && !aligned(workspace, 16)))
        return XNOR_E_ALIGN;
    if (!workspace) workspace_bytes = 0;
    hipStream_t st = (hipStream_t)stream;
    if (algo == XNOR_ALGO_AUTO) algo = pick_algo(g, workspace_bytes);
    switch (algo) {
        case XNOR_ALGO_DIRECT:
            return hip_status(xnor::launch_conv_direct(Ipk, Wpk, K, alpha, g, out, dot, st));
        case XNOR_ALGO_TILED:
            if (!xnor::conv_tiled_supports(g)) return XNOR_E_UNSUPPORTED;
            return hip_status(xnor::launch_conv_tiled(Ipk, Wpk, K, alpha, g, out, dot, st));
        case XNOR_ALGO_MFMA: {
            const size_t need = xnor::conv_mfma_workspace_bytes(g);
            if (need == 0) return XNOR_E_UNSUPPORTED;
            if (workspace_bytes < need) return XNOR_E_WORKSPACE;
            return hip_status(xnor::launch_conv_mfma(Ipk, Wpk, K, alpha, g, out, dot, workspace, st));
        }
        case XNOR_ALGO_MFMA_BANDS: {
            if (!xnor::conv_mfma_bands_supports(g)) return XNOR_E_UNSUPPORTED;
            if (workspace_bytes < xnor::conv_mfma_workspace_bytes(g)) return XNOR_E_WORKSPACE;
            return hip_status(xnor::launch_conv_mfma_bands(Ipk, Wpk, K, alpha, g, out, dot, workspace, st));
        }
        default:
            return XNOR_E_UNSUPPORTED;
    }
}

int xnor_conv2d_fwd_static(const uint32_t *Ipk, const uint32_t *Wpk, const float *K,
                           const float *alpha, const xnor_shape *s, float *out, int32_t *dot,
                           void *stream)
{
    if (!Ipk || !Wpk || !K || !alpha || !s || !out) return XNOR_E_NULL;
    xnor::Geom g;
    const int rc = make_geom(s, &g);
    if (rc) return rc;
    if (!aligned(Ipk, 4) || !aligned(Wpk, 4) || !aligned(K, 4) || !aligned(alpha, 4) ||
        !aligned(out, 4) || (dot && !aligned(dot, 4)))
        return XNOR_E_ALIGN;
    const size_t need = xnor::conv_mfma_workspace_bytes(g);
    if (need == 0) return XNOR_E_UNSUPPORTED;
    if (need > kStaticScratchBytes) return XNOR_E_WORKSPACE;
    void *ws = nullptr;
    const hipError_t e = static_scratch(&ws);
    if (e != hipSuccess) return hip_status(e);
    // every byte of the shape's filter layout is rewritten by the expansion that launch_conv_mfma
    // starts with, so nothing of the previous call's contents is read
    return hip_status(xnor::launch_conv_mfma(Ipk, Wpk, K, alpha, g, out, dot, ws, (hipStream_t)stream));
}

int xnor_box_filter_K(const float *A, const xnor_shape *s, float *K, void *stream)
{
    if (!A || !s || !K) return XNOR_E_NULL;
    xnor::Geom g;
    const int rc = make_geom(s, &g);
    if (rc) return rc;
    if (!aligned(A, 4) || !aligned(K, 4)) return XNOR_E_ALIGN;
    return hip_status(xnor::launch_box_filter_K(A, g, K, (hipStream_t)stream));
}

int xnor_forward_image_supported(const xnor_shape *s)
{
    if (!s) return XNOR_E_NULL;
    xnor::Geom g;
    const int rc = make_geom(s, &g);
    if (rc) return rc;
    return xnor::conv_image_supports(g) ? 1 : 0;
}

int xnor_forward_image(const float *I, const uint32_t *Wpk, const float *alpha, const xnor_shape *s,
                       float *out, int32_t *dot, void *stream)
{
    if (!I || !Wpk || !alpha || !s || !out) return XNOR_E_NULL;
    xnor::Geom g;
    const int rc = make_geom(s, &g);
    if (rc) return rc;
    if (!aligned(I, 4) || !aligned(Wpk, 4) || !aligned(alpha, 4) || !aligned(out, 4) ||
        (dot && !aligned(dot, 4)))
        return XNOR_E_ALIGN;
    if (!xnor::conv_image_supports(g)) return XNOR_E_UNSUPPORTED;
    return hip_status(xnor::launch_conv_image(I, Wpk, alpha, g, out, dot, (hipStream_t)stream));
}

int xnor_bwn_conv2d_fwd_algo(const float *I, const uint32_t *Wpk, const float *alpha,
                             const xnor_shape *s, float *out, int algo, void *stream)
{
    if (!I || !Wpk || !alpha || !s || !out) return XNOR_E_NULL;
    xnor::Geom g;
    const int rc = make_geom(s, &g);
    if (rc) return rc;
    if (!aligned(I, 4) || !aligned(Wpk, 4) || !aligned(alpha, 4) || !aligned(out, 4)) return XNOR_E_ALIGN;
    if (algo == XNOR_ALGO_AUTO) algo = xnor_bwn_pick_algo(s);
    switch (algo) {
        case XNOR_ALGO_DIRECT:
            return hip_status(xnor::launch_bwn_direct(I, Wpk, alpha, g, out, (hipStream_t)stream));
        case XNOR_ALGO_MFMA_SPLIT:
            if (!xnor::bwn_split_supports(g)) return XNOR_E_UNSUPPORTED;
            return hip_status(xnor::launch_bwn_split(I, Wpk, alpha, g, out, (hipStream_t)stream));
        case XNOR_ALGO_MFMA:
            if (!xnor::bwn_mfma_supports(g)) return XNOR_E_UNSUPPORTED;
            return hip_status(xnor::launch_bwn_mfma(I, Wpk, alpha, g, out, (hipStream_t)stream));
        default:
            return XNOR_E_UNSUPPORTED;
    }
}

int xnor_bwn_pick_algo(const xnor_shape *s)
{
    if (!s) return XNOR_E_NULL;
    xnor::Geom g;
    const int rc = make_geom(s, &g);
    if (rc) return rc;
    return xnor::bwn_split_supports(g) ? XNOR_ALGO_MFMA_SPLIT
           : xnor::bwn_mfma_supports(g) ? XNOR_ALGO_MFMA : XNOR_ALGO_DIRECT;
}

int xnor_bwn_split_plan(const xnor_shape *s, int compute_units, int *tiles, int *row_segments,
                        size_t *lds_bytes, long long *workgroups)
{
    if (!s || !tiles || !row_segments || !lds_bytes || !workgroups) return XNOR_E_NULL;
    if (compute_units < 0) return XNOR_E_SHAPE;
    xnor::Geom g;
    const int rc = make_geom(s, &g);
    if (rc) return rc;
    return xnor::bwn_split_plan(g, compute_units, tiles, row_segments, lds_bytes, workgroups)
               ? XNOR_OK : XNOR_E_UNSUPPORTED;
}

int xnor_bwn_conv2d_fwd(const float *I, const uint32_t *Wpk, const float *alpha, const xnor_shape *s,
                        float *out, void *stream)
{
    return xnor_bwn_conv2d_fwd_algo(I, Wpk, alpha, s, out, XNOR_ALGO_AUTO, stream);
}

int xnor_conv2d_fp32_fwd_algo(const float *I, const float *Wt, const xnor_shape *s, float *out, int algo,
                              void *stream)
{
    if (!I || !Wt || !s || !out) return XNOR_E_NULL;
    xnor::Geom g;
    const int rc = make_geom(s, &g);
    if (rc) return rc;
    if (!aligned(I, 4) || !aligned(Wt, 4) || !aligned(out, 4)) return XNOR_E_ALIGN;
    // (a few channels or filters leave the matrix tiles mostly empty: one thread per output then)
    if (algo == XNOR_ALGO_AUTO)
        algo = (xnor::conv_fp32_mfma_supports(g) && g.F >= 8 && g.C >= 4) ? XNOR_ALGO_MFMA : XNOR_ALGO_DIRECT;
    switch (algo) {
        case XNOR_ALGO_DIRECT:
            return hip_status(xnor::launch_conv_fp32_direct(I, Wt, g, out, (hipStream_t)stream));
        case XNOR_ALGO_MFMA:
            if (!xnor::conv_fp32_mfma_supports(g)) return XNOR_E_UNSUPPORTED;
            return hip_status(xnor::launch_conv_fp32_mfma(I, Wt, g, out, (hipStream_t)stream));
        default:
            return XNOR_E_UNSUPPORTED;
    }
}

int xnor_conv2d_fp32_fwd(const float *I, const float *Wt, const xnor_shape *s, float *out, void *stream)
{
    return xnor_conv2d_fp32_fwd_algo(I, Wt, s, out, XNOR_ALGO_AUTO, stream);
}

int xnor_conv2d_chain_workspace_bytes(const xnor_shape *s, size_t *bytes)
{
    if (!s || !bytes) return XNOR_E_NULL;
    xnor::Geom g;
    const int rc = make_geom(s, &g);
    if (rc) return rc;
    *bytes = xnor::conv_mfma_chain_workspace_bytes(g);
    return XNOR_OK;
}

// (Wpk null: the filters are already expanded in the workspace; exactly one of K, A)
int xnor_conv2d_fwd_chain(const uint32_t *Ipk, const uint32_t *Wpk, const float *K, const float *A,
                          const float *alpha, const xnor_shape *s, uint32_t *Opk, float *A_next,
                          void *workspace, size_t workspace_bytes, void *stream)
{
    if (!Ipk || (!K == !A) || !alpha || !s || !Opk || !A_next || !workspace) return XNOR_E_NULL;
    xnor::Geom g;
    const int rc = make_geom(s, &g);
    if (rc) return rc;
    if (!aligned(Ipk, 4) || (Wpk && !aligned(Wpk, 4)) || (K && !aligned(K, 4)) || (A && !aligned(A, 4)) || !aligned(alpha, 4) || !aligned(Opk, 4) ||
        !aligned(A_next, 4) || !aligned(workspace, 16))
        return XNOR_E_ALIGN;
    const size_t need = xnor::conv_mfma_chain_workspace_bytes(g);
    if (need == 0) return XNOR_E_UNSUPPORTED;
    if (workspace_bytes < need) return XNOR_E_WORKSPACE;
    return hip_status(xnor::launch_conv_mfma_chain(Ipk, Wpk, K, A, alpha, g, Opk, A_next, workspace,
                                                   (hipStream_t)stream));
}

int xnor_filter_expand(const uint32_t *Wpk, const xnor_shape *s, void *workspace,
                       size_t workspace_bytes, void *stream)
{
    if (!Wpk || !s || !workspace) return XNOR_E_NULL;
    xnor::Geom g;
    const int rc = make_geom(s, &g);
    if (rc) return rc;
    if (!aligned(Wpk, 4) || !aligned(workspace, 16)) return XNOR_E_ALIGN;
    const size_t need = xnor::conv_mfma_workspace_bytes(g);
    if (need == 0) return XNOR_E_UNSUPPORTED;
    if (workspace_bytes < need) return XNOR_E_WORKSPACE;
    return hip_status(xnor::launch_expand_filters(Wpk, g, workspace, (hipStream_t)stream));
}

int xnor_conv2d_fwd_expanded(const uint32_t *Ipk, const void *workspace, size_t workspace_bytes,
                             const float *K, const float *A, const float *alpha, const xnor_shape *s,
                             float *out, int32_t *dot, void *stream)
{
    if (!Ipk || !workspace || (!K == !A) || !alpha || !s || !out) return XNOR_E_NULL;   // (exactly one of K, A)
    xnor::Geom g;
    const int rc = make_geom(s, &g);
    if (rc) return rc;
    if (!aligned(Ipk, 4) || (K && !aligned(K, 4)) || (A && !aligned(A, 4)) || !aligned(alpha, 4) || !aligned(out, 4) ||
        (dot && !aligned(dot, 4)) || !aligned(workspace, 16))
        return XNOR_E_ALIGN;
    const size_t need = xnor::conv_mfma_workspace_bytes(g);
    if (need == 0) return XNOR_E_UNSUPPORTED;
    if (workspace_bytes < need) return XNOR_E_WORKSPACE;
    if (K) return hip_status(xnor::launch_conv_mfma_expanded(Ipk, K, alpha, g, out, dot, workspace, (hipStream_t)stream));
    return hip_status(xnor::launch_conv_mfma_expanded_from_A(Ipk, A, alpha, g, out, dot, workspace,
                                                             (hipStream_t)stream));
}

int xnor_conv2d_fwd(const uint32_t *Ipk, const uint32_t *Wpk, const float *K, const float *alpha,
                    const xnor_shape *s, float *out, int32_t *dot, void *workspace,
                    size_t workspace_bytes, void *stream)
{
    return xnor_conv2d_fwd_algo(Ipk, Wpk, K, alpha, s, out, dot, workspace, workspace_bytes,
                                XNOR_ALGO_AUTO, stream);
}

}  // extern "C"
