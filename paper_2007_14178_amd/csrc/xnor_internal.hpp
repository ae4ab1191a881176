// Internal declarations shared by the library's translation units (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "xnor.h"
#include "fp4_expand.hpp"

namespace xnor {

// Derived geometry, computed once on the host after validation.
struct Geom {
    int N, C, H, W, F, kh, kw, sh, sw, ph, pw;
    int OH, OW, Cw;
};

inline int ceil_div(long long a, long long b) { return (int)((a + b - 1) / b); }

// Launchers: enqueue on `st`, return the launch status.  Arguments are already validated.
hipError_t launch_binarize_pack(const float *x, int N, int C, int H, int W, uint32_t *packed,
                                hipStream_t st);
hipError_t launch_channel_mean_abs(const float *I, int N, int C, int H, int W, float *A,
                                   hipStream_t st);
bool pack_and_mean_supports(int C);
hipError_t launch_pack_and_mean(const float *x, int N, int C, int H, int W, uint32_t *packed,
                                float *A, hipStream_t st);
bool filter_pack_mean_supports(int taps);
hipError_t launch_filter_pack_mean(const float *Wt, int F, int C, int taps, uint32_t *Wpk, float *M,
                                   float *alpha, hipStream_t st);
bool prepare_both_supports(const float *x, int N, int C, int H, int W, int taps);
bool prepare_both_can_expand(int C, int taps);
hipError_t launch_prepare_both(const float *x, int N, int C, int H, int W, uint32_t *packed, float *A,
                               const float *Wt, int F, int taps, uint32_t *Wpk, float *M, float *alpha,
                               void *Wx, const ExpandLayout &L, hipStream_t st);
hipError_t launch_alpha_from_tap_means(const float *M, int F, int taps, float *alpha, hipStream_t st);
hipError_t launch_box_filter_K(const float *A, const Geom &g, float *K, hipStream_t st);
hipError_t launch_alpha(const float *Wt, int F, long long n_red, float *alpha, hipStream_t st);

hipError_t launch_conv_direct(const uint32_t *Ipk, const uint32_t *Wpk, const float *K,
                              const float *alpha, const Geom &g, float *out, int32_t *dot,
                              hipStream_t st);

bool conv_tiled_supports(const Geom &g);
hipError_t launch_conv_tiled(const uint32_t *Ipk, const uint32_t *Wpk, const float *K,
                             const float *alpha, const Geom &g, float *out, int32_t *dot,
                             hipStream_t st);

bool conv_image_supports(const Geom &g);
hipError_t launch_conv_image(const float *I, const uint32_t *Wpk, const float *alpha, const Geom &g,
                             float *out, int32_t *dot, hipStream_t st);

bool bwn_mfma_supports(const Geom &g);
bool bwn_split_supports(const Geom &g);
bool bwn_split_plan(const Geom &g, int compute_units, int *tiles, int *row_segments, size_t *lds_bytes,
                    long long *workgroups);
hipError_t launch_bwn_split(const float *I, const uint32_t *Wpk, const float *alpha, const Geom &g,
                            float *out, hipStream_t st);
bool conv_fp32_mfma_supports(const Geom &g);
hipError_t launch_conv_fp32_mfma(const float *I, const float *Wt, const Geom &g, float *out, hipStream_t st);
hipError_t launch_conv_fp32_direct(const float *I, const float *Wt, const Geom &g, float *out, hipStream_t st);
hipError_t launch_bwn_mfma(const float *I, const uint32_t *Wpk, const float *alpha, const Geom &g,
                           float *out, hipStream_t st);
hipError_t launch_bwn_direct(const float *I, const uint32_t *Wpk, const float *alpha, const Geom &g,
                             float *out, hipStream_t st);

bool conv_mfma_supports(const Geom &g);
size_t conv_mfma_workspace_bytes(const Geom &g);   // 0 if the shape is not supported
ExpandLayout conv_mfma_expand_layout(const Geom &g);
hipError_t launch_expand_filters(const uint32_t *Wpk, const Geom &g, void *workspace, hipStream_t st);
hipError_t launch_conv_mfma_expanded(const uint32_t *Ipk, const float *K, const float *alpha,
                                     const Geom &g, float *out, int32_t *dot, const void *workspace,
                                     hipStream_t st);
hipError_t launch_conv_mfma_expanded_from_A(const uint32_t *Ipk, const float *A, const float *alpha,
                                            const Geom &g, float *out, int32_t *dot,
                                            const void *workspace, hipStream_t st);
size_t conv_mfma_chain_workspace_bytes(const Geom &g);   // 0 if the shape is not supported
hipError_t launch_conv_mfma_chain(const uint32_t *Ipk, const uint32_t *Wpk, const float *K, const float *A,
                                  const float *alpha, const Geom &g, uint32_t *Opk, float *A_next,
                                  void *workspace, hipStream_t st);   // exactly one of K, A is given
hipError_t launch_conv_mfma(const uint32_t *Ipk, const uint32_t *Wpk, const float *K,
                            const float *alpha, const Geom &g, float *out, int32_t *dot,
                            void *workspace, hipStream_t st);
bool conv_mfma_bands_supports(const Geom &g);
hipError_t launch_conv_mfma_bands(const uint32_t *Ipk, const uint32_t *Wpk, const float *K,
                                  const float *alpha, const Geom &g, float *out, int32_t *dot,
                                  void *workspace, hipStream_t st);

}  // namespace xnor
