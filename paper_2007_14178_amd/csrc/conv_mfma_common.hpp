// Shared by the two matrix-core convolution kernels (Sec. III-A steps 1b-1d and 3, Eq. 11 on
// v_mfma_f32_32x32x64_f8f6f4): tile constants, the exact-division helper, load-width types.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "fp4_expand.hpp"
#include "xnor_internal.hpp"

namespace xnor {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int kWM = 2;            // 32-filter tiles per wave
constexpr int kWN = 4;            // 32-pixel tiles per wave (at most)
constexpr int kBandPixels = 2 * 32 * kWN;   // 2 wave columns
constexpr int kFilterTile = 2 * 32 * kWM;   // 2 wave rows
constexpr int kRing = 4;          // register ring of filter operands: loads run kRing-1 steps ahead
constexpr int kXcdShift = 3, kXcds = 1 << kXcdShift;   // MI355X: 8 XCDs of 32 CUs

// q = n / d for n*d < 2^32 via one mul_hi.
struct FastDiv {
    uint32_t mul, d;
};
inline FastDiv make_fastdiv(uint32_t d) { return FastDiv{d == 1 ? 0u : (uint32_t)(((1ull << 32) + d - 1) / d), d}; }
__device__ inline uint32_t fdiv(uint32_t n, FastDiv f) { return f.d == 1 ? n : __umulhi(n, f.mul); }

template <int VW>
struct WordVec;
template <>
struct WordVec<1> { typedef uint32_t type; };
template <>
struct WordVec<2> { typedef uint32_t type __attribute__((ext_vector_type(2))); };
template <>
struct WordVec<4> { typedef uint32_t type __attribute__((ext_vector_type(4))); };

constexpr size_t kKAlphaBytes = (kBandPixels + kFilterTile) * sizeof(float);
constexpr size_t kLdsTwoPerCU = 80 * 1024;
constexpr size_t kLdsMax = 160 * 1024;

// The persistent form of the kernel (conv_mfma_persistent.hip); conv_mfma.hip's launchers hand a
// layer to it where it takes the shape.  `P` of the chained form holds
// conv_mfma_persistent_sum_parts() partial sums per pixel.
bool conv_mfma_persistent_supports(const Geom &g);
bool conv_mfma_persistent_preferred(const Geom &g);   // ... and is expected to be the faster kernel
ExpandLayout conv_mfma_persistent_expand_layout(const Geom &g);
int conv_mfma_persistent_sum_parts(const Geom &g);
hipError_t launch_conv_mfma_persistent(const uint32_t *Ipk, const float *K, const float *A, const float *alpha,
                                       const Geom &g, float *out, int32_t *dot, uint32_t *Opk, float *P,
                                       const void *workspace, hipStream_t st);

}  // namespace xnor
