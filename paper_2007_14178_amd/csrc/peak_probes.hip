// Measurement probes: what this GPU sustains on the three resources the forward pass is priced
// against, so that a roofline fraction can be read against a measured ceiling next to the published
// one.  None of them is part of the forward pass.
//   * probe_mfma_fp4_kernel      register-only loop of the FP4 matrix instruction the convolution
//                                uses (v_mfma_f32_32x32x64_f8f6f4, both operands FP4), eight
//                                independent accumulators per wave, no memory traffic
//   * probe_mfma_bf16_kernel     register-only loop of v_mfma_f32_32x32x16_bf16 (what the
//                                Binary-Weight-Network kernel uses), +-1.0 as the A operand and
//                                either +-1.0 or values with random significands as the B operand:
//                                the rate the chip holds depends on how much the operands toggle
//   * probe_xor_popcount_kernel  register-only loop of v_xor_b32 + v_bcnt_u32_b32 pairs (32 binary
//                                multiply-accumulates per lane and pair), eight independent chains
//   * probe_copy_kernel          plain 16-byte-per-lane device copy
//   * probe_read_kernel          plain 16-byte-per-lane read of a buffer (what a kernel that reads far
//                                more than it writes, like the input pass, can be held against)
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "xnor.h"

namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int kMfmaPerIter = 8;      // two A operands x four B operands
constexpr int kPairsPerIter = 8;

// E2M1 nibbles: 0x2 = +1, 0xA = -1.  Every operand register holds +-1 values with lane-dependent
// signs (the multiplier's inputs toggle as they do in the convolution, not constants).
__global__ __launch_bounds__(256) void probe_mfma_fp4_kernel(int iters, float *sink)
{
    v16f acc[kMfmaPerIter];
    for (int j = 0; j < kMfmaPerIter; ++j)
        for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
    unsigned x = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 12345u;
    v8i A[2], B[4];
    for (int i = 0; i < 2; ++i) {
        A[i] = v8i{0, 0, 0, 0, 0, 0, 0, 0};
        for (int w = 0; w < 4; ++w) { x = x * 1664525u + 1013904223u; A[i][w] = (int)(0x22222222u | (x & 0x88888888u)); }
    }
    for (int i = 0; i < 4; ++i) {
        B[i] = v8i{0, 0, 0, 0, 0, 0, 0, 0};
        for (int w = 0; w < 4; ++w) { x = x * 1664525u + 1013904223u; B[i][w] = (int)(0x22222222u | (x & 0x88888888u)); }
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[i * 4 + j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(
                    A[i], B[j], acc[i * 4 + j], 4, 4, 0, 0x7f7f7f7f, 0, 0x7f7f7f7f);
    }
    float s = 0.f;
    for (int j = 0; j < kMfmaPerIter; ++j)
        for (int r = 0; r < 16; ++r) s += acc[j][r];
    // (sums of +-1 products are integers: the store never happens, but the compiler cannot know)
    if (s == 0.5f) sink[0] = s;
}

typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
constexpr int kBf16PerIter = 6;      // two A operands x three B operands

// A: +-1.0 with lane-dependent signs.  B: the same (random_b = 0), or bf16 values in +-[0.5, 4) with
// random significand bits.
__global__ __launch_bounds__(256) void probe_mfma_bf16_kernel(int iters, int random_b, float *sink)
{
    v16f acc[kBf16PerIter];
    for (int j = 0; j < kBf16PerIter; ++j)
        for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
    unsigned x = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 12345u;
    uint4 A[2], B[3];
    for (int i = 0; i < 2; ++i) {
        uint32_t w[4];
        for (int q = 0; q < 4; ++q) { x = x * 1664525u + 1013904223u; w[q] = 0x3f803f80u ^ (x & 0x80008000u); }
        A[i] = make_uint4(w[0], w[1], w[2], w[3]);
    }
    for (int i = 0; i < 3; ++i) {
        uint32_t w[4];
        for (int q = 0; q < 4; ++q) {
            uint32_t h[2];
            for (int e = 0; e < 2; ++e) {
                x = x * 1664525u + 1013904223u;
                h[e] = random_b ? (((x >> 3) & 0x807fu) | (0x3f00u + ((x >> 20) & 0x180u))) : (0x3f80u | ((x >> 5) & 0x8000u));
            }
            w[q] = h[0] | (h[1] << 16);
        }
        B[i] = make_uint4(w[0], w[1], w[2], w[3]);
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int t = 0; t < 3; ++t)
#pragma unroll
            for (int i = 0; i < 2; ++i)
                acc[t * 2 + i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, A[i]), __builtin_bit_cast(v8bf, B[t]),
                                                                         acc[t * 2 + i], 0, 0, 0);
    }
    float s = 0.f;
    for (int j = 0; j < kBf16PerIter; ++j)
        for (int r = 0; r < 16; ++r) s += acc[j][r];
    if (s == 0.4375f) sink[0] = s;   // (practically never; the compiler cannot know)
}

__global__ __launch_bounds__(256) void probe_xor_popcount_kernel(int iters, uint32_t *sink)
{
    uint32_t acc[kPairsPerIter], a[kPairsPerIter], w[kPairsPerIter];
    uint32_t x = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 977u;
    for (int j = 0; j < kPairsPerIter; ++j) {
        acc[j] = 0;
        x = x * 1664525u + 1013904223u; a[j] = x;
        x = x * 1664525u + 1013904223u; w[j] = x;
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < kPairsPerIter; ++j) {
            uint32_t t;
            asm volatile("v_xor_b32 %0, %2, %3\n\tv_bcnt_u32_b32 %1, %0, %1"
                         : "=&v"(t), "+v"(acc[j])
                         : "v"(a[j]), "v"(w[j]));
        }
    }
    uint32_t s = 0;
    for (int j = 0; j < kPairsPerIter; ++j) s += acc[j];
    if (s == 0xffffffffu) sink[0] = s;   // (a count of at most 32 * iters * 8 per lane: never)
}

__global__ __launch_bounds__(256) void probe_copy_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst,
                                                         long long n16)
{
    const long long stride = (long long)gridDim.x * 256;
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

__global__ __launch_bounds__(256) void probe_read_kernel(const uint4 *__restrict__ src, long long n16, uint32_t *sink)
{
    const long long stride = (long long)gridDim.x * 256;
    uint32_t acc = 0;
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) {
        const uint4 v = src[i];
        acc ^= v.x ^ v.y ^ v.z ^ v.w;
    }
    if (acc == 0x9e3779b9u) sink[0] = acc;   // (practically never; the compiler cannot know)
}

int status(hipError_t e) { return e == hipSuccess ? XNOR_OK : XNOR_E_HIP; }

}  // namespace

// Stores beside a matrix loop.  One workgroup of 8 waves per compute unit, two waves per SIMD:
// waves 0-3 run a register-only loop of the FP4 matrix instruction (LOOP 1: back to back, LOOP 2:
// an s_nop 7 behind every second one, LOOP 0: they exit at once), waves 4-7 each store 32 KB per
// repetition (together the 128 KB of one convolution item) as 32 stores of 16 bytes per lane
// (WIDE) or 128 dword stores, two multiplies per stored value as in the epilogue, and write the
// shader-clock time they took to `cycles`.  The matrix loop is long enough to outlast the stores.
typedef float probe_f4 __attribute__((ext_vector_type(4)));
template <bool WIDE, int LOOP>
__global__ __launch_bounds__(512) void probe_store_beside_mfma_kernel(float *__restrict__ dst, int reps,
                                                                      unsigned long long *__restrict__ cycles,
                                                                      float *__restrict__ sink)
{
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    if (wave < 4) {
        if (LOOP != 0) {
            v16f acc[8];
            for (int j = 0; j < 8; ++j)
                for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
            uint32_t x = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 12345u;
            v8i A[2], B[4];
            for (int i = 0; i < 2; ++i)
                for (int w = 0; w < 8; ++w) { x = x * 1664525u + 1013904223u; A[i][w] = w < 4 ? (int)(0x22222222u | (x & 0x88888888u)) : 0; }
            for (int i = 0; i < 4; ++i)
                for (int w = 0; w < 8; ++w) { x = x * 1664525u + 1013904223u; B[i][w] = w < 4 ? (int)(0x22222222u | (x & 0x88888888u)) : 0; }
            for (int it = 0; it < reps * 160; ++it) {
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    acc[j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(A[j & 1], B[j & 3], acc[j], 4, 4, 0, 0x7f7f7f7f, 0,
                                                                             0x7f7f7f7f);
                    if (LOOP == 2 && (j & 1)) asm volatile("s_nop 7");
                }
            }
            float s = 0.f;
            for (int j = 0; j < 8; ++j)
                for (int r = 0; r < 16; ++r) s += acc[j][r];
            if (s == 0.5f) sink[0] = s;
        }
        return;
    }
    float *base = dst + (long long)blockIdx.x * reps * 32768 + (wave - 4) * 8192;
    probe_f4 v = {(float)lane, 1.f, 2.f, 3.f};
    const float m = 1.0f + lane * 1e-6f;
    const unsigned long long t0 = __builtin_readcyclecounter();
    for (int r = 0; r < reps; ++r) {
        float *p = base + (long long)r * 32768;
        if (WIDE) {
#pragma unroll 8
            for (int i = 0; i < 32; ++i) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    asm volatile("v_mul_f32 %0, %0, %1" : "+v"(v[q]) : "v"(m));
                    asm volatile("v_mul_f32 %0, %0, %1" : "+v"(v[q]) : "v"(m));
                }
                *reinterpret_cast<probe_f4 *>(p + i * 256 + lane * 4) = v;
            }
        } else {
#pragma unroll 16
            for (int i = 0; i < 128; ++i) {
                asm volatile("v_mul_f32 %0, %0, %1" : "+v"(v[0]) : "v"(m));
                asm volatile("v_mul_f32 %0, %0, %1" : "+v"(v[1]) : "v"(m));
                p[i * 64 + lane] = v[0];
            }
        }
    }
    asm volatile("s_waitcnt vmcnt(0)");
    const unsigned long long t1 = __builtin_readcyclecounter();
    if (lane == 0) cycles[blockIdx.x * 4 + (wave - 4)] = t1 - t0;
    if (v[0] + v[1] + v[2] + v[3] == 0.123f) sink[1] = v[0];
}

extern "C" {

int xnor_probe_mfma_fp4(int workgroups, int iters, float *sink, double *flops, void *stream)
{
    if (!sink || !flops) return XNOR_E_NULL;
    if (workgroups <= 0 || iters <= 0 || workgroups > (1 << 20) || iters > (1 << 24)) return XNOR_E_SHAPE;
    probe_mfma_fp4_kernel<<<dim3(workgroups), dim3(256), 0, (hipStream_t)stream>>>(iters, sink);
    // 4 waves per workgroup, 32 x 32 x 64 multiply-accumulates per instruction, 2 flops each
    *flops = (double)workgroups * 4.0 * iters * kMfmaPerIter * (32.0 * 32.0 * 64.0) * 2.0;
    return status(hipGetLastError());
}

int xnor_probe_mfma_bf16(int workgroups, int iters, int random_b, float *sink, double *flops, void *stream)
{
    if (!sink || !flops) return XNOR_E_NULL;
    if (workgroups <= 0 || iters <= 0 || workgroups > (1 << 20) || iters > (1 << 24)) return XNOR_E_SHAPE;
    probe_mfma_bf16_kernel<<<dim3(workgroups), dim3(256), 0, (hipStream_t)stream>>>(iters, random_b != 0, sink);
    // 4 waves per workgroup, 32 x 32 x 16 multiply-accumulates per instruction, 2 flops each
    *flops = (double)workgroups * 4.0 * iters * kBf16PerIter * (32.0 * 32.0 * 16.0) * 2.0;
    return status(hipGetLastError());
}

int xnor_probe_xor_popcount(int workgroups, int iters, uint32_t *sink, double *binary_macs, void *stream)
{
    if (!sink || !binary_macs) return XNOR_E_NULL;
    if (workgroups <= 0 || iters <= 0 || workgroups > (1 << 20) || iters > (1 << 24)) return XNOR_E_SHAPE;
    probe_xor_popcount_kernel<<<dim3(workgroups), dim3(256), 0, (hipStream_t)stream>>>(iters, sink);
    *binary_macs = (double)workgroups * 256.0 * iters * kPairsPerIter * 32.0;
    return status(hipGetLastError());
}

int xnor_probe_copy(const void *src, void *dst, size_t bytes, void *stream)
{
    if (!src || !dst) return XNOR_E_NULL;
    if (bytes == 0 || bytes % 16 != 0) return XNOR_E_SHAPE;
    if (((uintptr_t)src | (uintptr_t)dst) & 15) return XNOR_E_ALIGN;
    const long long n16 = (long long)(bytes / 16);
    const long long want = (n16 + 255) / 256;
    const int grid = (int)(want < 256 * 32 ? want : 256 * 32);   // up to 32 workgroups per compute unit, grid-stride beyond
    probe_copy_kernel<<<dim3(grid), dim3(256), 0, (hipStream_t)stream>>>(static_cast<const uint4 *>(src),
                                                                           static_cast<uint4 *>(dst), n16);
    return status(hipGetLastError());
}

int xnor_probe_read(const void *src, size_t bytes, uint32_t *sink, void *stream)
{
    if (!src || !sink) return XNOR_E_NULL;
    if (bytes == 0 || bytes % 16 != 0) return XNOR_E_SHAPE;
    if ((uintptr_t)src & 15) return XNOR_E_ALIGN;
    const long long n16 = (long long)(bytes / 16);
    const long long want = (n16 + 255) / 256;
    const int grid = (int)(want < 256 * 32 ? want : 256 * 32);
    probe_read_kernel<<<dim3(grid), dim3(256), 0, (hipStream_t)stream>>>(static_cast<const uint4 *>(src), n16, sink);
    return status(hipGetLastError());
}

int xnor_probe_store_beside_mfma(int workgroups, int reps, int wide, int matrix_loop, float *dst, size_t dst_bytes,
                                 unsigned long long *cycles, float *sink, void *stream)
{
    if (!dst || !cycles || !sink) return XNOR_E_NULL;
    if (workgroups <= 0 || workgroups > 4096 || reps <= 0 || reps > 64 || matrix_loop < 0 || matrix_loop > 2)
        return XNOR_E_SHAPE;
    if (dst_bytes < (size_t)workgroups * reps * 131072) return XNOR_E_SHAPE;
    if (((uintptr_t)dst & 15) || ((uintptr_t)cycles & 7)) return XNOR_E_ALIGN;
    hipStream_t st = (hipStream_t)stream;
    const dim3 grid(workgroups), block(512);
#define XNOR_PROBE_SBM(W, L) probe_store_beside_mfma_kernel<W, L><<<grid, block, 0, st>>>(dst, reps, cycles, sink)
    if (wide) {
        if (matrix_loop == 0) XNOR_PROBE_SBM(true, 0);
        else if (matrix_loop == 1) XNOR_PROBE_SBM(true, 1);
        else XNOR_PROBE_SBM(true, 2);
    } else {
        if (matrix_loop == 0) XNOR_PROBE_SBM(false, 0);
        else if (matrix_loop == 1) XNOR_PROBE_SBM(false, 1);
        else XNOR_PROBE_SBM(false, 2);
    }
#undef XNOR_PROBE_SBM
    return status(hipGetLastError());
}

}  // extern "C"
