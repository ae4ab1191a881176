// HBM-streaming stages of the binary-convolution pipeline (Sec. III-A step list):
//   step 1a  sign-binarise + channel bit-pack          (Eq. 3 / Eq. 8)
//   step 2a  channel mean of |I| and its box filter K  (Eq. 10)
//            per-filter alpha = mean |W|               (Eq. 5)
// All three read fp32 once and write far less than they read, so each is laid out for coalesced
// 256-byte wavefront reads along the image's fastest axis with many loads in flight per lane.
#include <algorithm>
#include <atomic>

#include "xnor_internal.hpp"

namespace xnor {

// ------------------------------------------------------------------------------------------------
// Step 1a.  One lane owns one pixel and builds WPT packed words from 32*WPT channel planes; the 64
// lanes of a wave read 64 consecutive pixels of one plane (256 contiguous bytes) per load.
// The paper sets bits one by one in a register per spatial tile (Alg. 1); packing along channels
// instead gives every bit of every word a use in the convolution.
// ------------------------------------------------------------------------------------------------
template <int WPT>
__global__ __launch_bounds__(256) void binarize_pack_kernel(const float *__restrict__ x,
                                                            long long NP, int C, int HW, int Cw,
                                                            uint32_t *__restrict__ packed)
{
    const long long p = (long long)blockIdx.x * 256 + threadIdx.x;
    const int w0 = blockIdx.y * WPT;
    if (p >= NP) return;
    const long long n = p / HW;
    const int hw = (int)(p - n * HW);
    const float *src = x + (n * C) * (long long)HW + hw;

    uint32_t words[WPT];
#pragma unroll
    for (int k = 0; k < WPT; ++k) {
        const int cbase = 32 * (w0 + k);
        uint32_t word = 0;
        if (cbase + 32 <= C) {
            float v[32];
#pragma unroll
            for (int j = 0; j < 32; ++j) v[j] = __builtin_nontemporal_load(src + (long long)(cbase + j) * HW);
#pragma unroll
            for (int j = 0; j < 32; ++j) word |= (v[j] >= 0.0f ? 1u : 0u) << j;
        } else {
            for (int j = 0; j < 32 && cbase + j < C; ++j)
                word |= (src[(long long)(cbase + j) * HW] >= 0.0f ? 1u : 0u) << j;
        }
        words[k] = word;
    }
    uint32_t *dst = packed + p * Cw + w0;
    if (WPT == 4 && (Cw & 3) == 0) {
        *reinterpret_cast<uint4 *>(dst) = make_uint4(words[0], words[1], words[2], words[3]);
    } else {
#pragma unroll
        for (int k = 0; k < WPT; ++k)
            if (w0 + k < Cw) dst[k] = words[k];
    }
}

hipError_t launch_binarize_pack(const float *x, int N, int C, int H, int W, uint32_t *packed,
                                hipStream_t st)
{
    const int HW = H * W, Cw = (C + 31) / 32;
    const long long NP = (long long)N * HW;
    const bool vec4 = (Cw % 4 == 0) && ((reinterpret_cast<uintptr_t>(packed) & 15) == 0);
    if (vec4) {
        dim3 grid(ceil_div(NP, 256), Cw / 4);
        binarize_pack_kernel<4><<<grid, 256, 0, st>>>(x, NP, C, HW, Cw, packed);
    } else {
        dim3 grid(ceil_div(NP, 256), Cw);
        binarize_pack_kernel<1><<<grid, 256, 0, st>>>(x, NP, C, HW, Cw, packed);
    }
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Eq. 10, first half: A = (1/C) sum_c |I_c|.  A block is 64 pixels x S channel slices; each thread
// adds its slice in double, the slices are combined through LDS in a fixed order (deterministic,
// and the double accumulation keeps A within one rounding of the exact mean).
// The paper uses one thread per pixel over all channels; slicing the channels keeps enough loads
// in flight to stream HBM when N*H*W alone gives too few waves.
// ------------------------------------------------------------------------------------------------
constexpr int kMaxSlices = 16;

__global__ __launch_bounds__(64 * kMaxSlices) void channel_mean_abs_kernel(
    const float *__restrict__ I, long long NP, int C, int HW, int chunk, float *__restrict__ A)
{
    __shared__ double part[kMaxSlices][64];
    const int lane = threadIdx.x, s = threadIdx.y, S = blockDim.y;
    const long long p = (long long)blockIdx.x * 64 + lane;
    double acc = 0.0;
    if (p < NP) {
        const long long n = p / HW;
        const int hw = (int)(p - n * HW);
        const float *src = I + (n * C) * (long long)HW + hw;
        const int c0 = s * chunk;
        const int c1 = min(C, c0 + chunk);
        int c = c0;
        for (; c + 8 <= c1; c += 8) {
            float v[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = __builtin_nontemporal_load(src + (long long)(c + j) * HW);
#pragma unroll
            for (int j = 0; j < 8; ++j) acc += (double)fabsf(v[j]);
        }
        for (; c < c1; ++c) acc += (double)fabsf(src[(long long)c * HW]);
    }
    part[s][lane] = acc;
    __syncthreads();
    if (s == 0 && p < NP) {
        double sum = part[0][lane];
        for (int k = 1; k < S; ++k) sum += part[k][lane];
        A[p] = (float)(sum / (double)C);
    }
}

hipError_t launch_channel_mean_abs(const float *I, int N, int C, int H, int W, float *A,
                                   hipStream_t st)
{
    const int HW = H * W;
    const long long NP = (long long)N * HW;
    int S = 1;
    while (S < kMaxSlices && C / (2 * S) >= 8) S *= 2;
    const int chunk = (C + S - 1) / S;
    channel_mean_abs_kernel<<<dim3(ceil_div(NP, 64)), dim3(64, S), 0, st>>>(I, NP, C, HW, chunk, A);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Step 1a and the first half of Eq. 10 in ONE pass over the fp32 tensor: every element is read
// once, its sign goes into the packed word and its magnitude into the channel sum.  (The paper runs
// the two as separate kernels on two streams; on an HBM-bound pre-stage the second read is the cost.)
// Block = 64 pixels x S slices; slice s owns packed words s, s+S, ...  The words are collected in
// LDS and written out as one contiguous run of 64*Cw words; the slices' partial |x| sums (double)
// are combined in a fixed order.
// ------------------------------------------------------------------------------------------------
// Up to 4 slices: measured equal to 8 and faster than 16 (a 1024-thread block leaves one block per
// CU and nothing to overlap its final barrier and write-out with).
constexpr int kPackMeanSlices = 4;

__device__ __attribute__((always_inline)) void pack_and_mean_block(
    const float *__restrict__ x, long long NP, int C, int HW, int Cw, int Cwp,
    uint32_t *__restrict__ packed, float *__restrict__ A, long long block, double *pm_smem)
{
    const int lane = threadIdx.x, s = threadIdx.y, S = blockDim.y;
    double *part = pm_smem;                                              // [S][64]
    uint32_t *words = reinterpret_cast<uint32_t *>(pm_smem + S * 64);    // [64][Cwp], Cwp odd
    const long long p0 = block * 64;
    const long long p = p0 + lane;
    double acc = 0.0;
    if (p < NP) {
        const long long n = p / HW;
        const int hw = (int)(p - n * HW);
        const float *src = x + (n * C) * (long long)HW + hw;
        for (int w = s; w < Cw; w += S) {
            const int cbase = 32 * w;
            uint32_t word = 0;
            if (cbase + 32 <= C) {
                float v[32];
#pragma unroll
                for (int j = 0; j < 32; ++j) v[j] = __builtin_nontemporal_load(src + (long long)(cbase + j) * HW);
                // from the highest channel down, each bit shifted in at the bottom: one compare (0 <= x:
                // true for +0.0 and -0.0, false for NaN) and one add-with-carry (word + word + bit)
#pragma unroll
                for (int j = 31; j >= 0; --j) {
                    asm("v_cmp_le_f32 vcc, 0, %1\n\tv_addc_co_u32 %0, vcc, %0, %0, vcc" : "+v"(word) : "v"(v[j]) : "vcc");
                    acc += (double)fabsf(v[j]);
                }
            } else {
                for (int j = 0; j < 32 && cbase + j < C; ++j) {
                    const float v = src[(long long)(cbase + j) * HW];
                    word |= (v >= 0.0f ? 1u : 0u) << j;
                    acc += (double)fabsf(v);
                }
            }
            words[lane * Cwp + w] = word;
        }
    }
    part[s * 64 + lane] = acc;
    __syncthreads();
    if (s == 0 && p < NP) {
        double sum = part[lane];
        for (int k = 1; k < S; ++k) sum += part[k * 64 + lane];
        A[p] = (float)(sum / (double)C);
    }
    const int npx = (int)min((long long)64, NP - p0);
    const int nwords = npx * Cw;
    uint32_t *dst = packed + p0 * Cw;
    for (int i = s * 64 + lane; i < nwords; i += 64 * S) {
        const int px = i / Cw, w = i - px * Cw;
        dst[i] = words[px * Cwp + w];
    }
}

__global__ __launch_bounds__(64 * kPackMeanSlices) void pack_and_mean_kernel(
    const float *__restrict__ x, long long NP, int C, int HW, int Cw, int Cwp,
    uint32_t *__restrict__ packed, float *__restrict__ A)
{
    extern __shared__ double pm_smem[];
    pack_and_mean_block(x, NP, C, HW, Cw, Cwp, packed, A, blockIdx.x, pm_smem);
}

// The same pass with four consecutive pixels per lane (one 16-byte load per lane and channel, 1 KB
// contiguous per wave and load instruction): measured 6.7 TB/s for this access pattern against
// 5.5 TB/s with one pixel per lane.  Needs H*W to be a multiple of 4 (so that a lane's four pixels
// share an image) and 16-byte aligned x and A.  Block = 256 pixels x S slices.
typedef float floatx4 __attribute__((ext_vector_type(4)));
constexpr int kPack4Slices = 8;
constexpr int kPack4Batch = 8;      // channels whose loads are in flight together

__device__ __attribute__((always_inline)) void pack_and_mean4_block(
    const float *__restrict__ x, long long NP, int C, int HW, int Cw, int Cwp,
    uint32_t *__restrict__ packed, float *__restrict__ A, long long block, int ppb, double *pm_smem)
{
    // `ppb`: pixels per block, a multiple of 4 up to 256 (lanes beyond it idle): the host picks it so
    // that the blocks share out evenly over the compute units
    const int lane = threadIdx.x, s = threadIdx.y, S = blockDim.y;
    double *part = pm_smem;                                               // [S][4][64]
    uint32_t *words = reinterpret_cast<uint32_t *>(pm_smem + S * 256);    // [4][64][Cwp], Cwp odd
    const long long p0 = block * ppb;
    const long long p = p0 + 4 * lane;
    const bool mine = 4 * lane < ppb && p < NP;
    double acc[4] = {0.0, 0.0, 0.0, 0.0};
    if (mine) {
        const long long n = p / HW;
        const int hw = (int)(p - n * HW);
        const float *src = x + (n * C) * (long long)HW + hw;
        // batches of kPack4Batch channels; the next batch's loads are issued before the current
        // batch's values are used, so that a wave always has loads in flight
        auto fetch = [&](int w, int b, float4 (&v)[kPack4Batch]) __attribute__((always_inline)) {
#pragma unroll
            for (int j = 0; j < kPack4Batch; ++j) {
                const int c = 32 * w + b + j;
                if (w < Cw && c < C) {
                    const floatx4 t = __builtin_nontemporal_load(
                        reinterpret_cast<const floatx4 *>(src + (long long)c * HW));
                    v[j] = make_float4(t[0], t[1], t[2], t[3]);
                } else {
                    v[j] = make_float4(-1.f, -1.f, -1.f, -1.f);                     // tail channels: bit 0
                }
            }
        };
        float4 cur[kPack4Batch], nxt[kPack4Batch];
        // A word's channels are taken from the last batch down to the first and, within a batch, from
        // the last channel down: the word is built by shifting the next lower channel's bit in at the
        // bottom, which is one compare (0 <= x: true for +0.0 and -0.0, false for NaN) and one
        // add-with-carry (word + word + bit) per value instead of compare, select and shift-or.
        constexpr int kLastBatch = 32 - kPack4Batch;
        fetch(s, kLastBatch, cur);
        for (int w = s; w < Cw; w += S) {
            uint32_t word[4] = {0u, 0u, 0u, 0u};
            const int cbase = 32 * w;
            const bool whole = cbase + 32 <= C;               // (uniform) no tail channels in this word
#pragma unroll
            for (int b = kLastBatch; b >= 0; b -= kPack4Batch) {
                if (b > 0) fetch(w, b - kPack4Batch, nxt);
                else fetch(w + S, kLastBatch, nxt);
#pragma unroll
                for (int j = kPack4Batch - 1; j >= 0; --j) {
                    const float e[4] = {cur[j].x, cur[j].y, cur[j].z, cur[j].w};
                    if (whole) {
#pragma unroll
                        for (int k = 0; k < 4; ++k) {
                            asm("v_cmp_le_f32 vcc, 0, %1\n\tv_addc_co_u32 %0, vcc, %0, %0, vcc"
                                : "+v"(word[k]) : "v"(e[k]) : "vcc");
                            acc[k] += (double)fabsf(e[k]);
                        }
                    } else {
                        const bool live = cbase + b + j < C;  // (tail channels were fetched as -1: bit 0)
#pragma unroll
                        for (int k = 0; k < 4; ++k) {
                            word[k] = (word[k] << 1) | (e[k] >= 0.0f ? 1u : 0u);
                            acc[k] += live ? (double)fabsf(e[k]) : 0.0;
                        }
                    }
                }
#pragma unroll
                for (int j = 0; j < kPack4Batch; ++j) cur[j] = nxt[j];
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) words[(k * 64 + lane) * Cwp + w] = word[k];
        }
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) part[(s * 4 + k) * 64 + lane] = acc[k];
    __syncthreads();
    // pixel 4*lane + k: slice k % S adds up the slices' sums (fixed order) when S >= 4
    for (int k = s; k < 4; k += S) {
        if (mine && p + k < NP) {
            double sum = part[k * 64 + lane];
            for (int t = 1; t < S; ++t) sum += part[(t * 4 + k) * 64 + lane];
            A[p + k] = (float)(sum / (double)C);
        }
    }
    const int npx = (int)min((long long)ppb, NP - p0);
    const int nwords = npx * Cw;
    uint32_t *dst = packed + p0 * Cw;
    for (int i = s * 64 + lane; i < nwords; i += 64 * S) {
        const int px = i / Cw, w = i - px * Cw;
        dst[i] = words[((px & 3) * 64 + (px >> 2)) * Cwp + w];
    }
}

__global__ __launch_bounds__(64 * kPack4Slices) void pack_and_mean4_kernel(
    const float *__restrict__ x, long long NP, int C, int HW, int Cw, int Cwp,
    uint32_t *__restrict__ packed, float *__restrict__ A, int ppb)
{
    extern __shared__ double pm_smem[];
    pack_and_mean4_block(x, NP, C, HW, Cw, Cwp, packed, A, blockIdx.x, ppb, pm_smem);
}

// Pixels per block of the four-pixel pass.  A compute unit pulls from HBM at a rate of its own
// (outstanding misses, not lanes, are what it runs out of: measured, a second block on the same unit
// halves the first one's rate), so a launch is as long as its busiest unit: the pixels are shared out
// as equal blocks over a multiple of the units instead of as 256-pixel blocks that leave the last
// round partly empty.
// `filter_blocks`: short blocks launched behind the input blocks in the same grid (the one-launch
// prepare): where the last round of 256-pixel blocks leaves enough units idle for them (a filter
// block takes about a fifth of an input block's time), that layout is the better one: the filter
// side then costs nothing (measured at 128 images of 28 x 28, 392 + 512 blocks: the step 2.4 us
// shorter than with 512 equal input blocks and the filter blocks after them).
static int pixels_per_block4(long long NP, int filter_blocks = 0)
{
    static std::atomic<int> cus_cached{0};
    int cus = cus_cached.load(std::memory_order_relaxed);
    if (cus <= 0) {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
            cus = 256;
        cus_cached.store(cus, std::memory_order_relaxed);
    }
    if (filter_blocks > 0) {
        const long long rem = ((NP + 255) / 256) % cus, idle = rem ? cus - rem : 0;
        if (idle > 0 && filter_blocks <= 5 * idle) return 256;
    }
    const long long quads = (NP + 3) / 4;
    for (long long k = 1;; ++k) {
        const long long per = (quads + cus * k - 1) / (cus * k);
        if (per <= 64) return (int)std::max<long long>(per, 16) * 4;   // (at least a quarter of the lanes busy)
    }
}

bool pack_and_mean_supports(int C) { return (C + 31) / 32 <= 512; }

hipError_t launch_pack_and_mean(const float *x, int N, int C, int H, int W, uint32_t *packed,
                                float *A, hipStream_t st)
{
    const int HW = H * W, Cw = (C + 31) / 32, Cwp = Cw | 1;
    const long long NP = (long long)N * HW;
    if (HW % 4 == 0 && ((uintptr_t)x & 15) == 0 && NP >= 256 * 256) {
        int S4 = 1;
        while (S4 < kPack4Slices && 2 * S4 <= Cw) S4 *= 2;
        const size_t smem4 = (size_t)S4 * 256 * sizeof(double) + (size_t)256 * Cwp * sizeof(uint32_t);
        if (smem4 <= 64 * 1024) {
            const int ppb = pixels_per_block4(NP);
            pack_and_mean4_kernel<<<dim3(ceil_div(NP, ppb)), dim3(64, S4), smem4, st>>>(x, NP, C, HW, Cw,
                                                                                      Cwp, packed, A, ppb);
            return hipGetLastError();
        }
    }
    int S = 1;
    while (S < kPackMeanSlices && 2 * S <= Cw) S *= 2;
    const size_t smem = (size_t)S * 64 * sizeof(double) + (size_t)64 * Cwp * sizeof(uint32_t);
    pack_and_mean_kernel<<<dim3(ceil_div(NP, 64)), dim3(64, S), smem, st>>>(x, NP, C, HW, Cw, Cwp,
                                                                           packed, A);
    return hipGetLastError();
}

// Eq. 5 from per-tap channel means: alpha[f] = mean over the kh*kw taps of M[f][tap], where
// M = mean_c |Wt| is what pack_and_mean_kernel leaves in its A output when run on the filters.
__global__ __launch_bounds__(256) void alpha_from_tap_means_kernel(const float *__restrict__ M,
                                                                   int F, int taps,
                                                                   float *__restrict__ alpha)
{
    const int f = blockIdx.x * 256 + threadIdx.x;
    if (f >= F) return;
    double sum = 0.0;
    for (int t = 0; t < taps; ++t) sum += (double)M[(long long)f * taps + t];
    alpha[f] = (float)(sum / (double)taps);
}

hipError_t launch_alpha_from_tap_means(const float *M, int F, int taps, float *alpha, hipStream_t st)
{
    alpha_from_tap_means_kernel<<<ceil_div(F, 256), 256, 0, st>>>(M, F, taps, alpha);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Filters: step 1a (Eq. 3) and Eq. 5 in one pass, one workgroup per filter.  A filter's C*kh*kw
// floats are contiguous, so the workgroup reads them as one coalesced run into LDS (a chunk of CH
// channels at a time, CH a multiple of 32), then one thread per (tap, channel word) gathers its 32
// channel values from LDS (consecutive threads = consecutive taps = consecutive LDS words), builds
// the word and the |w| sum of its 32 channels.  Sums are combined in double in a fixed order:
// M[f][tap] = mean_c |Wt[f][c][tap]|, alpha[f] = mean over everything.
// ------------------------------------------------------------------------------------------------
constexpr int kFilterStageFloats = 8192;   // 32 KB of LDS for the staged chunk

__device__ __attribute__((always_inline)) void filter_pack_mean_block(
    const float *__restrict__ Wt, int C, int taps, int Cw, int CH, uint32_t *__restrict__ Wpk,
    float *__restrict__ M, float *__restrict__ alpha, int f, int tid, int nthr, double *fp_smem,
    uint4 *__restrict__ Wx = nullptr, ExpandLayout L = ExpandLayout{}, int F = 0)
{
    // With Wx the block also writes its filter's rows of the matrix-core kernel's expanded
    // workspace (what xnor_filter_expand would make of Wpk): the packed words are kept in LDS
    // ([taps][Cw] behind the staging area) and expanded once the filter is complete.
    const int WH = CH / 32;                                        // channel words per chunk
    double *part = fp_smem;                                         // [WH][taps]
    float *stage = reinterpret_cast<float *>(fp_smem + WH * taps);  // [CH][taps]
    uint32_t *kept = reinterpret_cast<uint32_t *>(stage + (size_t)CH * taps);   // [taps][Cw], only with Wx
    const float *src = Wt + (long long)f * C * taps;
    uint32_t *dst = Wpk + (long long)f * taps * Cw;
    double tap_total = 0.0;                                         // thread t < taps owns tap t
    for (int c0 = 0; c0 < C; c0 += CH) {
        const int nch = min(CH, C - c0);
        const int nfl = nch * taps;
        __syncthreads();                                            // previous chunk fully consumed
        for (int i = tid; i < nfl; i += nthr) stage[i] = src[(long long)c0 * taps + i];
        __syncthreads();
        const int nw = (nch + 31) / 32;
        for (int it = tid; it < nw * taps; it += nthr) {
            const int w = it / taps, tap = it - w * taps;
            const int nb = min(32, nch - 32 * w);
            uint32_t word = 0;
            double acc = 0.0;
            if (nb == 32) {
                // whole word: all 32 LDS reads in flight at once, four independent partial sums
                float v[32];
#pragma unroll
                for (int j = 0; j < 32; ++j) v[j] = stage[(32 * w + j) * taps + tap];
                double a4[4] = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
                for (int j = 0; j < 32; ++j) {
                    word |= (v[j] >= 0.0f ? 1u : 0u) << j;
                    a4[j & 3] += (double)fabsf(v[j]);
                }
                acc = (a4[0] + a4[1]) + (a4[2] + a4[3]);
            } else {
                for (int j = 0; j < nb; ++j) {
                    const float v = stage[(32 * w + j) * taps + tap];
                    word |= (v >= 0.0f ? 1u : 0u) << j;
                    acc += (double)fabsf(v);
                }
            }
            dst[tap * Cw + c0 / 32 + w] = word;
            if (Wx) kept[tap * Cw + c0 / 32 + w] = word;
            part[it] = acc;
        }
        __syncthreads();
        if (tid < taps)
            for (int w = 0; w < nw; ++w) tap_total += part[w * taps + tid];
    }
    __syncthreads();
    if (tid < taps) {
        M[(long long)f * taps + tid] = (float)(tap_total / (double)C);
        part[tid] = tap_total;
    }
    __syncthreads();
    if (tid == 0) {
        double sum = 0.0;
        for (int t = 0; t < taps; ++t) sum += part[t];
        alpha[f] = (float)(sum / ((double)C * (double)taps));
    }
    if (Wx) {
        // (the barriers above have made every kept word visible)
        const int tile = f >> 5, row = f & 31;
        uint4 *rows = Wx + (size_t)tile * L.tile_steps * 64;
        for (int e = tid; e < 2 * L.tile_steps; e += nthr) {
            const int step = e >> 1, kg = e & 1;
            rows[(size_t)step * 64 + row + 32 * kg] =
                expanded_entry(L, step, kg, taps, Cw, C, [&](int tap, int w) { return kept[tap * Cw + w]; });
        }
        if (f == F - 1) {
            // rows past the last filter are zeros: the rest of this tile and the tiles after it (the
            // workspace holds whole workgroup rows of 128 filters)
            const size_t first = ((size_t)tile * L.tile_steps * 64), end = L.ws_bytes / sizeof(uint4);
            for (size_t i = first + tid; i < end; i += nthr) {
                const int lane = (int)(i & 63);
                const size_t t = (i >> 6) / L.tile_steps;          // tile of entry i
                if (t > (size_t)tile || (lane & 31) > row) Wx[i] = make_uint4(0, 0, 0, 0);
            }
        }
    }
}

__global__ __launch_bounds__(256) void filter_pack_mean_kernel(
    const float *__restrict__ Wt, int C, int taps, int Cw, int CH, uint32_t *__restrict__ Wpk,
    float *__restrict__ M, float *__restrict__ alpha)
{
    extern __shared__ double fp_smem[];
    filter_pack_mean_block(Wt, C, taps, Cw, CH, Wpk, M, alpha, blockIdx.x, threadIdx.x, 256, fp_smem);
}

// Input side and filter side of a layer in ONE launch: the first blocks each pack up to 256 pixels
// of the input (pack_and_mean4_block; the pixels are shared out evenly over a multiple of the compute
// units, see pixels_per_block4), the last F blocks each prepare one filter (filter_pack_mean_block).
// The two sides do not depend on each other; the filter blocks, dispatched last, cost no launch of
// their own in front of the convolution.
__global__ __launch_bounds__(64 * kPack4Slices) void prepare_both_kernel(
    const float *__restrict__ x, long long NP, int C, int HW, int Cw, int Cwp,
    uint32_t *__restrict__ packed, float *__restrict__ A,
    const float *__restrict__ Wt, int F, int taps, int CH, uint32_t *__restrict__ Wpk,
    float *__restrict__ M, float *__restrict__ alpha, uint4 *__restrict__ Wx, ExpandLayout L, int ppb)
{
    extern __shared__ double both_smem[];
    const long long nb_in = (NP + ppb - 1) / ppb;
    if ((long long)blockIdx.x < nb_in)
        pack_and_mean4_block(x, NP, C, HW, Cw, Cwp, packed, A, blockIdx.x, ppb, both_smem);
    else
        filter_pack_mean_block(Wt, C, taps, Cw, CH, Wpk, M, alpha, (int)(blockIdx.x - nb_in),
                               threadIdx.y * 64 + threadIdx.x, 64 * blockDim.y, both_smem, Wx, L, F);
}

// The same with the one-pixel-per-lane input pass (64 pixels per block): for inputs whose H*W is not
// a multiple of 4, that are not 16-byte aligned, or that are too small to fill the chip with
// 256-pixel blocks.
__global__ __launch_bounds__(64 * kPackMeanSlices) void prepare_both1_kernel(
    const float *__restrict__ x, long long NP, int C, int HW, int Cw, int Cwp,
    uint32_t *__restrict__ packed, float *__restrict__ A,
    const float *__restrict__ Wt, int F, int taps, int CH, uint32_t *__restrict__ Wpk,
    float *__restrict__ M, float *__restrict__ alpha, uint4 *__restrict__ Wx, ExpandLayout L)
{
    extern __shared__ double both_smem[];
    const long long nb_in = (NP + 63) / 64;
    if ((long long)blockIdx.x < nb_in)
        pack_and_mean_block(x, NP, C, HW, Cw, Cwp, packed, A, blockIdx.x, both_smem);
    else
        filter_pack_mean_block(Wt, C, taps, Cw, CH, Wpk, M, alpha, (int)(blockIdx.x - nb_in),
                               threadIdx.y * 64 + threadIdx.x, 64 * blockDim.y, both_smem, Wx, L, F);
}

bool filter_pack_mean_supports(int taps) { return taps <= 256; }

hipError_t launch_filter_pack_mean(const float *Wt, int F, int C, int taps, uint32_t *Wpk, float *M,
                                   float *alpha, hipStream_t st)
{
    const int Cw = (C + 31) / 32;
    int CH = kFilterStageFloats / taps / 32 * 32;                   // >= 32 since taps <= 256
    CH = std::min(CH, Cw * 32);
    const int WH = CH / 32;
    const size_t smem = (size_t)WH * taps * sizeof(double) + (size_t)CH * taps * sizeof(float);
    filter_pack_mean_kernel<<<F, 256, smem, st>>>(Wt, C, taps, Cw, CH, Wpk, M, alpha);
    return hipGetLastError();
}

// One launch for both sides: with the four-pixel input pass where it applies with full-size blocks,
// else with the one-pixel pass; the caller falls back to separate launches where neither fits.
static bool four_pixel_pass(const float *x, int N, int C, int H, int W)
{
    const int HW = H * W, Cw = (C + 31) / 32;
    return HW % 4 == 0 && ((uintptr_t)x & 15) == 0 && (long long)N * HW >= 256 * 256 && Cw >= kPack4Slices;
}

static size_t filter_block_smem(int C, int taps, bool expand, int *CH_out)
{
    const int Cw = (C + 31) / 32;
    int CH = kFilterStageFloats / taps / 32 * 32;
    CH = std::min(CH, Cw * 32);
    *CH_out = CH;
    return (size_t)(CH / 32) * taps * sizeof(double) + (size_t)CH * taps * sizeof(float) +
           (expand ? (size_t)taps * Cw * sizeof(uint32_t) : 0);
}

// Which input pass a single launch for both sides can use: 4 (four pixels per lane), 1 (one pixel
// per lane) or 0 (neither fits: the caller launches the two sides separately).  Either pass shares
// its dynamic LDS (at most 64 KB) with the filter blocks' staging.
static int prepare_both_pass(const float *x, int N, int C, int H, int W, int taps, bool expand)
{
    const int Cw = (C + 31) / 32, Cwp = Cw | 1;
    if (Cw > 512 || taps > 256) return 0;
    int CH;
    const size_t smemf = filter_block_smem(C, taps, expand, &CH);
    if (smemf > 64 * 1024) return 0;
    if (four_pixel_pass(x, N, C, H, W)) {
        const size_t smem4 = (size_t)kPack4Slices * 256 * sizeof(double) + (size_t)256 * Cwp * sizeof(uint32_t);
        if (smem4 <= 64 * 1024) return 4;
    }
    // (the one-pixel pass: the filter block gives every tap a thread of its own)
    int S = 1;
    while (S < kPackMeanSlices && 2 * S <= Cw) S *= 2;
    if (64 * S < taps) return 0;
    const size_t smem1 = (size_t)kPackMeanSlices * 64 * sizeof(double) + (size_t)64 * Cwp * sizeof(uint32_t);
    return smem1 <= 64 * 1024 ? 1 : 0;
}

bool prepare_both_supports(const float *x, int N, int C, int H, int W, int taps)
{
    // (with the filter expansion's LDS counted: the caller may ask for it)
    return prepare_both_pass(x, N, C, H, W, taps, true) != 0;
}

// `Wx` (may be null): the matrix-core kernel's filter workspace, filled as by launch_expand_filters.
bool prepare_both_can_expand(int C, int taps) { return (long long)taps * ((C + 31) / 32) <= 4096; }

hipError_t launch_prepare_both(const float *x, int N, int C, int H, int W, uint32_t *packed, float *A,
                               const float *Wt, int F, int taps, uint32_t *Wpk, float *M, float *alpha,
                               void *Wx, const ExpandLayout &L, hipStream_t st)
{
    const int HW = H * W, Cw = (C + 31) / 32, Cwp = Cw | 1;
    const long long NP = (long long)N * HW;
    int CH;
    const size_t smemf = filter_block_smem(C, taps, Wx != nullptr, &CH);
    const int pass = prepare_both_pass(x, N, C, H, W, taps, Wx != nullptr);
    if (pass == 4) {
        const size_t smem4 = (size_t)kPack4Slices * 256 * sizeof(double) + (size_t)256 * Cwp * sizeof(uint32_t);
        const size_t smem = std::max(smem4, smemf);
        const int ppb = pixels_per_block4(NP, F);
        const long long blocks = (long long)F + ceil_div(NP, ppb);
        if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
        prepare_both_kernel<<<dim3((unsigned)blocks), dim3(64, kPack4Slices), smem, st>>>(
            x, NP, C, HW, Cw, Cwp, packed, A, Wt, F, taps, CH, Wpk, M, alpha, static_cast<uint4 *>(Wx), L, ppb);
        return hipGetLastError();
    }
    if (pass != 1) return hipErrorInvalidValue;   // (prepare_both_supports said no)
    int S = 1;
    while (S < kPackMeanSlices && 2 * S <= Cw) S *= 2;
    const size_t smem1 = (size_t)S * 64 * sizeof(double) + (size_t)64 * Cwp * sizeof(uint32_t);
    const size_t smem = std::max(smem1, smemf);
    const long long blocks = (long long)F + ceil_div(NP, 64);
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    prepare_both1_kernel<<<dim3((unsigned)blocks), dim3(64, S), smem, st>>>(
        x, NP, C, HW, Cw, Cwp, packed, A, Wt, F, taps, CH, Wpk, M, alpha, static_cast<uint4 *>(Wx), L);
    return hipGetLastError();
}

// Eq. 10, second half: K = A * k with constant taps 1/(kh*kw), at the convolution's output
// positions; taps outside the image add nothing.  One thread per output pixel (A is C times smaller
// than I, so this pass is negligible).
__global__ __launch_bounds__(256) void box_filter_K_kernel(const float *__restrict__ A, Geom g,
                                                           long long total, float *__restrict__ K)
{
    const long long o = (long long)blockIdx.x * 256 + threadIdx.x;
    if (o >= total) return;
    const int ox = (int)(o % g.OW);
    const long long t = o / g.OW;
    const int oy = (int)(t % g.OH);
    const long long n = t / g.OH;
    const float *a = A + n * (long long)g.H * g.W;
    double sum = 0.0;
    for (int ky = 0; ky < g.kh; ++ky) {
        const int iy = oy * g.sh - g.ph + ky;
        if (iy < 0 || iy >= g.H) continue;
        for (int kx = 0; kx < g.kw; ++kx) {
            const int ix = ox * g.sw - g.pw + kx;
            if (ix < 0 || ix >= g.W) continue;
            sum += (double)a[iy * g.W + ix];
        }
    }
    K[o] = (float)(sum / (double)(g.kh * g.kw));
}

hipError_t launch_box_filter_K(const float *A, const Geom &g, float *K, hipStream_t st)
{
    const long long total = (long long)g.N * g.OH * g.OW;
    box_filter_K_kernel<<<ceil_div(total, 256), 256, 0, st>>>(A, g, total, K);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Eq. 5: alpha[f] = ||Wt[f]||_1 / n.  One block per filter, double partial sums, fixed-order tree.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void alpha_kernel(const float *__restrict__ Wt, long long n_red,
                                                    float *__restrict__ alpha)
{
    __shared__ double part[256];
    const float *w = Wt + (long long)blockIdx.x * n_red;
    double acc = 0.0;
    for (long long i = threadIdx.x; i < n_red; i += 256) acc += (double)fabsf(w[i]);
    part[threadIdx.x] = acc;
    __syncthreads();
    for (int step = 128; step > 0; step >>= 1) {
        if ((int)threadIdx.x < step) part[threadIdx.x] += part[threadIdx.x + step];
        __syncthreads();
    }
    if (threadIdx.x == 0) alpha[blockIdx.x] = (float)(part[0] / (double)n_red);
}

hipError_t launch_alpha(const float *Wt, int F, long long n_red, float *alpha, hipStream_t st)
{
    alpha_kernel<<<F, 256, 0, st>>>(Wt, n_red, alpha);
    return hipGetLastError();
}

}  // namespace xnor
