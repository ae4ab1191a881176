// The whole forward pass in one kernel for images with one to four channels (first layers, and the
// workload the paper itself times: one channel, 3x3 filter, 256^2 ... 2048^2 pixels, Tables I-III).
//
// With so few channels a channel-packed word carries one to four useful bits, and per output there
// are only kh*kw*C binary MACs against 4 bytes read and 4*F bytes written: the layer is a stream
// through HBM, not arithmetic.  So nothing intermediate is written: steps 1a-1d, 2a-2b and 3 of
// Sec. III-A (Eq. 10, Eq. 11) run on registers between one read of the fp32 image and one write of
// the fp32 output.
//   * A lane owns one output column of a band of rows and slides down it (with a vertical stride an
//     output is due every sh-th input row).  For every input row it
//     loads the kw*C values under its window, forms their kw*C sign bits (bit = x >= 0) and the sum
//     of their magnitudes, and keeps the last kh of both: the spatially packed window of Sec. III-B
//     (kh*kw*C bits, rows side by side in as few 32-bit words as hold them) and the kh row sums
//     whose total is K * C*kh*kw.
//   * Per output and filter: popcount((window xor filter window) and mask); the mask holds the
//     in-image taps, so a padded tap adds nothing, and popcount(mask) = C * (#in-image taps).
//       dot = popcount(mask) - 2 * popcount(...),   out = float(dot) * K * alpha.
//     For rows whose window lies inside the image vertically the mask is a per-lane constant.
//   * Loads of the next rows are issued a few rows ahead of their use; neighbouring lanes read
//     overlapping addresses, which the vector cache serves.
// The paper's kernels (Alg. 1 and 2) also pack a spatial tile into one register, one channel and one
// 8x4 tile per thread, and run binarisation, K and the convolution as separate kernels on separate
// streams; here the row words live only in registers and the three are one pass.
#include <algorithm>

#include "xnor_internal.hpp"

namespace xnor {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
constexpr size_t kLdsBudget = 64 * 1024;

struct ImageParams {
    const float *I;
    const uint32_t *Wpk;
    const float *alpha;
    float *out;
    int32_t *dot;
    int N, H, W, F, OH, OW, ph, pw, sh, sw;
    int rows_per_band, bands, xtiles;
    int group, fgroups;  // filters per wave, ceil(F / group)
    long long waves;     // N * fgroups * bands * xtiles
    float kscale;        // 1 / (C * kh * kw)
};

template <int K, int C>
struct Cfg {
    static constexpr int kRowBits = K * C;                       // sign bits of one window row
    static constexpr int kRowsPerWord = 32 / kRowBits;
    static constexpr int kWords = (K + kRowsPerWord - 1) / kRowsPerWord;
    static constexpr int kAhead = kRowBits <= 3 ? 8 : kRowBits <= 7 ? 4 : kRowBits <= 12 ? 2 : 1;
    static constexpr uint32_t kChanMask = (1u << C) - 1u;
};

template <int K, int C, bool ONE_FILTER, bool UNIT_STRIDE>
__global__ __launch_bounds__(kThreads) void conv_image_kernel(ImageParams p)
{
    const int sh = UNIT_STRIDE ? 1 : p.sh, sw = UNIT_STRIDE ? 1 : p.sw;   // stride 1 is compiled in
    using G = Cfg<K, C>;
    constexpr int RB = G::kRowBits, NW = G::kWords, RPW = G::kRowsPerWord, D = G::kAhead;
    extern __shared__ uint32_t lds[];        // filter windows [F][NW], then alpha [F]
    uint32_t *wf = lds;
    float *al = reinterpret_cast<float *>(lds + (size_t)p.F * NW);

    // filter windows in the window's bit order: row r of the filter sits at bit (r % RPW) * RB of
    // word r / RPW, tap kx at kx * C inside the row, channel c at bit c of the tap
    auto filter_window = [&](int f, uint32_t (&w)[NW]) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < NW; ++i) w[i] = 0;
#pragma unroll
        for (int r = 0; r < K; ++r)
#pragma unroll
            for (int kx = 0; kx < K; ++kx)
                w[r / RPW] |= (p.Wpk[((size_t)f * K + r) * K + kx] & G::kChanMask)
                              << ((r % RPW) * RB + kx * C);
    };
    if (!ONE_FILTER) {
        for (int f = threadIdx.x; f < p.F; f += kThreads) {
            uint32_t w[NW];
            filter_window(f, w);
#pragma unroll
            for (int i = 0; i < NW; ++i) wf[(size_t)f * NW + i] = w[i];
            al[f] = p.alpha[f];
        }
        __syncthreads();
    }

    const int lane = threadIdx.x & 63;
    const long long gw = (long long)blockIdx.x * kWaves + (threadIdx.x >> 6);
    if (gw >= p.waves) return;
    const int xt = __builtin_amdgcn_readfirstlane((int)(gw % p.xtiles));
    const long long t = gw / p.xtiles;
    const int band = __builtin_amdgcn_readfirstlane((int)(t % p.bands));
    const long long u = t / p.bands;
    const int f0 = __builtin_amdgcn_readfirstlane((int)(u % p.fgroups)) * p.group;
    const int f1 = min(p.F, f0 + p.group);
    const int n = __builtin_amdgcn_readfirstlane((int)(u / p.fgroups));
    const int x = xt * 64 + lane;
    if (x >= p.OW) return;

    // which of the window's columns lie inside the image: a per-lane constant
    bool cv[K];
    uint32_t row_mask = 0;
#pragma unroll
    for (int kx = 0; kx < K; ++kx) {
        const int xin = x * sw - p.pw + kx;
        cv[kx] = xin >= 0 && xin < p.W;
        row_mask |= cv[kx] ? (G::kChanMask << (kx * C)) : 0u;
    }
    uint32_t full_mask[NW];
#pragma unroll
    for (int i = 0; i < NW; ++i) full_mask[i] = 0;
#pragma unroll
    for (int r = 0; r < K; ++r) full_mask[r / RPW] |= row_mask << ((r % RPW) * RB);
    int full_valid = 0;
#pragma unroll
    for (int i = 0; i < NW; ++i) full_valid += __builtin_popcount(full_mask[i]);

    const int y0 = band * p.rows_per_band;
    const int y1 = min(p.OH, y0 + p.rows_per_band);
    const int nin = (y1 - y0 - 1) * sh + K;   // input rows this band walks through
    const int yb = y0 * sh - p.ph;            // the first of them (negative: above the image)
    const size_t HW = (size_t)p.H * p.W;
    const float *src = p.I + (size_t)n * C * HW + (x * sw - p.pw);   // only dereferenced where valid
    const size_t OHW = (size_t)p.OH * p.OW;

    float pre[D][RB];
    auto issue = [&](int slot, int i) __attribute__((always_inline)) {
        const int yin = yb + i;
        const bool rv = i < nin && yin >= 0 && yin < p.H;
#pragma unroll
        for (int c = 0; c < C; ++c)
#pragma unroll
            for (int kx = 0; kx < K; ++kx)
                pre[slot][c * K + kx] =
                    (rv && cv[kx]) ? src[(size_t)c * HW + (size_t)yin * p.W + kx] : 0.f;
    };

    uint32_t rw[K];   // sign bits of the last K input rows
    float hs[K];      // sums of |I| over those rows' kw*C values
#pragma unroll
    for (int r = 0; r < K; ++r) { rw[r] = 0; hs[r] = 0.f; }

#pragma unroll
    for (int d = 0; d < D; ++d) issue(d, d);

    // a single filter stays in registers: its words come through wave-uniform loads that are in
    // flight together with the first image rows, and no workgroup barrier is needed
    uint32_t fw[NW];
    float a0 = 0.f;
    if (ONE_FILTER) {
        filter_window(0, fw);
        a0 = p.alpha[0];
    }

    int skip = 1;                           // input rows until the next output row is due
    for (int i0 = 0; i0 < nin; i0 += D) {
#pragma unroll
        for (int d = 0; d < D; ++d) {
            const int i = i0 + d;
            if (i >= nin) break;
            uint32_t bits = 0;
            float hsum = 0.f;
#pragma unroll
            for (int c = 0; c < C; ++c)
#pragma unroll
                for (int kx = 0; kx < K; ++kx) {
                    const float v = pre[d][c * K + kx];
                    bits |= (v >= 0.f) ? (1u << (kx * C + c)) : 0u;
                    hsum += fabsf(v);
                }
            issue(d, i + D);
#pragma unroll
            for (int r = 0; r + 1 < K; ++r) { rw[r] = rw[r + 1]; hs[r] = hs[r + 1]; }
            rw[K - 1] = bits;
            hs[K - 1] = hsum;
            // an output row is complete when its last window row has arrived: every sh-th row
            if (i < K - 1) continue;
            if (--skip > 0) continue;
            skip = sh;

            const int y = y0 + (i - (K - 1)) / sh;
            uint32_t win[NW], m[NW];
#pragma unroll
            for (int w = 0; w < NW; ++w) win[w] = 0;
#pragma unroll
            for (int r = 0; r < K; ++r) win[r / RPW] |= rw[r] << ((r % RPW) * RB);
            int nvalid;
            const int ytop = y * sh - p.ph;
            if (ytop >= 0 && ytop + K - 1 < p.H) {
#pragma unroll
                for (int w = 0; w < NW; ++w) m[w] = full_mask[w];
                nvalid = full_valid;
            } else {
#pragma unroll
                for (int w = 0; w < NW; ++w) m[w] = 0;
#pragma unroll
                for (int r = 0; r < K; ++r) {
                    const bool rv = ytop + r >= 0 && ytop + r < p.H;
                    m[r / RPW] |= rv ? (row_mask << ((r % RPW) * RB)) : 0u;
                }
                nvalid = 0;
#pragma unroll
                for (int w = 0; w < NW; ++w) nvalid += __builtin_popcount(m[w]);
            }
            float ksum = hs[0];
#pragma unroll
            for (int r = 1; r < K; ++r) ksum += hs[r];
            const float kk = ksum * p.kscale;
            const size_t o = (size_t)n * p.F * OHW + (size_t)y * p.OW + x;
            if (ONE_FILTER) {
                int pop = 0;
#pragma unroll
                for (int w = 0; w < NW; ++w) pop += __builtin_popcount((win[w] ^ fw[w]) & m[w]);
                const int d1 = nvalid - 2 * pop;
                p.out[o] = (float)d1 * (kk * a0);
                if (p.dot) p.dot[o] = d1;
            } else {
                for (int f = f0; f < f1; ++f) {
                    int pop = 0;
#pragma unroll
                    for (int w = 0; w < NW; ++w)
                        pop += __builtin_popcount((win[w] ^ wf[(size_t)f * NW + w]) & m[w]);
                    const int d1 = nvalid - 2 * pop;
                    p.out[o + (size_t)f * OHW] = (float)d1 * (kk * al[f]);
                    if (p.dot) p.dot[o + (size_t)f * OHW] = d1;
                }
            }
        }
    }
}

template <int K, int C>
hipError_t launch_kc(const ImageParams &p, dim3 grid, size_t lds, hipStream_t st)
{
    const bool unit = p.sh == 1 && p.sw == 1;
    if (p.F == 1 && unit)
        conv_image_kernel<K, C, true, true><<<grid, dim3(kThreads), lds, st>>>(p);
    else if (p.F == 1)
        conv_image_kernel<K, C, true, false><<<grid, dim3(kThreads), lds, st>>>(p);
    else if (unit)
        conv_image_kernel<K, C, false, true><<<grid, dim3(kThreads), lds, st>>>(p);
    else
        conv_image_kernel<K, C, false, false><<<grid, dim3(kThreads), lds, st>>>(p);
    return hipGetLastError();
}

template <int K>
hipError_t launch_k(int C, const ImageParams &p, dim3 grid, size_t lds, hipStream_t st)
{
    switch (C) {
        case 1: return launch_kc<K, 1>(p, grid, lds, st);
        case 2: return launch_kc<K, 2>(p, grid, lds, st);
        case 3: return launch_kc<K, 3>(p, grid, lds, st);
        default: return launch_kc<K, 4>(p, grid, lds, st);
    }
}

int window_words(int k, int C) { return (k + 32 / (k * C) - 1) / (32 / (k * C)); }

}  // namespace

bool conv_image_supports(const Geom &g)
{
    if (g.C < 1 || g.C > 4) return false;
    if (g.kh != g.kw || (g.kh != 3 && g.kh != 5 && g.kh != 7)) return false;
    if ((size_t)g.F * (window_words(g.kh, g.C) + 1) * 4 > kLdsBudget) return false;
    return true;
}

hipError_t launch_conv_image(const float *I, const uint32_t *Wpk, const float *alpha, const Geom &g,
                             float *out, int32_t *dot, hipStream_t st)
{
    ImageParams p;
    p.I = I; p.Wpk = Wpk; p.alpha = alpha; p.out = out; p.dot = dot;
    p.N = g.N; p.H = g.H; p.W = g.W; p.F = g.F; p.OH = g.OH; p.OW = g.OW; p.ph = g.ph; p.pw = g.pw; p.sh = g.sh; p.sw = g.sw;
    p.xtiles = ceil_div(g.OW, 64);
    // Band height: tall bands re-read fewer halo rows, short ones give more waves.  Halve from 64
    // until the chip has about eight waves per SIMD; an image too small for that even with bands
    // of 8 rows is bound by the chain of load latencies down a band, so it gets bands of 4.
    // (Measured, one channel, 3x3: 4096^2 is fastest with 32 rows, 2048^2 with 16 or 8, 1024^2
    // with 8, 512^2 and below with 4.)
    auto waves_with = [&](int rows) { return (long long)g.N * p.xtiles * ceil_div(g.OH, rows); };
    int rows = 64;
    while (rows > 8 && waves_with(rows) < 256LL * 4 * 8) rows /= 2;
    if (waves_with(rows) < 256LL * 4 * 2) rows = 4;
    p.rows_per_band = std::max(1, std::min(rows, g.OH));
    p.bands = ceil_div(g.OH, p.rows_per_band);
    // With many filters and a small image the filters are shared out over waves as well (each
    // wave rebuilds the window, which costs little next to the work of its filters).
    p.group = g.F;
    while (p.group > 4 && waves_with(p.rows_per_band) * ceil_div(g.F, p.group) < 256LL * 4 * 4)
        p.group = (p.group + 1) / 2;
    p.fgroups = ceil_div(g.F, p.group);
    p.waves = waves_with(p.rows_per_band) * p.fgroups;
    p.kscale = 1.0f / (float)(g.C * g.kh * g.kw);
    const long long blocks = (p.waves + kWaves - 1) / kWaves;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    const size_t lds = g.F == 1 ? 0 : (size_t)g.F * (window_words(g.kh, g.C) + 1) * 4;
    const dim3 grid((unsigned)blocks);
    switch (g.kh) {
        case 3: return launch_k<3>(g.C, p, grid, lds, st);
        case 5: return launch_k<5>(g.C, p, grid, lds, st);
        default: return launch_k<7>(g.C, p, grid, lds, st);
    }
}

}  // namespace xnor
