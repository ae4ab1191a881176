// Binary-Weight-Network convolution (Sec. II-A, Eq. 1): the input keeps its real values, the
// weights are their signs, and the per-filter alpha of Eq. 5 scales the sum:
//     O[n][f][oy][ox] = alpha[f] * sum_{in-image taps, c} (B[f][c][ky][kx] = +1 ? +I : -I).
// No input binarisation and no K.  The filter signs come packed (xnor_filter_prepare /
// xnor_binarize_pack: bit 1 = +1).
//
// The paper describes this as a convolution of additions and subtractions.  On this chip the
// cheapest way to add or subtract 4608 fp32 values per output is a dense fp32 contraction on the
// matrix cores with +-1.0 as one operand: v_mfma_f32_32x32x2_f32 retires 2048 of them per
// instruction, and a product with +-1.0 is exact, so the result is the fp32 sum.
//
//   bwn_mfma_kernel: rows of the MFMA = 32 filters, columns = 32 consecutive output pixels of one
//   image, reduction = channel pairs at a fixed tap.  A workgroup (4 waves = 4 filter tiles) owns
//   up to 6 pixel tiles; per chunk of channels it stages the input rows under them once in LDS as
//   fp32, zero where the image ends (that is the zero padding), and the chunk's filter words.  The
//   B operand of each MFMA is one LDS dword per lane (lane = pixel, its channel = pair member);
//   the A operand is +-1.0 made from the lane's filter word with three integer instructions per
//   NT MFMAs.  The accumulator layout gives each lane 16 filters of one pixel, so stores run
//   along the pixels of a filter plane.
//   bwn_direct_kernel: one thread per output, any shape; the fallback and the cross-check.
//
// The same kernel with REALW = true is the real-valued ("vanilla") convolution that Sec. IV's
// Table I sets the XNOR convolution against: the A operand is then the fp32 weight itself, staged
// per channel chunk in LDS as [tap][channel][filter] next to the input rows, and there is no alpha.
//   conv_fp32_direct_kernel: one thread per output, any shape.
//   conv_fp32_rows_kernel: few channels, unit stride along x: four outputs per thread.
#include <algorithm>
#include <atomic>

#include "xnor_internal.hpp"

namespace xnor {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kThreads = 256;
constexpr int kFiltersPerWg = 128;   // 4 waves x 32 rows
constexpr int kMaxTiles = 6;         // pixel tiles (of 32) per workgroup: 6 x 16 accumulator registers
constexpr size_t kLdsBudget = 64 * 1024;   // two workgroups per compute unit
constexpr size_t kLdsWide = 128 * 1024;    // wide rows, staged synchronously: one workgroup per compute unit
constexpr int kPre = 32;             // input values a thread fetches ahead per chunk
constexpr int kPreWords = 8;         // filter words a thread fetches ahead per chunk (kh*kw <= 16)
constexpr int kPreWeights = 36;      // real weights a thread fetches ahead per chunk (8 channels x 9 taps x 128 filters)
constexpr int kPreW4 = kPreWeights / 4;
constexpr int kWPitch = kFiltersPerWg + 1;   // floats per (tap, channel) row of staged real weights: the
                                             // transposing writes of one filter's run then spread over the banks

struct BwnParams {
    const float *I;
    const uint32_t *Wpk;   // packed filter signs (Binary-Weight-Network form), or
    const float *Wt;       // the fp32 filters [F][C][kh][kw] (real-valued form)
    const float *alpha;
    float *out;
    int N, C, H, W, F, kh, kw, sh, sw, ph, pw, OH, OW, Cw;
    int tiles;          // pixel tiles per workgroup
    int groups;         // workgroups along the pixels of one image
    int fgroups;        // workgroups along the filters
    int chan;           // channels per chunk: 32, 16 or 8 (a chunk never straddles a packed word)
    int rows_max;       // staged input rows (upper bound over the pixel groups)
    int pitch;          // staged floats per row = W + 2*pw
    uint32_t inv_plane, inv_pitch;   // ceil(2^32 / (rows_max * pitch)), ceil(2^32 / pitch): exact quotients below 2^16
                                     // (0 for a divisor of 1, whose reciprocal does not fit: see quot())
    uint32_t inv_per, inv_taps;      // the same for chan * taps and taps (real-valued form)
    int w4;                          // real-valued form: the chunk's weights can be fetched 16 bytes per lane
};

// n / d through one multiply-high with inv = ceil(2^32 / d), exact for n*d < 2^32; d = 1 has no
// such 32-bit reciprocal (2^32) and is flagged by inv = 0 (uniform: a scalar select).
__device__ inline uint32_t quot(uint32_t n, uint32_t inv) { return inv == 0 ? n : __umulhi(n, inv); }
uint32_t reciprocal(unsigned long long d) { return d == 1 ? 0u : (uint32_t)(((1ULL << 32) + d - 1) / d); }

// The work of one workgroup with NT pixel tiles.  NT is a template parameter so that the MFMA
// loop is one basic block (operands of the next MFMAs are loaded ahead of the current ones) and
// the accumulators are NT x 16 fixed registers.
template <int NT, bool AHEAD, bool REALW>
__device__ __attribute__((always_inline)) void bwn_workgroup(const BwnParams &p, int n, int fbase,
                                                              int p0, int p1)
{
    extern __shared__ float lds[];
    // [chan][rows][pitch] input, then [taps][128] filter words or [taps][chan][kWPitch] filter values
    const int plane = p.rows_max * p.pitch;
    float *tile = lds;
    uint32_t *fw = reinterpret_cast<uint32_t *>(lds + (size_t)p.chan * plane);
    float *wf = lds + (size_t)p.chan * plane;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int col = lane & 31, half = lane >> 5;
    const int OHW = p.OH * p.OW;
    const int oy0 = p0 / p.OW, oy1 = (p1 - 1) / p.OW;
    const int iy0 = oy0 * p.sh - p.ph;
    const int rows = (oy1 - oy0) * p.sh + p.kh;         // <= rows_max
    const int taps = p.kh * p.kw;

    // per pixel tile: this lane's LDS float index of tap (0,0), channel `half`, chunk start
    int base[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j) {
        const int px = min(p0 + 32 * j + col, p1 - 1);
        const int oy = px / p.OW, ox = px - oy * p.OW;
        base[j] = half * plane + (oy - oy0) * p.sh * p.pitch + ox * p.sw;
    }

    floatx16 acc[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;

    const int chunks_per_word = 32 / p.chan;
    const int nchunks = (p.C + p.chan - 1) / p.chan;
    const float *img = p.I + (size_t)n * p.C * p.H * p.W;

    // Staging.  The chunk's input rows are fetched into registers one chunk ahead, while the
    // previous chunk's MFMAs run, and written to LDS between two barriers.  The staged block is
    // walked as one flat array [chan][rows_max][pitch]: thread t owns elements t, t + 256, ...;
    // channel, row and column come from two multiply-high divisions (constants from the host);
    // every load is issued unconditionally (from element 0 of the image where the slot lies outside
    // it or past the band's rows) and zeroed by a select, so there is no divergent code.
    const int nelem = p.chan * plane;                          // <= kPre * 256 (the host's plan sees to it)
    const bool words_ahead = !REALW && AHEAD && taps * kFiltersPerWg <= kPreWords * kThreads;
    const bool weights_ahead = REALW && AHEAD && kFiltersPerWg * p.chan * taps <= kPreWeights * kThreads;
    float nxt[kPre];
    uint32_t nxw[kPreWords];
    float nxf[REALW ? kPreWeights : 1];
    // The 16-byte form of the same prefetch (whole chunks of 8 channels, aligned runs): lane = filter,
    // the two halves of the workgroup take alternate groups of four weights of the filter's run, so
    // channel and tap of every weight are wave-uniform and the index arithmetic is scalar.
    const bool w4 = weights_ahead && p.w4;
    const int w4_half = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 7);
    const int w4_groups = (p.chan * taps) >> 3;             // groups of four per half
    // where element i of the chunk's [filter][channel][tap] weights lies: its offset in Wt (or -1: no
    // such filter or channel) and its place in the transposed LDS block
    auto weight_slot = [&](int i, int c0, int &lds_at) __attribute__((always_inline)) -> long long {
        const int per = p.chan * taps;
        const int f = (int)quot((uint32_t)i, p.inv_per), e = i - f * per;
        const int c = (int)quot((uint32_t)e, p.inv_taps), t = e - c * taps;
        lds_at = (t * p.chan + c) * kWPitch + f;
        const int fg = fbase + f;
        return (fg < p.F && c0 + c < p.C) ? ((long long)fg * p.C + c0) * taps + e : -1;
    };
    // (the thread index passes through an empty asm in each call: otherwise the per-element offsets,
    // which do not change from chunk to chunk, are all kept in registers across the MFMA loop)
    auto prefetch = [&](int ch) __attribute__((always_inline)) {
        const int c0 = ch * p.chan;
        int t0 = threadIdx.x;
        asm volatile("" : "+v"(t0));
#pragma unroll
        for (int q = 0; q < kPre; ++q) {
            if (q * kThreads >= nelem) break;                  // uniform
            const uint32_t e = (uint32_t)(q * kThreads + t0);
            const uint32_t c = quot(e, p.inv_plane);
            const uint32_t rem = e - c * (uint32_t)plane;
            const uint32_t r = quot(rem, p.inv_pitch);
            const int xw = (int)(rem - r * (uint32_t)p.pitch);
            const int iy = iy0 + (int)r, ix = xw - p.pw, cg = c0 + (int)c;
            const bool ok = (int)c < p.chan && (int)r < rows && (unsigned)iy < (unsigned)p.H &&
                            (unsigned)ix < (unsigned)p.W && cg < p.C;
            const float v = img[ok ? (unsigned)((cg * p.H + iy) * p.W + ix) : 0u];   // one image: below 2^30 floats
            nxt[q] = ok ? v : 0.f;
        }
        if (w4) {
            const int fg = min(fbase + (t0 & (kFiltersPerWg - 1)), p.F - 1);   // (filters past the last: zeroed on commit)
            const float4 *src = reinterpret_cast<const float4 *>(p.Wt + ((size_t)fg * p.C + c0) * taps);
#pragma unroll
            for (int q = 0; q < kPreW4; ++q) {
                if (q >= w4_groups) break;                     // uniform
                const float4 v = src[2 * q + w4_half];
                nxf[REALW ? 4 * q + 0 : 0] = v.x; nxf[REALW ? 4 * q + 1 : 0] = v.y;
                nxf[REALW ? 4 * q + 2 : 0] = v.z; nxf[REALW ? 4 * q + 3 : 0] = v.w;
            }
        } else if (weights_ahead) {
#pragma unroll
            for (int q = 0; q < kPreWeights; ++q) {
                if (q * kThreads >= kFiltersPerWg * p.chan * taps) break;   // uniform
                int at;
                const long long src = weight_slot(q * kThreads + t0, c0, at);
                const float v = p.Wt[src < 0 ? 0 : src];
                nxf[REALW ? q : 0] = src < 0 ? 0.f : v;
            }
        }
        if (words_ahead) {
            const int cw = ch / chunks_per_word, bit0 = (ch % chunks_per_word) * p.chan;
#pragma unroll
            for (int q = 0; q < kPreWords; ++q) {
                const int i = q * kThreads + t0;
                const int t = i / kFiltersPerWg, f = fbase + (i - t * kFiltersPerWg);
                // (loaded unconditionally, from word 0 where there is no such filter or tap: a load
                //  under a condition is waited for before the next one is issued)
                const bool live = i < taps * kFiltersPerWg && f < p.F;
                const uint32_t w = p.Wpk[live ? ((size_t)f * taps + t) * p.Cw + cw : 0];
                nxw[q] = live ? w >> bit0 : 0u;
            }
        }
    };
    auto commit = [&](int ch) __attribute__((always_inline)) {
        int t0 = threadIdx.x;
        asm volatile("" : "+v"(t0));
        if (AHEAD) {
#pragma unroll
            for (int q = 0; q < kPre; ++q) {
                if (q * kThreads >= nelem) break;              // uniform
                const int e = q * kThreads + t0;
                if (e < nelem) tile[e] = nxt[q];
            }
        }
        if (REALW) {
            // the chunk's weights of filter f are one run of chan * taps floats in memory; they go to
            // LDS transposed, [tap][channel][filter], so that a wave reads its 32 filters side by side
            const int c0 = ch * p.chan;
            if (w4) {
                const int f = t0 & (kFiltersPerWg - 1);
                const bool live = fbase + f < p.F;
#pragma unroll
                for (int q = 0; q < kPreW4; ++q) {
                    if (q >= w4_groups) break;                 // uniform
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        const int e = 4 * (2 * q + w4_half) + k;           // uniform: place in the filter's run
                        const int c = (int)quot((uint32_t)e, p.inv_taps), t = e - c * taps;
                        wf[(t * p.chan + c) * kWPitch + f] = live ? nxf[REALW ? 4 * q + k : 0] : 0.f;
                    }
                }
            } else if (weights_ahead) {
#pragma unroll
                for (int q = 0; q < kPreWeights; ++q) {
                    if (q * kThreads >= kFiltersPerWg * p.chan * taps) break;   // uniform
                    int at;
                    weight_slot(q * kThreads + t0, c0, at);
                    wf[at] = nxf[REALW ? q : 0];
                }
            } else {
                for (int i = threadIdx.x; i < kFiltersPerWg * p.chan * taps; i += kThreads) {
                    int at;
                    const long long src = weight_slot(i, c0, at);
                    const float v = p.Wt[src < 0 ? 0 : src];
                    wf[at] = src < 0 ? 0.f : v;
                }
            }
        } else if (words_ahead) {
#pragma unroll
            for (int q = 0; q < kPreWords; ++q) {
                const int i = q * kThreads + threadIdx.x;
                if (i < taps * kFiltersPerWg) fw[i] = nxw[q];
            }
        } else {
            const int cw = ch / chunks_per_word, bit0 = (ch % chunks_per_word) * p.chan;
            for (int i = threadIdx.x; i < taps * kFiltersPerWg; i += kThreads) {
                const int t = i / kFiltersPerWg, f = fbase + (i - t * kFiltersPerWg);
                fw[i] = f < p.F ? p.Wpk[((size_t)f * taps + t) * p.Cw + cw] >> bit0 : 0u;
            }
        }
    };

    // Rows too wide for the registers set aside above (more than kPre values per thread and chunk)
    // are staged the plain way, global -> LDS between the two barriers, eight loads in flight.
    auto stage_now = [&](int ch) __attribute__((always_inline)) {
        const int c0 = ch * p.chan;
        const int nseg = p.chan * rows;
        for (int xw0 = 0; xw0 < p.pitch; xw0 += 32) {
            const int xw = xw0 + (threadIdx.x & 31), ix = xw - p.pw;
            const bool colok = xw < p.pitch && ix >= 0 && ix < p.W;
            for (int sg = threadIdx.x >> 5; sg < nseg; sg += 64) {
                float v[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int s2 = sg + 8 * u;
                    const int c = s2 / rows, r = s2 - c * rows;
                    const int iy = iy0 + r, cg = c0 + c;
                    const bool in = s2 < nseg && colok && cg < p.C && iy >= 0 && iy < p.H;
                    v[u] = in ? img[(unsigned)((cg * p.H + iy) * p.W + ix)] : 0.f;
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int s2 = sg + 8 * u;
                    const int c = s2 / rows, r = s2 - c * rows;
                    if (s2 < nseg && xw < p.pitch) tile[c * plane + r * p.pitch + xw] = v[u];
                }
            }
        }
    };

    if (AHEAD) prefetch(0);
    for (int ch = 0; ch < nchunks; ++ch) {
        __syncthreads();                                 // the previous chunk has been read
        if (!AHEAD) stage_now(ch);
        commit(ch);
        __syncthreads();
        if (AHEAD && ch + 1 < nchunks) prefetch(ch + 1);

        for (int ky = 0; ky < p.kh; ++ky)
            for (int kx = 0; kx < p.kw; ++kx) {
                const int tap = ky * p.kw + kx;
                const uint32_t word = REALW ? 0u : fw[tap * kFiltersPerWg + wave * 32 + col] >> half;
                // (real weights: this lane's filter, channel `half` of the chunk, this tap)
                const float *wcol = wf + (tap * p.chan + half) * kWPitch + wave * 32 + col;
                const int toff = ky * p.pitch + kx;
                // B operands are read one step (NT MFMAs) ahead of their use; the scheduling
                // barriers keep the compiler from moving each read back next to its MFMA
                const int ncp = p.chan / 2;
                float bc[NT], bn[NT];
                float ac = 0.f, an = 0.f;
#pragma unroll
                for (int j = 0; j < NT; ++j) bc[j] = tile[base[j] + toff];
                if (REALW) ac = wcol[0];
                for (int q = 0; q < p.chan / 8; ++q) {       // four channel pairs at a time
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int cp = 4 * q + u;
                        const int nx = min(cp + 1, ncp - 1);
                        const int off = toff + 2 * nx * plane;
#pragma unroll
                        for (int j = 0; j < NT; ++j) bn[j] = tile[base[j] + off];
                        if (REALW) an = wcol[2 * nx * kWPitch];
                        __builtin_amdgcn_sched_barrier(0);
                        // bit (2*cp + half) of the chunk: 1 -> +1.0f, 0 -> -1.0f
                        const float a = REALW ? ac : __uint_as_float(0xBF800000u ^ (((word >> (2 * cp)) & 1u) << 31));
#pragma unroll
                        for (int j = 0; j < NT; ++j)
                            acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, bc[j], acc[j], 0, 0, 0);
                        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                        for (int j = 0; j < NT; ++j) bc[j] = bn[j];
                        ac = an;
                    }
                }
            }
    }

    // accumulator register r of a lane: filter row 8*(r/4) + 4*half + r%4 of the wave's tile,
    // pixel column `col`
    float al[16];
    int fr[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        fr[r] = fbase + wave * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
        al[r] = REALW ? 1.f : fr[r] < p.F ? p.alpha[fr[r]] : 0.f;
    }
    float *dst = p.out + (size_t)n * p.F * OHW;
#pragma unroll
    for (int j = 0; j < NT; ++j) {
        const int px = p0 + 32 * j + col;
        if (px < p1) {
#pragma unroll
            for (int r = 0; r < 16; ++r)
                if (fr[r] < p.F) dst[(size_t)fr[r] * OHW + px] = REALW ? acc[j][r] : acc[j][r] * al[r];
        }
    }
}

template <bool AHEAD, bool REALW>
__global__ __launch_bounds__(kThreads, 2) void bwn_mfma_kernel(BwnParams p)
{
    int b = blockIdx.x;
    const int h = b % p.fgroups; b /= p.fgroups;
    const int g = b % p.groups;
    const int n = b / p.groups;
    const int p0 = g * p.tiles * 32;
    const int p1 = min(p.OH * p.OW, p0 + p.tiles * 32);
    const int fbase = h * kFiltersPerWg;
    const int nt = (p1 - p0 + 31) >> 5;                  // tiles this workgroup really has
    if (AHEAD) {
        switch (nt) {
            case 1: bwn_workgroup<1, AHEAD, REALW>(p, n, fbase, p0, p1); break;
            case 2: bwn_workgroup<2, AHEAD, REALW>(p, n, fbase, p0, p1); break;
            case 3: bwn_workgroup<3, AHEAD, REALW>(p, n, fbase, p0, p1); break;
            case 4: bwn_workgroup<4, AHEAD, REALW>(p, n, fbase, p0, p1); break;
            case 5: bwn_workgroup<5, AHEAD, REALW>(p, n, fbase, p0, p1); break;
            default: bwn_workgroup<6, AHEAD, REALW>(p, n, fbase, p0, p1); break;
        }
    } else {
        // wide rows: few tiles per workgroup anyway; two specialisations are enough
        if (nt <= 2) bwn_workgroup<2, AHEAD, REALW>(p, n, fbase, p0, p1);
        else bwn_workgroup<6, AHEAD, REALW>(p, n, fbase, p0, p1);
    }
}

__global__ __launch_bounds__(256) void bwn_direct_kernel(const float *__restrict__ I,
                                                         const uint32_t *__restrict__ Wpk,
                                                         const float *__restrict__ alpha, Geom g,
                                                         long long total, float *__restrict__ out)
{
    const long long o = (long long)blockIdx.x * 256 + threadIdx.x;
    if (o >= total) return;
    const int ox = (int)(o % g.OW);
    long long t = o / g.OW;
    const int oy = (int)(t % g.OH);
    t /= g.OH;
    const int f = (int)(t % g.F);
    const long long n = t / g.F;
    const size_t HW = (size_t)g.H * g.W;
    const float *img = I + n * g.C * HW;
    const uint32_t *flt = Wpk + (size_t)f * g.kh * g.kw * g.Cw;
    float acc = 0.f;
    for (int ky = 0; ky < g.kh; ++ky) {
        const int iy = oy * g.sh - g.ph + ky;
        if (iy < 0 || iy >= g.H) continue;
        for (int kx = 0; kx < g.kw; ++kx) {
            const int ix = ox * g.sw - g.pw + kx;
            if (ix < 0 || ix >= g.W) continue;
            const float *src = img + (size_t)iy * g.W + ix;
            float tap = 0.f;                      // per-tap partial sums keep the adder chain short
            for (int w = 0; w < g.Cw; ++w) {
                const uint32_t bits = flt[(ky * g.kw + kx) * g.Cw + w];
                const int cn = min(32, g.C - 32 * w);
                float part = 0.f;
                for (int j = 0; j < cn; ++j) {
                    const float v = src[(size_t)(32 * w + j) * HW];
                    part += ((bits >> j) & 1u) ? v : -v;
                }
                tap += part;
            }
            acc += tap;
        }
    }
    out[o] = acc * alpha[f];
}

// Real-valued convolution, one thread per output, any shape: fp32 products summed per tap over the
// channels, the taps' sums added up after (short adder chains).
__global__ __launch_bounds__(256) void conv_fp32_direct_kernel(const float *__restrict__ I,
                                                               const float *__restrict__ Wt, Geom g,
                                                               long long total, float *__restrict__ out)
{
    const long long o = (long long)blockIdx.x * 256 + threadIdx.x;
    if (o >= total) return;
    const int ox = (int)(o % g.OW);
    long long t = o / g.OW;
    const int oy = (int)(t % g.OH);
    t /= g.OH;
    const int f = (int)(t % g.F);
    const long long n = t / g.F;
    const size_t HW = (size_t)g.H * g.W;
    const int taps = g.kh * g.kw;
    const float *img = I + n * g.C * HW;
    const float *flt = Wt + (size_t)f * g.C * taps;
    float acc = 0.f;
    for (int ky = 0; ky < g.kh; ++ky) {
        const int iy = oy * g.sh - g.ph + ky;
        if (iy < 0 || iy >= g.H) continue;
        for (int kx = 0; kx < g.kw; ++kx) {
            const int ix = ox * g.sw - g.pw + kx;
            if (ix < 0 || ix >= g.W) continue;
            const float *src = img + (size_t)iy * g.W + ix;
            const float *w = flt + ky * g.kw + kx;
            float tap = 0.f;
            for (int c0 = 0; c0 < g.C; c0 += 32) {
                const int cn = min(32, g.C - c0);
                float part = 0.f;
                for (int j = 0; j < cn; ++j) part += src[(size_t)(c0 + j) * HW] * w[(size_t)(c0 + j) * taps];
                tap += part;
            }
            acc += tap;
        }
    }
    out[o] = acc;
}

// Real-valued convolution for images of few channels (the shape of Tables I-III), unit stride
// along x: a thread owns four consecutive outputs of one row of one filter plane, reads the KW + 3
// inputs under them once per (channel, filter row) and stores 16 bytes.  The arithmetic is two
// orders of magnitude below the memory traffic at these shapes; what matters is one coalesced
// pass over the image and one over the output.
template <int KW>
__global__ __launch_bounds__(256) void conv_fp32_rows_kernel(const float *__restrict__ I,
                                                             const float *__restrict__ Wt, Geom g,
                                                             int xgroups, long long total,
                                                             float *__restrict__ out)
{
    const long long o = (long long)blockIdx.x * 256 + threadIdx.x;
    if (o >= total) return;
    const int xg = (int)(o % xgroups);
    long long t = o / xgroups;
    const int oy = (int)(t % g.OH);
    t /= g.OH;
    const int f = (int)(t % g.F);
    const long long n = t / g.F;
    const int ox0 = 4 * xg, ix0 = ox0 - g.pw;
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    for (int c = 0; c < g.C; ++c) {
        const float *plane = I + (n * g.C + c) * (long long)g.H * g.W;
        const float *w = Wt + ((long long)f * g.C + c) * g.kh * KW;
        for (int ky = 0; ky < g.kh; ++ky) {
            const int iy = oy * g.sh - g.ph + ky;
            if (iy < 0 || iy >= g.H) continue;
            const float *row = plane + (long long)iy * g.W;
            float v[KW + 3];
#pragma unroll
            for (int i = 0; i < KW + 3; ++i) {
                const int ix = ix0 + i;
                v[i] = (ix >= 0 && ix < g.W) ? row[ix] : 0.f;
            }
#pragma unroll
            for (int kx = 0; kx < KW; ++kx) {
                const float wk = w[ky * KW + kx];
#pragma unroll
                for (int i = 0; i < 4; ++i) acc[i] += v[i + kx] * wk;
            }
        }
    }
    float *dst = out + ((n * g.F + f) * g.OH + oy) * (long long)g.OW + ox0;
    if (ox0 + 3 < g.OW && (g.OW & 3) == 0) {
        *reinterpret_cast<float4 *>(dst) = make_float4(acc[0], acc[1], acc[2], acc[3]);
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (ox0 + i < g.OW) dst[i] = acc[i];
    }
}

struct Plan {
    bool ok, ahead;
    int tiles, chan, rows_max, pitch;
    size_t lds;
};

Plan make_plan(const Geom &g, bool realw = false)
{
    Plan pl{};
    // LDS behind the staged input rows: one word per (tap, filter), or the chunk's fp32 weights
    auto filter_lds = [&](int chan) -> size_t {
        return realw ? (size_t)g.kh * g.kw * chan * kWPitch * 4 : (size_t)g.kh * g.kw * kFiltersPerWg * 4;
    };
    const long long OHW = (long long)g.OH * g.OW;
    if (g.kh * g.kw > 64 || OHW > (1 << 24) || (long long)g.C * g.H * g.W >= (1LL << 30)) return pl;
    pl.pitch = g.W + 2 * g.pw;
    // Pixel tiles per workgroup.  The matrix pipe of a compute unit is shared by the workgroups on
    // it, so a launch takes about ceil(workgroups / 256 CUs) x (tiles per workgroup + a fixed
    // per-workgroup cost of about one tile), and a compute unit with a single workgroup (one wave
    // per SIMD) cannot hide its own stalls, which counts like a second one: take the tile count
    // that minimises that, tiles shared out evenly over the image's workgroups; ties go to more
    // tiles (more reuse of each A operand).
    const int total = (int)((OHW + 31) / 32);
    int most = 1;
    long long best = -1;
    for (int t = 1; t <= std::min(kMaxTiles, total); ++t) {
        const int groups = ceil_div(total, t), even = ceil_div(total, groups);
        const long long blocks = (long long)g.N * ceil_div(g.F, kFiltersPerWg) * groups;
        const long long cost = std::max<long long>(2, (blocks + 255) / 256) * (even + 1);
        if (best < 0 || cost <= best) { best = cost; most = even; }
    }
    for (int tiles = most; tiles >= 1; --tiles) {
        // 32*tiles consecutive pixels span at most this many output rows
        const int orows = (int)std::min<long long>(g.OH, (32LL * tiles + g.OW - 2) / g.OW + 1);
        const int rows = (orows - 1) * g.sh + g.kh;
        // no more channels per chunk than the layer has (rounded up to 8)
        for (int chan = g.C > 16 ? 32 : g.C > 8 ? 16 : 8; chan >= 8; chan /= 2) {
            const size_t lds = (size_t)chan * rows * pl.pitch * 4 + filter_lds(chan);
            const long long elems = (long long)chan * rows * pl.pitch;      // staged values per chunk
            if (lds <= kLdsBudget && elems <= (long long)kPre * kThreads && elems < (1 << 16)) {
                pl.ok = true; pl.ahead = true; pl.tiles = tiles; pl.chan = chan; pl.rows_max = rows; pl.lds = lds;
                return pl;
            }
        }
    }
    // wide rows: the same search without the register limit (the kernel then stages synchronously)
    for (int tiles = most; tiles >= 1; --tiles) {
        const int orows = (int)std::min<long long>(g.OH, (32LL * tiles + g.OW - 2) / g.OW + 1);
        const int rows = (orows - 1) * g.sh + g.kh;
        for (int chan = g.C > 16 ? 32 : g.C > 8 ? 16 : 8; chan >= 8; chan /= 2) {
            const size_t lds = (size_t)chan * rows * pl.pitch * 4 + filter_lds(chan);
            if (lds <= kLdsWide) {
                pl.ok = true; pl.ahead = false; pl.tiles = tiles; pl.chan = chan; pl.rows_max = rows; pl.lds = lds;
                return pl;
            }
        }
    }
    return pl;
}

}  // namespace

bool bwn_mfma_supports(const Geom &g) { return make_plan(g).ok; }
bool conv_fp32_mfma_supports(const Geom &g) { return make_plan(g, true).ok; }

namespace {

template <bool REALW>
hipError_t launch_mfma_form(const float *I, const uint32_t *Wpk, const float *Wt, const float *alpha,
                            const Geom &g, float *out, hipStream_t st)
{
    const Plan pl = make_plan(g, REALW);
    if (!pl.ok) return hipErrorInvalidValue;
    BwnParams p;
    p.I = I; p.Wpk = Wpk; p.Wt = Wt; p.alpha = alpha; p.out = out;
    p.N = g.N; p.C = g.C; p.H = g.H; p.W = g.W; p.F = g.F; p.kh = g.kh; p.kw = g.kw;
    p.sh = g.sh; p.sw = g.sw; p.ph = g.ph; p.pw = g.pw; p.OH = g.OH; p.OW = g.OW; p.Cw = g.Cw;
    p.tiles = pl.tiles; p.chan = pl.chan; p.rows_max = pl.rows_max; p.pitch = pl.pitch;
    const long long OHW = (long long)g.OH * g.OW;
    p.inv_plane = reciprocal((unsigned long long)pl.rows_max * pl.pitch);
    p.inv_pitch = reciprocal((unsigned long long)pl.pitch);
    p.inv_per = reciprocal((unsigned long long)pl.chan * g.kh * g.kw);
    p.inv_taps = reciprocal((unsigned long long)g.kh * g.kw);
    p.w4 = REALW && pl.chan == 8 && g.C % 8 == 0 && g.kh * g.kw <= kPreW4 &&
           (reinterpret_cast<uintptr_t>(Wt) & 15) == 0;
    p.groups = ceil_div(OHW, 32LL * pl.tiles);
    p.fgroups = ceil_div(g.F, kFiltersPerWg);
    const long long blocks = (long long)g.N * p.groups * p.fgroups;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    if (pl.ahead) {
        bwn_mfma_kernel<true, REALW><<<dim3((unsigned)blocks), dim3(kThreads), pl.lds, st>>>(p);
    } else {
        if (pl.lds > 64 * 1024) {
            // raise the kernel's dynamic-LDS limit once per device (one flag set per instance)
            static std::atomic<unsigned long long> raised{0};
            int dev = 0;
            if (hipGetDevice(&dev) != hipSuccess) return hipGetLastError();
            const unsigned long long bit = 1ull << (dev & 63);
            if (!(raised.load() & bit)) {
                const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&bwn_mfma_kernel<false, REALW>),
                                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsWide);
                if (e != hipSuccess) return e;
                raised.fetch_or(bit);
            }
        }
        bwn_mfma_kernel<false, REALW><<<dim3((unsigned)blocks), dim3(kThreads), pl.lds, st>>>(p);
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_bwn_mfma(const float *I, const uint32_t *Wpk, const float *alpha, const Geom &g,
                           float *out, hipStream_t st)
{
    return launch_mfma_form<false>(I, Wpk, nullptr, alpha, g, out, st);
}

hipError_t launch_conv_fp32_mfma(const float *I, const float *Wt, const Geom &g, float *out, hipStream_t st)
{
    return launch_mfma_form<true>(I, nullptr, Wt, nullptr, g, out, st);
}

hipError_t launch_conv_fp32_direct(const float *I, const float *Wt, const Geom &g, float *out, hipStream_t st)
{
    // few channels, unit stride along x, an odd window of up to 7 columns, output 16-byte aligned:
    // four outputs per thread
    if (g.C <= 4 && g.sw == 1 && (g.kw == 1 || g.kw == 3 || g.kw == 5 || g.kw == 7) &&
        (reinterpret_cast<uintptr_t>(out) & 15) == 0) {
        const int xgroups = ceil_div(g.OW, 4);
        const long long total4 = (long long)g.N * g.F * g.OH * xgroups;
        const unsigned blocks = (unsigned)ceil_div(total4, 256);
        switch (g.kw) {
            case 1: conv_fp32_rows_kernel<1><<<blocks, 256, 0, st>>>(I, Wt, g, xgroups, total4, out); break;
            case 3: conv_fp32_rows_kernel<3><<<blocks, 256, 0, st>>>(I, Wt, g, xgroups, total4, out); break;
            case 5: conv_fp32_rows_kernel<5><<<blocks, 256, 0, st>>>(I, Wt, g, xgroups, total4, out); break;
            default: conv_fp32_rows_kernel<7><<<blocks, 256, 0, st>>>(I, Wt, g, xgroups, total4, out); break;
        }
        return hipGetLastError();
    }
    const long long total = (long long)g.N * g.F * g.OH * g.OW;
    conv_fp32_direct_kernel<<<ceil_div(total, 256), 256, 0, st>>>(I, Wt, g, total, out);
    return hipGetLastError();
}

hipError_t launch_bwn_direct(const float *I, const uint32_t *Wpk, const float *alpha, const Geom &g,
                             float *out, hipStream_t st)
{
    const long long total = (long long)g.N * g.F * g.OH * g.OW;
    bwn_direct_kernel<<<ceil_div(total, 256), 256, 0, st>>>(I, Wpk, alpha, g, total, out);
    return hipGetLastError();
}

}  // namespace xnor
