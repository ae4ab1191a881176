// XNOR convolution on the matrix cores (Sec. III-A steps 1b-1d and 3, Eq. 11).
//
// The sign dot product of Eq. 11 is a dense contraction over (tap, channel), so it maps onto MFMA.
// CDNA4's block-scaled MFMA takes FP4 (E2M1) operands at twice the FP8/int8 rate; +1, -1 and 0 are
// exact in FP4 (codes 0x2, 0xA, 0x0) and the fp32 accumulator holds every partial sum (an integer
// below 2^24) exactly, so the result equals N_valid - 2*popcount(Ipk xor Wpk) bit for bit.
//   * bit 1 -> +1.0, bit 0 -> -1.0 (step 1c: a 0 bit stands for -1)
//   * out-of-image taps, channels >= C and filters >= F are FP4 zeros: they add nothing, which is
//     the zero padding of the +-1 tensor -- no border correction is needed
//
// v_mfma_scale_f32_32x32x64_f8f6f4, D[32x32] += A[32x64] * B[64x32], FP4 operands (4 VGPRs each):
//   A: lane l holds row l%32, k = 32*(l/32) .. +31      -> one packed channel word of one filter
//   B: lane l holds col l%32, k = 32*(l/32) .. +31      -> one packed channel word of one pixel
//   D: lane l, register r holds row 8*(r/4) + 4*(l/32) + r%4, col l%32
// Rows are filters and columns are pixels, so one store instruction writes 32 consecutive pixels of
// a filter plane (128 contiguous bytes) per half-wave.
//
// Work split: a workgroup (4 waves as 2x2) owns a "band" of TH consecutive output rows of the
// batch (rows of all images numbered n*OH+oy; a band may run across image boundaries, each image
// segment gets its own halo rows) times 64*WM filters.  The band's input rows are expanded from
// bits to FP4 once into LDS, zero-filled where they fall outside the image, in a slot-per-pixel
// layout whose pitch is an odd number of 16-byte units (conflict-free ds_read_b128).  A lane's
// B operand for tap (ky,kx) then sits at its pixel's slot + (ky*Wp+kx) slots: no per-tap bounds
// logic.  Filter words are expanded once per call into a workspace laid out in A-operand order
// and stream from L2 straight into registers.
#include <algorithm>

#include "xnor_internal.hpp"

namespace xnor {
namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int kWM = 2;            // 32-filter tiles per wave
constexpr int kWN = 4;            // 32-pixel tiles per wave (at most)
constexpr int kBandPixels = 2 * 32 * kWN;   // 2 wave columns
constexpr int kFilterTile = 2 * 32 * kWM;   // 2 wave rows
constexpr int kScaleOne = 0x7f7f7f7f;       // E8M0 exponent 127 = 2^0

// q = n / d for n*d < 2^32 via one mul_hi.
struct FastDiv {
    uint32_t mul, d;
};
FastDiv make_fastdiv(uint32_t d) { return FastDiv{d == 1 ? 0u : (uint32_t)(((1ull << 32) + d - 1) / d), d}; }
__device__ inline uint32_t fdiv(uint32_t n, FastDiv f) { return f.d == 1 ? n : __umulhi(n, f.mul); }

struct MfmaParams {
    const uint32_t *Ipk;
    const uint4 *Wx;
    const float *K, *alpha;
    float *out;
    int32_t *dot;
    int N, C, H, W, F, kh, kw, sh, sw, ph, pw, OH, OW, Cw;
    int TH;          // output rows (of the whole batch) per band
    int total_rows;  // N*OH
    int Wp;          // staged columns per input row  = (OW-1)*sw + kw
    int RHfull;      // staged rows of a whole image  = (OH-1)*sh + kh
    int S2;          // k-steps (64 channels) per tap over all channels
    int CH;          // packed words per LDS channel chunk (even)
    int nchunks;
    int pitch16;     // LDS slot pitch in 16-byte units (CH + 1, odd)
    FastDiv dCHV, dWp, dRH;
};

// 8 sign bits -> 8 FP4 codes (bit 1 -> 0x2 = +1.0, bit 0 -> 0xA = -1.0); channel i -> nibble i.
// Two bits select one byte of a four-entry table through v_perm_b32.
__device__ inline uint32_t expand8(uint32_t b)
{
    uint32_t t = b | (b << 6);
    t |= t << 12;
    t &= 0x03030303u;
    return __builtin_amdgcn_perm(0u, 0x222AA2AAu, t);
}

// One packed word -> 32 FP4 values; `nvalid` channels are real, the rest become FP4 zero.
__device__ inline uint4 expand_word(uint32_t w, int nvalid)
{
    uint4 e;
    e.x = expand8(w & 0xffu);
    e.y = expand8((w >> 8) & 0xffu);
    e.z = expand8((w >> 16) & 0xffu);
    e.w = expand8(w >> 24);
    if (nvalid < 32) {
        auto m = [&](int d) -> uint32_t {
            const int nv = nvalid - 8 * d;
            return nv >= 8 ? 0xffffffffu : (nv <= 0 ? 0u : ((1u << (4 * nv)) - 1u));
        };
        e.x &= m(0); e.y &= m(1); e.z &= m(2); e.w &= m(3);
    }
    return e;
}

// Filter words -> FP4 in A-operand order: Wx[tile32][tap][step][lane] (one uint4 per lane), lane l
// = filter 32*tile32 + l%32, packed word 2*step + l/32.  Filters >= F, words >= Cw and channels
// >= C come out as zeros.
__global__ __launch_bounds__(256) void expand_filters_kernel(const uint32_t *__restrict__ Wpk,
                                                             uint4 *__restrict__ Wx, int F, int C,
                                                             int Cw, int taps, int S2, long long total)
{
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    const int lane = (int)(i & 63);
    long long t = i >> 6;
    const int step = (int)(t % S2);
    t /= S2;
    const int tap = (int)(t % taps);
    const int tile = (int)(t / taps);
    const int f = tile * 32 + (lane & 31);
    const int w = 2 * step + (lane >> 5);
    uint4 e = make_uint4(0, 0, 0, 0);
    if (f < F && w < Cw) {
        const int nvalid = min(32, C - 32 * w);
        e = expand_word(Wpk[((long long)f * taps + tap) * Cw + w], nvalid);
    }
    Wx[i] = e;
}

template <int VW>
struct WordVec;
template <>
struct WordVec<1> { typedef uint32_t type; };
template <>
struct WordVec<2> { typedef uint2 type; };
template <>
struct WordVec<4> { typedef uint4 type; };

template <int VW>
__global__ __launch_bounds__(256, 2) void conv_mfma_kernel(MfmaParams p)
{
    extern __shared__ uint4 lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, kg = lane >> 5;
    const int OHW = p.OH * p.OW;

    // ---- the band: TH rows of the batch's output rows, numbered R = n*OH + oy ----
    const int R0 = blockIdx.x * p.TH;
    const int rows = min(p.TH, p.total_rows - R0);
    const int npix = rows * p.OW;
    const int n_first = R0 / p.OH, oy0 = R0 - n_first * p.OH;
    const int r0 = (p.OH - 1 - oy0) * p.sh + p.kh;   // staged rows of the first image if it runs to its end
    const int R_last = R0 + rows - 1;
    const int n_last = R_last / p.OH, oy_last = R_last - n_last * p.OH;
    const int srows = (n_last == n_first) ? (oy_last - oy0) * p.sh + p.kh
                                          : r0 + (n_last - n_first - 1) * p.RHfull + oy_last * p.sh + p.kh;
    const int nslots = srows * p.Wp;

    // ---- this wave's pixel tiles; the band's tiles are split evenly over the two wave columns ----
    const int NT = (npix + 31) >> 5;
    const int nt0 = (NT + 1) >> 1;
    const int tile0 = wn ? nt0 : 0;
    const int my_nt = wn ? NT - nt0 : nt0;

    uint32_t baseB[kWN];   // LDS index (16-byte units) of the lane's pixel, tap (0,0), k-group kg
    bool pix_ok[kWN];
    int img[kWN], pixoff[kWN], kidx[kWN];
#pragma unroll
    for (int j = 0; j < kWN; ++j) {
        const int q = (tile0 + j) * 32 + l32;
        pix_ok[j] = (j < my_nt) && (q < npix);
        const int qq = pix_ok[j] ? q : 0;
        const int Rl = qq / p.OW, ox = qq - Rl * p.OW;
        const int R = R0 + Rl;
        const int n = R / p.OH, oy = R - n * p.OH;
        const int srow = (n == n_first) ? (oy - oy0) * p.sh
                                        : r0 + (n - n_first - 1) * p.RHfull + oy * p.sh;
        baseB[j] = (uint32_t)((srow * p.Wp + ox * p.sw) * p.pitch16 + kg);
        img[j] = n;
        pixoff[j] = oy * p.OW + ox;
        kidx[j] = R * p.OW + ox;
    }

    const int taps = p.kh * p.kw;
    const uint4 *Aptr[kWM];
#pragma unroll
    for (int i = 0; i < kWM; ++i) {
        const int tile = blockIdx.y * (2 * kWM) + wm * kWM + i;
        Aptr[i] = p.Wx + ((long long)tile * taps * p.S2) * 64 + lane;
    }

    v16f acc[kWM][kWN];
#pragma unroll
    for (int i = 0; i < kWM; ++i)
#pragma unroll
        for (int j = 0; j < kWN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    const int CHV = p.CH / VW;
    const int items = nslots * CHV;
    const int Cw2 = 2 * p.S2;

    for (int c = 0; c < p.nchunks; ++c) {
        const int w_base = c * p.CH;
        const int steps = min(p.CH, Cw2 - w_base) >> 1;
        if (c > 0) __syncthreads();   // everyone is done reading the previous chunk

        // ---- stage: packed input words of the band's rows -> FP4 in LDS, zeros outside the image ----
        constexpr int U = 4;
        for (int base = 0; base < items; base += 256 * U) {
            typename WordVec<VW>::type v[U];
            int dst[U];
            bool live[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int it = base + u * 256 + tid;
                const bool in_range = it < items;
                const uint32_t itc = in_range ? (uint32_t)it : 0u;
                const uint32_t slot = fdiv(itc, p.dCHV);
                const int wq = (int)(itc - slot * CHV);
                const uint32_t rowg = fdiv(slot, p.dWp);
                const int col = (int)(slot - rowg * p.Wp);
                int n, iy;
                if ((int)rowg < r0) {
                    n = n_first;
                    iy = oy0 * p.sh - p.ph + (int)rowg;
                } else {
                    const uint32_t t = rowg - (uint32_t)r0;
                    const uint32_t sg = fdiv(t, p.dRH);
                    n = n_first + 1 + (int)sg;
                    iy = (int)(t - sg * p.RHfull) - p.ph;
                }
                const int ix = col - p.pw;
                const int w = w_base + wq * VW;
                live[u] = in_range && n < p.N && iy >= 0 && iy < p.H && ix >= 0 && ix < p.W && w < p.Cw;
                dst[u] = in_range ? (int)(slot * p.pitch16 + wq * VW) : -1;
                typename WordVec<VW>::type z = {};
                v[u] = z;
                if (live[u])
                    v[u] = *reinterpret_cast<const typename WordVec<VW>::type *>(
                        p.Ipk + (((long long)n * p.H + iy) * p.W + ix) * p.Cw + w);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (dst[u] < 0) continue;
                // outside the image (or past the last channel word) the FP4 image is 0.0, not -1.0
                uint32_t words[VW];
                if constexpr (VW == 1) { words[0] = v[u]; }
                if constexpr (VW == 2) { words[0] = v[u].x; words[1] = v[u].y; }
                if constexpr (VW == 4) { words[0] = v[u].x; words[1] = v[u].y; words[2] = v[u].z; words[3] = v[u].w; }
#pragma unroll
                for (int k = 0; k < VW; ++k)
                    lds[dst[u] + k] = live[u] ? expand_word(words[k], 32) : make_uint4(0, 0, 0, 0);
            }
        }
        __syncthreads();

        // ---- contract: taps x 64-channel steps ----
        for (int ky = 0; ky < p.kh; ++ky)
            for (int kx = 0; kx < p.kw; ++kx) {
                const int tap = ky * p.kw + kx;
                const uint32_t tapoff = (uint32_t)((ky * p.Wp + kx) * p.pitch16);
                const long long a_off = ((long long)tap * p.S2 + (w_base >> 1)) * 64;
                for (int s = 0; s < steps; ++s) {
                    v8i a[kWM], b[kWN];
#pragma unroll
                    for (int i = 0; i < kWM; ++i) {
                        const uint4 t = Aptr[i][a_off + (long long)s * 64];
                        a[i] = v8i{(int)t.x, (int)t.y, (int)t.z, (int)t.w, 0, 0, 0, 0};
                    }
#pragma unroll
                    for (int j = 0; j < kWN; ++j) {
                        if (j < my_nt) {
                            const uint4 t = lds[baseB[j] + tapoff + 2 * s];
                            b[j] = v8i{(int)t.x, (int)t.y, (int)t.z, (int)t.w, 0, 0, 0, 0};
                        }
                    }
#pragma unroll
                    for (int i = 0; i < kWM; ++i)
#pragma unroll
                        for (int j = 0; j < kWN; ++j)
                            if (j < my_nt)
                                acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(
                                    a[i], b[j], acc[i][j], 4, 4, 0, kScaleOne, 0, kScaleOne);
                }
            }
    }

    // ---- step 3: out = float(dot) * K * alpha; lanes run along pixels, registers along filters ----
#pragma unroll
    for (int j = 0; j < kWN; ++j) {
        if (!pix_ok[j]) continue;
        const float kv = p.K[kidx[j]];
#pragma unroll
        for (int i = 0; i < kWM; ++i) {
            const int f_base = (blockIdx.y * (2 * kWM) + wm * kWM + i) * 32 + kg * 4;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int f = f_base + (r >> 2) * 8 + (r & 3);
                if (f < p.F) {
                    const long long o = ((long long)img[j] * p.F + f) * OHW + pixoff[j];
                    const float d = acc[i][j][r];
                    p.out[o] = d * (kv * p.alpha[f]);
                    if (p.dot) p.dot[o] = (int32_t)d;
                }
            }
        }
    }
}

// Tiling chosen on the host for one layer.
struct MfmaPlan {
    bool ok;
    int TH, Wp, RHfull, S2, CH, nchunks, pitch16, slots_max, vw;
    size_t lds_bytes, ws_bytes;
    int f_tiles;   // workgroup rows of kFilterTile filters
};

constexpr size_t kLdsTwoPerCU = 80 * 1024;
constexpr size_t kLdsMax = 160 * 1024;

MfmaPlan make_plan(const Geom &g, const void *Ipk)
{
    MfmaPlan pl{};
    pl.ok = false;
    if (g.OW > kBandPixels) return pl;   // a band is at least one whole output row
    const long long total_rows = (long long)g.N * g.OH;
    pl.TH = (int)std::min<long long>(total_rows, kBandPixels / g.OW);
    const long long wp = (long long)(g.OW - 1) * g.sw + g.kw, rh = (long long)(g.OH - 1) * g.sh + g.kh;
    if (wp > 4096 || rh > 4096) return pl;   // keeps the staging index math inside the fast-division range
    pl.Wp = (int)wp;
    pl.RHfull = (int)rh;
    const int Cw2 = (g.Cw + 1) & ~1;
    pl.S2 = Cw2 / 2;
    // most staged rows any band can need: try every starting row of an image
    long long max_rows = 0;
    for (int oy0 = 0; oy0 < g.OH; ++oy0) {
        const long long r0 = (long long)(g.OH - 1 - oy0) * g.sh + g.kh;
        const long long last = (long long)oy0 + std::min<long long>(pl.TH, total_rows) - 1;
        const long long n_last = last / g.OH, oy_last = last % g.OH;
        const long long sr = n_last == 0 ? (oy_last - oy0) * g.sh + g.kh
                                         : r0 + (n_last - 1) * rh + oy_last * g.sh + g.kh;
        max_rows = std::max(max_rows, sr);
    }
    const long long slots = max_rows * wp;
    if (slots > (1 << 16)) return pl;
    pl.slots_max = (int)slots;
    // fewest channel chunks whose staged band fits the LDS budget (two workgroups per CU if possible)
    auto fit = [&](size_t budget) -> bool {
        for (int nch = 1; nch <= pl.S2; ++nch) {
            const int CH = 2 * ((pl.S2 + nch - 1) / nch);
            const size_t bytes = (size_t)slots * (CH + 1) * 16;
            if (bytes <= budget) {
                pl.CH = CH;
                pl.nchunks = (Cw2 + CH - 1) / CH;
                pl.pitch16 = CH + 1;
                pl.lds_bytes = bytes;
                return true;
            }
        }
        return false;
    };
    if (!fit(kLdsTwoPerCU) && !fit(kLdsMax)) return pl;
    if ((long long)slots * pl.CH >= (1 << 20)) return pl;   // fast-division range
    const uintptr_t ip = reinterpret_cast<uintptr_t>(Ipk);
    pl.vw = (g.Cw % 4 == 0 && pl.CH % 4 == 0 && (ip & 15) == 0) ? 4
          : (g.Cw % 2 == 0 && (ip & 7) == 0)                    ? 2 : 1;
    pl.f_tiles = ceil_div(g.F, kFilterTile);
    pl.ws_bytes = (size_t)pl.f_tiles * (kFilterTile / 32) * g.kh * g.kw * pl.S2 * 64 * sizeof(uint4);
    if (ceil_div(total_rows, pl.TH) > 0x7fffffffLL || pl.f_tiles > 65535) return pl;
    pl.ok = true;
    return pl;
}

}  // namespace

bool conv_mfma_supports(const Geom &g)
{
    return make_plan(g, nullptr).ok;
}

size_t conv_mfma_workspace_bytes(const Geom &g)
{
    const MfmaPlan pl = make_plan(g, nullptr);
    return pl.ok ? pl.ws_bytes : 0;
}

hipError_t launch_conv_mfma(const uint32_t *Ipk, const uint32_t *Wpk, const float *K,
                            const float *alpha, const Geom &g, float *out, int32_t *dot,
                            void *workspace, hipStream_t st)
{
    const MfmaPlan pl = make_plan(g, Ipk);
    if (!pl.ok) return hipErrorInvalidValue;
    const int taps = g.kh * g.kw;

    // filters -> FP4 in A-operand order (per call: the library keeps no state)
    uint4 *Wx = static_cast<uint4 *>(workspace);
    const long long wx_items = (long long)(pl.ws_bytes / sizeof(uint4));
    expand_filters_kernel<<<ceil_div(wx_items, 256), 256, 0, st>>>(Wpk, Wx, g.F, g.C, g.Cw, taps,
                                                                   pl.S2, wx_items);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;

    MfmaParams p{};
    p.Ipk = Ipk; p.Wx = Wx; p.K = K; p.alpha = alpha; p.out = out; p.dot = dot;
    p.N = g.N; p.C = g.C; p.H = g.H; p.W = g.W; p.F = g.F; p.kh = g.kh; p.kw = g.kw;
    p.sh = g.sh; p.sw = g.sw; p.ph = g.ph; p.pw = g.pw; p.OH = g.OH; p.OW = g.OW; p.Cw = g.Cw;
    p.TH = pl.TH;
    p.total_rows = g.N * g.OH;
    p.Wp = pl.Wp; p.RHfull = pl.RHfull; p.S2 = pl.S2; p.CH = pl.CH; p.nchunks = pl.nchunks;
    p.pitch16 = pl.pitch16;
    p.dCHV = make_fastdiv(pl.CH / pl.vw);
    p.dWp = make_fastdiv(pl.Wp);
    p.dRH = make_fastdiv(pl.RHfull);

    const dim3 grid(ceil_div(p.total_rows, pl.TH), pl.f_tiles);
    auto launch = [&](auto kernel) -> hipError_t {
        hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                             hipFuncAttributeMaxDynamicSharedMemorySize,
                                             (int)pl.lds_bytes);
        if (err != hipSuccess) return err;
        kernel<<<grid, 256, pl.lds_bytes, st>>>(p);
        return hipGetLastError();
    };
    switch (pl.vw) {
        case 4: return launch(conv_mfma_kernel<4>);
        case 2: return launch(conv_mfma_kernel<2>);
        default: return launch(conv_mfma_kernel<1>);
    }
}

}  // namespace xnor
