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
#include <atomic>

#include "xnor_internal.hpp"

namespace xnor {
namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int kWM = 2;            // 32-filter tiles per wave
constexpr int kWN = 4;            // 32-pixel tiles per wave (at most)
constexpr int kBandPixels = 2 * 32 * kWN;   // 2 wave columns
constexpr int kFilterTile = 2 * 32 * kWM;   // 2 wave rows
constexpr int kRing = 4;          // register ring of filter operands: loads run kRing-1 steps ahead
constexpr int kPatchPitch = 36;    // floats per row of a wave's 32x32 output patch in LDS (144 bytes)
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
    int chunk_steps; // k-steps the workspace holds per (filter tile, chunk): taps*CH/2 rounded up to
                     // the ring depth, plus one ring of zero steps for the prefetch overrun
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

// Filter words -> FP4 in A-operand order: Wx[tile32][chunk][step][lane] (one uint4 per lane).
// Within a chunk the steps run tap-major: step = tap * steps_c + s, packed word = chunk*CH + 2*s +
// lane/32, filter = 32*tile32 + lane%32; so the MFMA loop walks the workspace linearly.  Steps past
// taps*steps_c (padding up to chunk_steps), filters >= F, words >= Cw and channels >= C are zeros.
__global__ __launch_bounds__(256) void expand_filters_kernel(const uint32_t *__restrict__ Wpk,
                                                             uint4 *__restrict__ Wx, int F, int C,
                                                             int Cw, int taps, int CH, int nchunks,
                                                             int chunk_steps, int Cw2, long long total)
{
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    const int lane = (int)(i & 63);
    long long t = i >> 6;
    const int step = (int)(t % chunk_steps);
    t /= chunk_steps;
    const int chunk = (int)(t % nchunks);
    const int tile = (int)(t / nchunks);
    const int steps_c = min(CH, Cw2 - chunk * CH) >> 1;
    uint4 e = make_uint4(0, 0, 0, 0);
    if (step < taps * steps_c) {
        const int tap = step / steps_c, s = step - tap * steps_c;
        const int f = tile * 32 + (lane & 31);
        const int w = chunk * CH + 2 * s + (lane >> 5);
        if (f < F && w < Cw) {
            const int nvalid = min(32, C - 32 * w);
            e = expand_word(Wpk[((long long)f * taps + tap) * Cw + w], nvalid);
        }
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

// One LDS channel chunk: for every tap and every 64-channel step, NTW pixel tiles x kWM filter
// tiles of MFMAs.  The loop body has no branches: the filter operands are read linearly from the
// workspace through a register ring (loads run kRing-1 steps ahead; the workspace is zero-padded to
// a whole number of rings plus one), the pixel operands come from LDS one step ahead, and the
// (tap, step) cursor of the pixel operand advances with selects.
template <int NTW>
__device__ __forceinline__ void contract_chunk(const MfmaParams &p, const uint4 *lds,
                                               const uint4 *const (&Achunk)[kWM],
                                               const uint32_t (&baseB)[kWN], v16f (&acc)[kWM][kWN],
                                               int steps)
{
    constexpr int D = kRing;
    static_assert(D % 2 == 0, "the unrolled body alternates two pixel-operand buffers");
    const int T = p.kh * p.kw * steps;

    int l_off = 0;
    uint4 abuf[D][kWM];
    auto load_a = [&](uint4 (&dst)[kWM]) {
#pragma unroll
        for (int i = 0; i < kWM; ++i) dst[i] = Achunk[i][l_off];
        l_off += 64;
    };
#pragma unroll
    for (int u = 0; u < D - 1; ++u) load_a(abuf[u]);

    // pixel-operand cursor: offset of (tap, step) from the lane's slot, in 16-byte units; past the
    // last tap it parks on tap 0 (those steps multiply zero filter operands)
    int b_s = 0, b_kx = 0, b_ky = 0;
    uint32_t b_off = 0;
    uint4 bbuf[2][NTW];
    auto load_b = [&](uint4 (&dst)[NTW]) {
#pragma unroll
        for (int j = 0; j < NTW; ++j) dst[j] = lds[baseB[j] + b_off];
        ++b_s;
        const bool wrap_s = b_s == steps;
        b_s = wrap_s ? 0 : b_s;
        b_kx += wrap_s ? 1 : 0;
        const bool wrap_x = b_kx == p.kw;
        b_kx = wrap_x ? 0 : b_kx;
        b_ky += wrap_x ? 1 : 0;
        const uint32_t tap_off = b_ky < p.kh ? (uint32_t)((b_ky * p.Wp + b_kx) * p.pitch16) : 0u;
        b_off = wrap_s ? tap_off : b_off + 2;
    };
    load_b(bbuf[0]);

    for (int t = 0; t < T; t += D) {
#pragma unroll
        for (int u = 0; u < D; ++u) {
            load_a(abuf[(u + D - 1) % D]);
            load_b(bbuf[(u + 1) % 2]);
#pragma unroll
            for (int i = 0; i < kWM; ++i) {
                const uint4 va = abuf[u][i];
                const v8i a = v8i{(int)va.x, (int)va.y, (int)va.z, (int)va.w, 0, 0, 0, 0};
#pragma unroll
                for (int j = 0; j < NTW; ++j) {
                    const uint4 vb = bbuf[u % 2][j];
                    const v8i b = v8i{(int)vb.x, (int)vb.y, (int)vb.z, (int)vb.w, 0, 0, 0, 0};
                    acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(
                        a, b, acc[i][j], 4, 4, 0, kScaleOne, 0, kScaleOne);
                }
            }
            // Pin the accumulators between steps (an empty volatile asm that "modifies" them):
            // left free, the compiler interleaves the MFMAs of all unrolled steps and runs out of
            // registers for the operands it then has to keep alive.
#pragma unroll
            for (int i = 0; i < kWM; ++i)
#pragma unroll
                for (int j = 0; j < NTW; ++j) asm volatile("" : "+v"(acc[i][j]));
        }
    }
}

template <int VW>
__global__ __launch_bounds__(256, 2) void conv_mfma_kernel(MfmaParams p)
{
    extern __shared__ uint4 lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform, kept in an SGPR
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
#pragma unroll
    for (int j = 0; j < kWN; ++j) {
        const int q = (tile0 + j) * 32 + l32;
        const int qq = (j < my_nt && q < npix) ? q : 0;   // idle lanes read pixel 0 and store nothing
        const int Rl = qq / p.OW, ox = qq - Rl * p.OW;
        const int R = R0 + Rl;
        const int n = R / p.OH, oy = R - n * p.OH;
        const int srow = (n == n_first) ? (oy - oy0) * p.sh
                                        : r0 + (n - n_first - 1) * p.RHfull + oy * p.sh;
        baseB[j] = (uint32_t)((srow * p.Wp + ox * p.sw) * p.pitch16 + kg);
    }

    const uint4 *Aptr[kWM];   // this lane's filter operands, chunk 0, step 0
#pragma unroll
    for (int i = 0; i < kWM; ++i) {
        const int tile = blockIdx.y * (2 * kWM) + wm * kWM + i;
        Aptr[i] = p.Wx + ((long long)tile * p.nchunks * p.chunk_steps) * 64 + lane;
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
        // every wave with work runs all kWN tiles; tiles past the band's end read slot 0 and are
        // never stored (one code path keeps the accumulators out of scratch)
        if (my_nt > 0) {
            const uint4 *Achunk[kWM];
#pragma unroll
            for (int i = 0; i < kWM; ++i) Achunk[i] = Aptr[i] + (long long)c * p.chunk_steps * 64;
            contract_chunk<kWN>(p, lds, Achunk, baseB, acc, steps);
        }
    }

    // ---- step 3: out = float(dot) * K * alpha ----
    // The MFMA result has pixels along lanes and filters along registers, which would make every
    // store a 4-byte-per-lane instruction.  Each wave instead passes its 32x32 tiles through a
    // private LDS patch and reads them back with four consecutive pixels of one filter per lane,
    // so that one store instruction writes eight 128-byte runs (16 bytes per lane).
    __syncthreads();   // all waves are done with the staged input
    const float *__restrict__ Kp = p.K;
    const float *__restrict__ alphap = p.alpha;
    float *__restrict__ outp = p.out;
    int32_t *__restrict__ dotp = p.dot;
    float *patch = reinterpret_cast<float *>(lds) + wave * (32 * kPatchPitch);
    const int p4 = (lane & 7) * 4;      // first of this lane's four pixels within a tile
    const int fl = lane >> 3;           // filter within a tile, plus 8*k
    if (my_nt > 0) {
#pragma unroll
        for (int j = 0; j < kWN; ++j) {
            if (j >= my_nt) break;
            // the lane's pixel quad: position, validity, contiguity
            const int q0 = (tile0 + j) * 32 + p4;
            const int nv = min(4, npix - q0);                 // valid pixels of the quad (may be <= 0)
            const int qc = nv > 0 ? q0 : 0;
            const int Rl = qc / p.OW, ox = qc - Rl * p.OW;
            const int R = R0 + Rl;
            const int n = R / p.OH, oy = R - n * p.OH;
            const int po = oy * p.OW + ox;                    // offset inside the (n, f) plane
            const bool quad = nv == 4 && po + 3 < OHW;        // four pixels of one image: one 16-byte run
            const long long kbase = (long long)R * p.OW + ox; // K is dense over (n, oy, ox)
            float kq[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) kq[e] = e < nv ? Kp[kbase + e] : 0.0f;
            const long long obase = (long long)n * p.F * OHW + po;
#pragma unroll
            for (int i = 0; i < kWM; ++i) {
                const int f_tile = (blockIdx.y * (2 * kWM) + wm * kWM + i) * 32;
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    patch[((r >> 2) * 8 + kg * 4 + (r & 3)) * kPatchPitch + l32] = acc[i][j][r];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const int f = f_tile + fl + 8 * k;
                    const float4 d = *reinterpret_cast<const float4 *>(&patch[(fl + 8 * k) * kPatchPitch + p4]);
                    if (f >= p.F || nv <= 0) continue;
                    const float al = alphap[f];
                    const long long o = obase + (long long)f * OHW;
                    const float dd[4] = {d.x, d.y, d.z, d.w};
                    if (quad) {
                        *reinterpret_cast<float4 *>(outp + o) =
                            make_float4(d.x * (kq[0] * al), d.y * (kq[1] * al), d.z * (kq[2] * al), d.w * (kq[3] * al));
                        if (dotp)
                            *reinterpret_cast<int4 *>(dotp + o) = make_int4((int)d.x, (int)d.y, (int)d.z, (int)d.w);
                    } else {
                        // quad cut by the band's end or by an image boundary: pixel by pixel
                        for (int e = 0; e < nv; ++e) {
                            const int Re = (int)((kbase + e) / p.OW), oxe = (int)((kbase + e) - (long long)Re * p.OW);
                            const int ne = Re / p.OH, oye = Re - ne * p.OH;
                            const long long oe = ((long long)ne * p.F + f) * OHW + oye * p.OW + oxe;
                            outp[oe] = dd[e] * (kq[e] * al);
                            if (dotp) dotp[oe] = (int32_t)dd[e];
                        }
                    }
                }
            }
        }
    }
}

// Tiling chosen on the host for one layer.
struct MfmaPlan {
    bool ok;
    int TH, Wp, RHfull, S2, CH, nchunks, pitch16, slots_max, vw, chunk_steps;
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
    pl.lds_bytes = std::max(pl.lds_bytes, (size_t)4 * 32 * kPatchPitch * sizeof(float));   // output patches
    if ((long long)slots * pl.CH >= (1 << 20)) return pl;   // fast-division range
    const uintptr_t ip = reinterpret_cast<uintptr_t>(Ipk);
    pl.vw = (g.Cw % 4 == 0 && pl.CH % 4 == 0 && (ip & 15) == 0) ? 4
          : (g.Cw % 2 == 0 && (ip & 7) == 0)                    ? 2 : 1;
    pl.f_tiles = ceil_div(g.F, kFilterTile);
    pl.chunk_steps = (g.kh * g.kw * (pl.CH / 2) + kRing - 1) / kRing * kRing + kRing;
    pl.ws_bytes = (size_t)pl.f_tiles * (kFilterTile / 32) * pl.nchunks * pl.chunk_steps * 64 * sizeof(uint4);
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
    expand_filters_kernel<<<ceil_div(wx_items, 256), 256, 0, st>>>(
        Wpk, Wx, g.F, g.C, g.Cw, taps, pl.CH, pl.nchunks, pl.chunk_steps, 2 * pl.S2, wx_items);
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
    p.chunk_steps = pl.chunk_steps;
    p.dCHV = make_fastdiv(pl.CH / pl.vw);
    p.dWp = make_fastdiv(pl.Wp);
    p.dRH = make_fastdiv(pl.RHfull);

    const dim3 grid(ceil_div(p.total_rows, pl.TH), pl.f_tiles);
    auto launch = [&](auto kernel) -> hipError_t {
        // raise the kernel's dynamic-LDS limit to the hardware maximum once per device (the call
        // is slow on the host); one flag set per template instance
        static std::atomic<unsigned long long> raised{0};
        int dev = 0;
        hipError_t err = hipGetDevice(&dev);
        if (err != hipSuccess) return err;
        const unsigned long long bit = 1ull << (dev & 63);
        if (!(raised.load(std::memory_order_acquire) & bit)) {
            err = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsMax);
            if (err != hipSuccess) return err;
            raised.fetch_or(bit, std::memory_order_release);
        }
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
