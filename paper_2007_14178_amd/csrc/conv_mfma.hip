// XNOR convolution on the matrix cores (Sec. III-A steps 1b-1d and 3, Eq. 11).
//
// The sign dot product of Eq. 11 is a dense contraction over (tap, channel), so it maps onto MFMA.
// CDNA4's f8f6f4 MFMA takes FP4 (E2M1) operands at twice the FP8/int8 rate; +1, -1 and 0 are
// exact in FP4 (codes 0x2, 0xA, 0x0) and the fp32 accumulator holds every partial sum (an integer
// below 2^24) exactly, so the result equals N_valid - 2*popcount(Ipk xor Wpk) bit for bit.
//   * bit 1 -> +1.0, bit 0 -> -1.0 (step 1c: a 0 bit stands for -1)
//   * out-of-image taps, channels >= C and filters >= F are FP4 zeros: they add nothing, which is
//     the zero padding of the +-1 tensor -- no border correction is needed
//
// v_mfma_f32_32x32x64_f8f6f4 (the form without block scales: no scale operands to read),
// D[32x32] += A[32x64] * B[64x32], FP4 operands (cbsz:4 blgp:4, 4 VGPRs each):
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
#include <type_traits>

#include "conv_mfma_common.hpp"

namespace xnor {
namespace {

struct MfmaParams {
    const uint32_t *Ipk;
    const uint4 *Wx;
    const float *K, *alpha;
    const float *A;  // if not null: K is not given but formed here from A (second half of Eq. 10)
    float *out;
    int32_t *dot;
    uint32_t *Opk;   // chained form: packed signs of the output [N][OH][OW][Cwn] ...
    float *P;        // ... and per (pixel, filter tile) sums of |out| [N*OH*OW][f_tiles]
    int Cwn, f_tiles;
    int N, C, H, W, F, kh, kw, sh, sw, ph, pw, OH, OW, Cw;
    int TH;          // output rows (of the whole batch) per band
    int total_rows;  // N*OH
    int Wp;          // staged columns per input row  = (OW-1)*sw + kw
    int RHfull;      // staged rows of a whole image  = (OH-1)*sh + kh
    int S2;          // k-steps (64 channels) per tap over all channels
    int CH;          // packed words per LDS channel chunk (even)
    int nchunks;
    int pitch16;     // LDS slot pitch in 16-byte units (CH + 1, odd)
    int buf16;       // distance between the two LDS chunk buffers in 16-byte units (0: one buffer)
    int kl16;        // start of the K / alpha area in LDS (16-byte units): behind the step table
    int tab16;       // start of the step-offset table in LDS (16-byte units)
    int tab_len;     // its uint32 entries: one per step of the tile, a multiple of 4
    int chunk_pad;   // steps per chunk in the workspace and the table (a whole number of rings)
    int ragged;      // the last chunk has fewer than CH words
    int near_out;    // a band's outputs lie within 2^31 bytes of its first image's first filter plane of a tile
    int tile_steps;  // k-steps the workspace holds per filter tile: every chunk padded to a whole
                     // number of rings, plus one ring of zero steps for the prefetch overrun
    FastDiv dCHV, dWp, dRH;
    FastDiv dOW, dOH;   // for a pixel of the band (below 2^9) and a row counted from the band's first image (below 2^13)
    int nbands, bands_per_xcd;
};

// Filter words -> FP4 in A-operand order: Wx[tile32][step][lane] (one uint4 per lane).  The steps
// of a tile run chunk-major, then tap-major, each chunk padded with zero steps to a whole number of
// register rings: step = chunk*chunk_pad + tap*steps_c + s, packed word = chunk*CH + 2*s + lane/32,
// filter = 32*tile32 + lane%32 -- exactly the order in which the MFMA loop consumes them, so it
// walks the workspace linearly.  Padding steps, filters >= F, words >= Cw and channels >= C are zeros.
__global__ __launch_bounds__(256) void expand_filters_kernel(const uint32_t *__restrict__ Wpk,
                                                             uint4 *__restrict__ Wx, int F, int C,
                                                             int Cw, int taps, int CH, int nchunks,
                                                             int chunk_pad, int tile_steps, int Cw2,
                                                             long long total)
{
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    const int lane = (int)(i & 63);
    const long long t = i >> 6;
    const int step = (int)(t % tile_steps);
    const int tile = (int)(t / tile_steps);
    ExpandLayout L;
    L.ok = 1; L.CH = CH; L.nchunks = nchunks; L.chunk_pad = chunk_pad; L.tile_steps = tile_steps; L.Cw2 = Cw2;
    L.ws_bytes = 0;
    const int f = tile * 32 + (lane & 31);
    uint4 e = make_uint4(0, 0, 0, 0);
    if (f < F)
        e = expanded_entry(L, step, lane >> 5, taps, Cw, C,
                           [&](int tap, int w) { return Wpk[((long long)f * taps + tap) * Cw + w]; });
    Wx[i] = e;
}

// The kernel.  Per workgroup: the band's input words are expanded to FP4 into LDS one channel
// chunk at a time, double-buffered: while the MFMA loop runs on chunk c, the words of chunk c+1
// are fetched (at the chunk's start) and expanded into the other buffer (half-way through), so
// that only chunk 0 is staged with the matrix cores idle.  The MFMA loop is one flat loop over
// all (chunk, tap, 64-channel step) of the tile; the filter operands stream linearly from the
// workspace through a register ring that runs kRing-1 steps ahead across chunk boundaries; the
// pixel operands come from LDS one step ahead.
template <int VW, bool CHAIN>
__global__ __launch_bounds__(256, 2) void conv_mfma_kernel(MfmaParams p)
{
    extern __shared__ uint4 lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform, kept in an SGPR
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, kg = lane >> 5;
    const int OHW = p.OH * p.OW;

    // ---- which (band, filter tile): workgroups are handed to the 8 XCDs round-robin by their id,
    // and each XCD has its own L2.  XCD x takes a contiguous range of bands and runs through them
    // once per filter tile, so that a band's input rows (and its neighbours' shared halo rows) are
    // fetched into that one L2 once and found there by the other filter tiles' workgroups.
    const int xcd = blockIdx.x & (kXcds - 1);
    const int seq = blockIdx.x >> kXcdShift;
    // (a division by a run-time value goes through the vector ALU: bring the wave-uniform quotient
    // back into a scalar register, or everything derived from it occupies vector registers)
    const int ftile = __builtin_amdgcn_readfirstlane(seq / p.bands_per_xcd);
    const int band = xcd * p.bands_per_xcd + (seq - ftile * p.bands_per_xcd);
    if (band >= p.nbands) return;   // padding of the last XCD's range (uniform over the workgroup)

    // ---- the band: TH rows of the batch's output rows, numbered R = n*OH + oy ----
    const int R0 = band * p.TH;
    const int rows = min(p.TH, p.total_rows - R0);
    const int npix = rows * p.OW;
    const int n_first = __builtin_amdgcn_readfirstlane(R0 / p.OH), oy0 = R0 - n_first * p.OH;
    const int r0 = (p.OH - 1 - oy0) * p.sh + p.kh;   // staged rows of the first image if it runs to its end
    const int dn_last = (int)fdiv((uint32_t)(oy0 + rows - 1), p.dOH);   // (uniform)
    const int n_last = n_first + dn_last, oy_last = oy0 + rows - 1 - dn_last * p.OH;
    const int srows = (n_last == n_first) ? (oy_last - oy0) * p.sh + p.kh
                                          : r0 + (n_last - n_first - 1) * p.RHfull + oy_last * p.sh + p.kh;
    const int nslots = srows * p.Wp;

    // ---- this wave's pixel tiles; the band's tiles are split evenly over the two wave columns ----
    const int NT = (npix + 31) >> 5;
    const int nt0 = (NT + 1) >> 1;
    const int tile0 = wn ? nt0 : 0;
    const int my_nt = wn ? NT - nt0 : nt0;

    // ---- staging: packed input words of the band's rows -> FP4 in LDS, zeros outside the image ----
    typedef typename WordVec<VW>::type wvec;
    const int CHV = p.CH / VW;
    const int items = nslots * CHV;          // one item = VW consecutive words of one slot
    const int Cw2 = 2 * p.S2;
    constexpr int UP = 2;                    // items per thread fetched ahead into registers
    wvec sv[UP];
    // all offsets into Ipk are taken from the band's first image (32 bits are enough, see make_plan)
    const uint32_t *const band_base = p.Ipk + (long long)n_first * p.H * p.W * p.Cw;

    // where item `it` of chunk `c` comes from (word offset from band_base) and goes to
    auto locate = [&](int it, int c, int &dst, bool &live) -> uint32_t {
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
            const uint32_t tt = rowg - (uint32_t)r0;
            const uint32_t sg = fdiv(tt, p.dRH);
            n = n_first + 1 + (int)sg;
            iy = (int)(tt - sg * p.RHfull) - p.ph;
        }
        const int ix = col - p.pw;
        const int w = c * p.CH + wq * VW;
        live = in_range && n < p.N && iy >= 0 && iy < p.H && ix >= 0 && ix < p.W && w < p.Cw;
        dst = in_range ? (int)(slot * p.pitch16 + wq * VW) : -1;
        return live ? (uint32_t)((((n - n_first) * p.H + iy) * p.W + ix) * p.Cw + w) : 0u;
    };
    // VW words at byte offset `off_b` from band_base into `v`.  The load is an asm statement so that
    // the compiler keeps no count of it: its own wait for these words (vmcnt(0), it knows of no
    // younger loads) would drain the filter-operand ring of the MFMA loop; stage_commit waits with
    // the right count instead.  "+v": the load lands in the register that holds a dead item's zeros.
    auto fetch_words = [&](wvec &v, uint32_t off_b) {
        if constexpr (VW == 4)
            asm volatile("global_load_dwordx4 %0, %1, %2" : "+v"(v) : "v"(off_b), "s"(band_base));
        else if constexpr (VW == 2)
            asm volatile("global_load_dwordx2 %0, %1, %2" : "+v"(v) : "v"(off_b), "s"(band_base));
        else
            asm volatile("global_load_dword %0, %1, %2" : "+v"(v) : "v"(off_b), "s"(band_base));
    };
    // one item's words -> FP4 at byte offset `dst_b` of a chunk buffer; a dead item is FP4 zeros
    // (outside the image, or past the last channel word, the +-1 tensor is 0.0, not -1.0)
    char *const lds_bytes = reinterpret_cast<char *>(lds);
    auto put = [&](uint32_t buf_b, uint32_t dst_b, bool live, const wvec &v) {
        uint32_t words[VW];
        if constexpr (VW == 1) { words[0] = v; }
        if constexpr (VW == 2) { words[0] = v.x; words[1] = v.y; }
        if constexpr (VW == 4) { words[0] = v.x; words[1] = v.y; words[2] = v.z; words[3] = v.w; }
        uint4 *dst = reinterpret_cast<uint4 *>(lds_bytes + buf_b + dst_b);
        if (live) {
#pragma unroll
            for (int k = 0; k < VW; ++k) dst[k] = expand_word(words[k], 32);
        } else {
#pragma unroll
            for (int k = 0; k < VW; ++k) dst[k] = make_uint4(0, 0, 0, 0);
        }
    };
    // A thread's first UP items are the same slots in every chunk, a chunk only shifts the source
    // by its first word: per item two registers are kept across the MFMA loop, the byte offset of
    // its words in chunk 0 (kDead: slot outside every image) and where it goes in a chunk buffer
    // (byte offset | first word within the chunk << 18; kNoItem: the thread has no such item).
    constexpr uint32_t kDead = 0xffffffffu, kNoItem = 0xffffffffu;
    uint32_t soff[UP], spk[UP];
#pragma unroll
    for (int u = 0; u < UP; ++u) {
        const int it = u * 256 + tid;
        int dst;
        bool live0;
        const uint32_t off = locate(it, 0, dst, live0);
        const uint32_t w0 = it < items ? ((uint32_t)it - fdiv((uint32_t)it, p.dCHV) * CHV) * VW : 0u;
        soff[u] = live0 ? off * 4u : kDead;   // (a word past Cw in chunk 0 is past Cw in every chunk)
        spk[u] = dst < 0 ? kNoItem : ((uint32_t)dst * 16u) | (w0 << 18);
    }
    // chunks whose word range is cut by Cw exist only if CH does not divide Cw
    auto item_live = [&](int u, int c) -> bool {
        return soff[u] != kDead && (!p.ragged || c * p.CH + (int)(spk[u] >> 18) < p.Cw);
    };
    auto stage_issue = [&](int c) {
#pragma unroll
        for (int u = 0; u < UP; ++u) {
            wvec z = {};
            sv[u] = z;
            if (item_live(u, c)) fetch_words(sv[u], soff[u] + (uint32_t)(c * p.CH) * 4u);
        }
    };
    // `in_loop`: called from inside the MFMA loop at least kRing steps after stage_issue, i.e. with
    // at least 2*kRing filter-operand loads issued after the words were fetched (loads return in
    // order); otherwise everything in flight is waited for.  `zero_dead`: dead items are written
    // (as zeros) too; slots outside the image stay zero from the first fill of either buffer, so
    // later chunks skip them unless channel words can die with the chunk (p.ragged).
    auto stage_commit = [&](int c, uint32_t buf_b, bool in_loop, bool zero_dead) {
        static_assert(UP == 2, "the wait below names both fetched items");
        // (the words pass through the asm: their expansion cannot move above the wait)
        if (in_loop) asm volatile("s_waitcnt vmcnt(6)" : "+v"(sv[0]), "+v"(sv[1]));
        else asm volatile("s_waitcnt vmcnt(0)" : "+v"(sv[0]), "+v"(sv[1]));
#pragma unroll
        for (int u = 0; u < UP; ++u) {
            if (spk[u] == kNoItem) continue;
            const bool live = item_live(u, c);
            if (live || zero_dead) put(buf_b, spk[u] & 0x3ffffu, live, sv[u]);
        }
        for (int it = UP * 256 + tid; it < items; it += 256) {   // bands with more items: fetched here
            int dst;
            bool live;
            const uint32_t off = locate(it, c, dst, live);
            wvec z = {};
            wvec v = z;
            if (live) fetch_words(v, off * 4u);
            asm volatile("s_waitcnt vmcnt(0)" : "+v"(v));   // (this drains the MFMA loop's ring too)
            put(buf_b, (uint32_t)dst * 16u, live, v);
        }
    };
    // the band's K values and this workgroup's 128 alphas go to LDS for the last phase: fetched
    // here, written once the staged words have been waited for anyway
    float *const Kl = reinterpret_cast<float *>(lds + p.kl16);   // [kBandPixels], zeros past the band
    float *const Al = Kl + kBandPixels;                            // [kFilterTile], zeros past F
    // Fetch first, compute afterwards: the first chunk's words, the filter operands of steps 0..2,
    // K and alpha are requested here; the table, the lane's LDS addresses and the accumulators are
    // set up while those loads are in flight.
    stage_issue(0);
    float k_mine = 0.0f, a_mine = 0.0f;
    if (tid < npix) {
        if (p.A) {
            // K of this band's pixel `tid` from the channel mean A: the same sum, order and rounding
            // as the stand-alone box filter (double accumulation over the in-image taps, one divide)
            const int Rl = (int)fdiv((uint32_t)tid, p.dOW), ox = tid - Rl * p.OW;
            const int dn = (int)fdiv((uint32_t)(oy0 + Rl), p.dOH);
            const int n = n_first + dn, oy = oy0 + Rl - dn * p.OH;
            const float *a = p.A + (long long)n * p.H * p.W;
            // no branches around the loads (out-of-image taps read a clamped address and add 0), so
            // that the unrolled loop has all its loads in flight at once
            double sum = 0.0;
            const int iy0 = oy * p.sh - p.ph, ix0 = ox * p.sw - p.pw;
            int ky = 0, kx = 0;
#pragma unroll 9
            for (int t = 0; t < p.kh * p.kw; ++t) {
                const int iy = iy0 + ky, ix = ix0 + kx;
                const bool in = (unsigned)iy < (unsigned)p.H && (unsigned)ix < (unsigned)p.W;
                const float v = a[in ? iy * p.W + ix : 0];
                sum += in ? (double)v : 0.0;
                if (++kx == p.kw) { kx = 0; ++ky; }
            }
            k_mine = (float)(sum / (double)(p.kh * p.kw));
        } else {
            k_mine = p.K[(long long)R0 * p.OW + tid];
        }
    }
    if (tid < kFilterTile && ftile * kFilterTile + tid < p.F) a_mine = p.alpha[ftile * kFilterTile + tid];
    v4i A[kRing][kWM];
    uint32_t a_off = (uint32_t)lane * 16u;   // byte offset of this lane's operand of the next step to load
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint4 *)lds;
    uint32_t bB[kWN];   // LDS byte address of the lane's pixel, tap (0,0), k-group kg
#pragma unroll
    for (int j = 0; j < kWN; ++j) {
        const int q = (tile0 + j) * 32 + l32;
        const int qq = (j < my_nt && q < npix) ? q : 0;   // idle lanes read pixel 0 and store nothing
        const int Rl = (int)fdiv((uint32_t)qq, p.dOW), ox = qq - Rl * p.OW;
        const int dn = (int)fdiv((uint32_t)(oy0 + Rl), p.dOH);
        const int n = n_first + dn, oy = oy0 + Rl - dn * p.OH;
        const int srow = (n == n_first) ? (oy - oy0) * p.sh
                                        : r0 + (n - n_first - 1) * p.RHfull + oy * p.sh;
        bB[j] = lds_base + (uint32_t)((srow * p.Wp + ox * p.sw) * p.pitch16 + kg) * 16u;
    }

    const uint4 *Abase[kWM];   // filter operands of this wave's tiles, step 0 (wave-uniform)
#pragma unroll
    for (int i = 0; i < kWM; ++i) {
        const int tile = ftile * (2 * kWM) + wm * kWM + i;
        Abase[i] = p.Wx + ((long long)tile * p.tile_steps) * 64;
    }

    v16f acc[kWM][kWN];
#pragma unroll
    for (int i = 0; i < kWM; ++i)
#pragma unroll
        for (int j = 0; j < kWN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    // ring fill: filter operands of steps 0..2 (ordinary loads; the compiler waits for them at the pins)
#pragma unroll
    for (int u = 0; u < kRing - 1; ++u) {
#pragma unroll
        for (int i = 0; i < kWM; ++i)
            A[u][i] = *reinterpret_cast<const v4i *>(reinterpret_cast<const char *>(Abase[i]) + a_off);
        a_off += 1024;
    }
    // The pixel operand of step t sits at (chunk buffer, tap(t), step-in-tap(t)) from the lane's
    // slot.  That offset is the same for every lane, so it is tabulated once per workgroup in LDS
    // (one entry per step of the tile in workspace order, in bytes) instead of being tracked with
    // scalar arithmetic in the MFMA loop; zero-padded steps and the prefetch overrun point at tap 0.
    uint32_t *const table = reinterpret_cast<uint32_t *>(lds + p.tab16);
    for (int tt = tid; tt < p.tab_len; tt += 256) {
        const int c = min(tt / p.chunk_pad, p.nchunks - 1), t = tt - c * p.chunk_pad;
        const int steps_c = min(p.CH, Cw2 - c * p.CH) >> 1;
        uint32_t off = (uint32_t)((c & 1) * p.buf16);   // 16-byte units here, bytes in the table
        if (t < p.kh * p.kw * steps_c) {
            const int tap = t / steps_c, s = t - tap * steps_c;
            const int ky = tap / p.kw, kx = tap - ky * p.kw;
            off += (uint32_t)((ky * p.Wp + kx) * p.pitch16 + 2 * s);
        }
        table[tt] = off * 16u;
    }
    stage_commit(0, 0u, false, true);
    Kl[tid] = k_mine;
    if (tid < kFilterTile) Al[tid] = a_mine;
    if (p.nchunks > 1) {
        // the second buffer's slots outside the image: zero once, no chunk writes them again
#pragma unroll
        for (int u = 0; u < UP; ++u)
            if (spk[u] != kNoItem && soff[u] == kDead) {
                wvec z = {};
                put((uint32_t)p.buf16 * 16u, spk[u] & 0x3ffffu, false, z);
            }
    }
    __syncthreads();

    // ---- contract ----
    // The steady-state loop is written as a fixed sequence of single-instruction asm statements
    // (volatile, so they stay in this order) with its own s_waitcnt counts: left to the compiler's
    // scheduler the operand loads end up right in front of the MFMAs that use them and a lone wave
    // then waits out every LDS and L2 latency with the matrix pipe idle.  Per 64-channel step and
    // wave: 8 MFMAs; between them the 4 pixel-operand reads for the NEXT step (LDS, ~7 MFMAs =
    // 220 cycles ahead of their first use), the table entry two steps ahead, and the 2 filter-
    // operand loads for the step THREE ahead (L2, ring of kRing register sets).
    //   LDS queue order per step:  T, B0, B1, B2, B3   (returns are in order: lgkmcnt(3) before
    //                              the MFMA on Bj leaves the three younger requests in flight)
    //   VMEM order per step:       A0, A1 of step s+3  (vmcnt(5) before the first use of A0(s),
    //                              vmcnt(4) before A1(s))
    // The compiler does not know about loads issued inside asm statements, so nothing it emits may
    // sit between a load and the wait that covers it other than address arithmetic, and every
    // register with a load in flight stays an operand of a later statement until it is drained.
    constexpr int D = kRing;
    static_assert(D == 4, "the wait counts below are written for a ring of four");
    const int taps = p.kh * p.kw;

#define XNOR_MFMA(ACC, A, B)                                                                         \
    asm volatile("v_mfma_f32_32x32x64_f8f6f4 %0, %1, %2, %0 cbsz:4 blgp:4" \
                 : "+v"(ACC) : "v"(A), "v"(B))
#define XNOR_LDS128(DST, ADDR) asm volatile("ds_read_b128 %0, %1" : "=v"(DST) : "v"(ADDR))
#define XNOR_LDS32(DST, ADDR, OFF) asm volatile("ds_read_b32 %0, %1 offset:" #OFF : "=v"(DST) : "v"(ADDR))
#define XNOR_GLD(DST, VOFF, SBASE, OFF) \
    asm volatile("global_load_dwordx4 %0, %1, %2 offset:" #OFF : "=v"(DST) : "v"(VOFF), "s"(SBASE))
#define XNOR_ADD(DST, X, Y) asm volatile("v_add_u32 %0, %1, %2" : "=v"(DST) : "v"(X), "v"(Y))
#define XNOR_WAIT(S) asm volatile("s_waitcnt " S)

    v4i B[2][kWN];

#pragma unroll
    for (int u = 0; u < D - 1; ++u)
#pragma unroll
        for (int i = 0; i < kWM; ++i) asm volatile("" : "+v"(A[u][i]));
#pragma unroll
    for (int i = 0; i < kWM; ++i) A[D - 1][i] = v4i{0, 0, 0, 0};

    for (int c = 0; c < p.nchunks; ++c) {
        const int steps = min(p.CH, Cw2 - c * p.CH) >> 1;   // 64-channel steps per tap in this chunk
        const int Tp = (taps * steps + D - 1) / D * D;       // steps incl. the zero padding of the workspace
        const bool more = c + 1 < p.nchunks;
        if (more) stage_issue(c + 1);                        // fetch the next chunk's words now ...
        bool committed = !more;

        // prime: table entries 0 and 1, then the pixel operands of step 0 (the loop's first wait
        // covers them)
        uint32_t boff[2], tmp[kWN];
        uint32_t tab_addr = lds_base + (uint32_t)(p.tab16 * 16 + c * p.chunk_pad * 4);
        XNOR_LDS32(boff[0], tab_addr, 0);
        XNOR_LDS32(boff[1], tab_addr, 4);
        tab_addr += 8;                                       // entry 2 is read in step 0
        asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(boff[0]), "+v"(boff[1]));
#pragma unroll
        for (int j = 0; j < kWN; ++j) {
            XNOR_ADD(tmp[j], bB[j], boff[0]);
            XNOR_LDS128(B[0][j], tmp[j]);
        }
        if (c == 0) {
#pragma unroll
            for (int j = 0; j < kWN; ++j) B[1][j] = v4i{0, 0, 0, 0};
        }

        for (int g = 0; g < Tp; g += D) {
#pragma unroll
            for (int u = 0; u < D; ++u) {
                // step s = g + u uses A[u], B[u%2]; loads B[(u+1)%2] for s+1 at boff[(u+1)%2],
                // table entry s+2 into boff[u%2], A[(u+3)%4] for s+3
                XNOR_WAIT("vmcnt(5) lgkmcnt(3)");
                XNOR_MFMA(acc[0][0], A[u][0], B[u % 2][0]);
                if (u == 0) XNOR_LDS32(boff[u % 2], tab_addr, 0);
                if (u == 1) XNOR_LDS32(boff[u % 2], tab_addr, 4);
                if (u == 2) XNOR_LDS32(boff[u % 2], tab_addr, 8);
                if (u == 3) XNOR_LDS32(boff[u % 2], tab_addr, 12);
                XNOR_ADD(tmp[0], bB[0], boff[(u + 1) % 2]);
                XNOR_WAIT("lgkmcnt(3)");
                XNOR_MFMA(acc[0][1], A[u][0], B[u % 2][1]);
                XNOR_LDS128(B[(u + 1) % 2][0], tmp[0]);
                XNOR_ADD(tmp[1], bB[1], boff[(u + 1) % 2]);
                XNOR_WAIT("lgkmcnt(3)");
                XNOR_MFMA(acc[0][2], A[u][0], B[u % 2][2]);
                XNOR_LDS128(B[(u + 1) % 2][1], tmp[1]);
                XNOR_ADD(tmp[2], bB[2], boff[(u + 1) % 2]);
                XNOR_WAIT("lgkmcnt(3)");
                XNOR_MFMA(acc[0][3], A[u][0], B[u % 2][3]);
                XNOR_LDS128(B[(u + 1) % 2][2], tmp[2]);
                XNOR_ADD(tmp[3], bB[3], boff[(u + 1) % 2]);
                XNOR_WAIT("vmcnt(4)");
                XNOR_MFMA(acc[1][0], A[u][1], B[u % 2][0]);
                XNOR_LDS128(B[(u + 1) % 2][3], tmp[3]);
                XNOR_MFMA(acc[1][1], A[u][1], B[u % 2][1]);
                if (u == 0) XNOR_GLD(A[(u + 3) % D][0], a_off, Abase[0], 0);
                if (u == 1) XNOR_GLD(A[(u + 3) % D][0], a_off, Abase[0], 1024);
                if (u == 2) XNOR_GLD(A[(u + 3) % D][0], a_off, Abase[0], 2048);
                if (u == 3) XNOR_GLD(A[(u + 3) % D][0], a_off, Abase[0], 3072);
                XNOR_MFMA(acc[1][2], A[u][1], B[u % 2][2]);
                if (u == 0) XNOR_GLD(A[(u + 3) % D][1], a_off, Abase[1], 0);
                if (u == 1) XNOR_GLD(A[(u + 3) % D][1], a_off, Abase[1], 1024);
                if (u == 2) XNOR_GLD(A[(u + 3) % D][1], a_off, Abase[1], 2048);
                if (u == 3) XNOR_GLD(A[(u + 3) % D][1], a_off, Abase[1], 3072);
                XNOR_MFMA(acc[1][3], A[u][1], B[u % 2][3]);
            }
            a_off += 4096;
            tab_addr += 16;
            // ... and expand them into the other buffer half-way through this chunk
            if (!committed && 2 * (g + D) >= Tp) {
                stage_commit(c + 1, (uint32_t)(((c + 1) & 1) * p.buf16) * 16u, true, p.ragged != 0);
                committed = true;
            }
        }
        // The reads issued for the step past the chunk's end land in B[0] / boff: drain them while
        // those registers are still operands, then they may be reused.
        asm volatile("s_waitcnt lgkmcnt(0)"
                     : "+v"(B[0][0]), "+v"(B[0][1]), "+v"(B[0][2]), "+v"(B[0][3]), "+v"(B[1][0]), "+v"(B[1][1]),
                       "+v"(B[1][2]), "+v"(B[1][3]), "+v"(boff[0]), "+v"(boff[1]));
        if (more) __syncthreads();   // chunk c+1 is complete in its buffer; chunk c's buffer is free
    }
    // the ring has run three (all-zero) steps ahead: let those loads land before the registers are reused
    asm volatile("s_waitcnt vmcnt(0)"
                 : "+v"(A[0][0]), "+v"(A[0][1]), "+v"(A[1][0]), "+v"(A[1][1]), "+v"(A[2][0]), "+v"(A[2][1]),
                   "+v"(A[3][0]), "+v"(A[3][1]));
#undef XNOR_MFMA
#undef XNOR_LDS128
#undef XNOR_LDS32
#undef XNOR_GLD
#undef XNOR_ADD
#undef XNOR_WAIT

    // ---- step 3: out = float(dot) * K * alpha ----
    __syncthreads();   // all waves are done with the staged input
    if constexpr (CHAIN) {
        // Chained form (the paper's closing proposal, Sec. V: hand the binary output to the next
        // layer without the conversion to real values).  The next layer needs of this output O only
        // sign(O) packed along its channels (= these filters) and the channel mean of |O| (Eq. 10).
        // Both come straight from the accumulators: lane l holds pixel l%32 of a tile and, in
        // register r, filter 8*(r/4) + 4*(l/32) + r%4, so a lane builds half of a 32-filter word,
        // its partner lane l^32 the other half.  o = float(dot) * (K * alpha) is formed exactly as
        // in the fp32 output, the bit is (o >= 0) and |o| is summed in double.
        int lane_c = lane;
        asm volatile("" : "+v"(lane_c));
        const int l32c = lane_c & 31, kgc = lane_c >> 5;
        const float *Kl = reinterpret_cast<const float *>(lds + p.kl16);
        const float *Al = Kl + kBandPixels;
        double *Ps = reinterpret_cast<double *>(lds);          // [2 wave rows][kBandPixels]
        float al[kWM][16];
#pragma unroll
        for (int i = 0; i < kWM; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) al[i][r] = Al[(wm * kWM + i) * 32 + 8 * (r >> 2) + 4 * kgc + (r & 3)];
#pragma unroll
        for (int j = 0; j < kWN; ++j) {
            if (j >= my_nt) break;
            const int q = (tile0 + j) * 32 + l32c;
            const bool valid = q < npix;
            const float kv = Kl[valid ? q : 0];
            double asum = 0.0;
            uint32_t word[kWM];
#pragma unroll
            for (int i = 0; i < kWM; ++i) {
                const int f_tile = (ftile * (2 * kWM) + wm * kWM + i) * 32;
                uint32_t w = 0;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int row = 8 * (r >> 2) + 4 * kgc + (r & 3);
                    const float o = acc[i][j][r] * (kv * al[i][r]);
                    if (f_tile + row < p.F) {              // bits and sums of filters that exist only
                        w |= (o >= 0.0f ? 1u : 0u) << row;
                        asum += (double)fabsf(o);
                    }
                }
                word[i] = w | (uint32_t)__shfl_xor((int)w, 32);
            }
            asum += __shfl_xor(asum, 32);
            if (valid && kgc == 0) {
                const long long pix = (long long)R0 * p.OW + q;      // pixels of a band are consecutive
#pragma unroll
                for (int i = 0; i < kWM; ++i) {
                    const int wi = ftile * (2 * kWM) + wm * kWM + i;
                    if (wi < p.Cwn) p.Opk[pix * p.Cwn + wi] = word[i];
                }
                Ps[wm * kBandPixels + q] = asum;
            }
        }
        __syncthreads();
        if (wm == 0) {
#pragma unroll
            for (int j = 0; j < kWN; ++j) {
                if (j >= my_nt) break;
                const int q = (tile0 + j) * 32 + l32c;
                if (q < npix && kgc == 0)
                    p.P[((long long)R0 * p.OW + q) * p.f_tiles + ftile] =
                        (float)(Ps[q] + Ps[kBandPixels + q]);
            }
        }
        return;
    }
    // fp32 output straight from the accumulators: lane l holds pixel l%32 of a tile and, in register
    // r, filter 8*(r/4) + 4*(l/32) + r%4, so one store instruction writes 32 consecutive pixels of
    // two filter planes (two 128-byte runs).  The band's K and the tile's alpha wait in LDS since
    // the kernel's start (no global-load latency here).  This phase is bound by its own instruction
    // stream (a wave issues its 128 stores one after the other), so a store costs two multiplies and
    // one 64-bit add: the address walks the lane's 16 filter planes (one plane on, after every
    // fourth five planes on) instead of being formed from the plane index each time, and tiles
    // whose 32 filters all exist (uniform per tile) carry no per-store predicate.
    float *__restrict__ outp = p.out;
    int32_t *__restrict__ dotp = p.dot;
    // lane-derived indices of this phase are formed from a copy of the lane id that the compiler
    // cannot see through, or it computes them at kernel start and holds them across the MFMA loop
    int lane_e = lane;
    asm volatile("" : "+v"(lane_e));
    const int l32e = lane_e & 31, kge = lane_e >> 5;
    float al[kWM][16];
#pragma unroll
    for (int i = 0; i < kWM; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) al[i][r] = Al[(wm * kWM + i) * 32 + 8 * (r >> 2) + 4 * kge + (r & 3)];
    const long long plane1 = (long long)OHW * 4, plane5 = 5 * plane1;   // bytes between filter planes
    // Per pixel tile of the wave: the lane's byte offset from (the band's first image, a filter
    // tile's first plane) to (its image, its 4*kg-th plane, its pixel), and its K.
    const int n_first_e = __builtin_amdgcn_readfirstlane(R0 / p.OH);
    long long lane_b[kWN];
    float kvs[kWN];
    bool lane_ok[kWN];
#pragma unroll
    for (int j = 0; j < kWN; ++j) {
        const int q = (tile0 + j) * 32 + l32e;                // pixel within the band
        lane_ok[j] = j < my_nt && q < npix;
        const int qq = lane_ok[j] ? q : 0;
        const int Rl = (int)fdiv((uint32_t)qq, p.dOW), ox = qq - Rl * p.OW;
        const int oy0_e = R0 - n_first_e * p.OH;
        const int dn = (int)fdiv((uint32_t)(oy0_e + Rl), p.dOH);
        const int n = n_first_e + dn, oy = oy0_e + Rl - dn * p.OH;
        kvs[j] = Kl[qq];
        lane_b[j] = (((long long)(n - n_first_e) * p.F + 4 * kge) * OHW + oy * p.OW + ox) * 4;
    }
    // tiles of this wave whose 32 pixels all exist (uniform): only the band's last tile can be ragged
    const int nfull = max(0, min(my_nt, (npix - tile0 * 32) >> 5));
    // One filter tile (32 planes) of the wave's pixel tiles.  While a band's outputs lie within
    // 2 GiB (p.near_out, decided on the host) a store is "scalar base + 32-bit lane offset": the
    // walk over the planes is scalar arithmetic and the vector ALU only multiplies.  The whole
    // tiles go plane by plane, the wave's tiles of one plane back to back: they are consecutive
    // pixels, so the cache lines that two tiles share are completed by consecutive stores.
    auto store_filter_tile = [&](auto *tile_base, int nfilt, auto value) {
        typedef typename std::remove_pointer<decltype(tile_base)>::type elem_t;
        typedef __attribute__((address_space(1))) elem_t *ptr_t;
        const bool all = nfilt >= 32;
        int first_slow = 0;
        if (p.near_out && all) {
            uint32_t v32[kWN];
#pragma unroll
            for (int j = 0; j < kWN; ++j) {
                v32[j] = (uint32_t)lane_b[j];
                asm volatile("" : "+v"(v32[j]));
            }
            const char *ub = reinterpret_cast<const char *>(tile_base);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
#pragma unroll
                for (int j = 0; j < kWN; ++j)
                    if (j < nfull) *(ptr_t)(ub + v32[j]) = value(j, r);
                ub += (r & 3) == 3 ? plane5 : plane1;
            }
            first_slow = nfull;
        }
        // ragged tiles, partial filter tiles, far outputs: one 64-bit vector add per store (a pointer
        // that has passed through an asm statement is a generic one to the compiler: the stores
        // name the address space)
#pragma unroll
        for (int j = 0; j < kWN; ++j) {
            if (j < first_slow || !lane_ok[j]) continue;
            char *pr = const_cast<char *>(reinterpret_cast<const char *>(tile_base)) + lane_b[j];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                if (all || 4 * kge + 8 * (r >> 2) + (r & 3) < nfilt) *(ptr_t)pr = value(j, r);
                pr += (r & 3) == 3 ? plane5 : plane1;
                asm volatile("" : "+v"(pr));   // (keeps the walk: one add per store)
            }
        }
    };
#pragma unroll
    for (int i = 0; i < kWM; ++i) {
        const int ft = (ftile * (2 * kWM) + wm * kWM + i) * 32;   // the tile's first filter (uniform)
        const int nfilt = p.F - ft;                                  // how many of its 32 exist
        const long long tile_el = ((long long)n_first_e * p.F + ft) * OHW;   // (uniform)
        store_filter_tile(outp + tile_el, nfilt,
                          [&](int j, int r) -> float { return acc[i][j][r] * (kvs[j] * al[i][r]); });
        if (dotp)
            store_filter_tile(dotp + tile_el, nfilt,
                              [&](int j, int r) -> int32_t { return (int32_t)acc[i][j][r]; });
    }
}

// Tiling chosen on the host for one layer.
struct MfmaPlan {
    bool ok;
    int TH, Wp, RHfull, S2, CH, nchunks, pitch16, buf16, tab16, tab_len, kl16, slots_max, vw, chunk_pad, tile_steps;
    size_t lds_bytes, ws_bytes;
    int f_tiles;   // workgroup rows of kFilterTile filters
};

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
    // Channel chunks: one chunk in one LDS buffer if the whole band fits, else the fewest chunks
    // whose two buffers (double buffering) fit; first within the budget that lets two workgroups
    // share a CU, then within all of LDS.  A chunk must span a few rings of steps so that the
    // "fetch next chunk / expand next chunk" hand-offs inside the MFMA loop stay in order.
    const int taps = g.kh * g.kw;
    auto fit = [&](size_t budget) -> bool {
        for (int nch = 1; nch <= pl.S2; ++nch) {
            const int CH = 2 * ((pl.S2 + nch - 1) / nch);
            const int nchunks = (Cw2 + CH - 1) / CH;
            const size_t one = (size_t)slots * (CH + 1) * 16;
            const long long chunk_pad = ((long long)taps * (CH / 2) + kRing - 1) / kRing * kRing;
            const long long tab_len = (nchunks * chunk_pad + kRing + 3) & ~3LL;   // = tile_steps, rounded up
            const size_t data = nchunks > 1 ? 2 * one : one;
            const size_t bytes = data + (size_t)tab_len * sizeof(uint32_t) + kKAlphaBytes;
            if (bytes <= budget) {
                pl.CH = CH;
                pl.nchunks = nchunks;
                pl.pitch16 = CH + 1;
                pl.buf16 = nchunks > 1 ? (int)(one / 16) : 0;
                pl.tab16 = (int)(data / 16);
                pl.tab_len = (int)tab_len;
                pl.lds_bytes = bytes;
                return true;
            }
        }
        return false;
    };
    if (!fit(kLdsTwoPerCU) && !fit(kLdsMax)) return pl;
    // K and alpha sit behind the staging area; the chained epilogue reuses the area's start for its
    // per-pixel sums (2 x kBandPixels doubles)
    const size_t ka_off = std::max(pl.lds_bytes - kKAlphaBytes, (size_t)2 * kBandPixels * sizeof(double));
    pl.kl16 = (int)(ka_off / 16);
    pl.lds_bytes = ka_off + kKAlphaBytes;
    if ((long long)slots * pl.CH >= (1 << 20)) return pl;   // fast-division range
    // staging addresses are 32-bit byte offsets from the band's first image
    if ((long long)(pl.TH / g.OH + 2) * g.H * g.W * g.Cw >= (1LL << 30)) return pl;
    const uintptr_t ip = reinterpret_cast<uintptr_t>(Ipk);
    pl.vw = (g.Cw % 4 == 0 && pl.CH % 4 == 0 && (ip & 15) == 0) ? 4
          : (g.Cw % 2 == 0 && (ip & 7) == 0)                    ? 2 : 1;
    pl.f_tiles = ceil_div(g.F, kFilterTile);
    pl.chunk_pad = (taps * (pl.CH / 2) + kRing - 1) / kRing * kRing;
    pl.tile_steps = pl.nchunks * pl.chunk_pad + kRing;
    pl.ws_bytes = (size_t)pl.f_tiles * (kFilterTile / 32) * pl.tile_steps * 64 * sizeof(uint4);
    // (bands padded to a multiple of 8) x filter tiles is the grid
    if ((ceil_div(total_rows, pl.TH) + 8) * pl.f_tiles > (1LL << 30)) return pl;
    pl.ok = true;
    return pl;
}

}  // namespace

// Which of the two kernels runs a layer (and so which workspace layout its filters take): the
// persistent one where it takes the shape and its rounds of items come out even enough (or this
// file's kernel does not take the shape), this file's one-workgroup-per-band kernel otherwise.
static bool use_persistent(const Geom &g)
{
    if (!conv_mfma_persistent_supports(g)) return false;
    return conv_mfma_persistent_preferred(g) || !make_plan(g, nullptr).ok;
}

bool conv_mfma_supports(const Geom &g)
{
    return use_persistent(g) || make_plan(g, nullptr).ok;
}

ExpandLayout conv_mfma_expand_layout(const Geom &g)
{
    if (use_persistent(g)) return conv_mfma_persistent_expand_layout(g);
    const MfmaPlan pl = make_plan(g, nullptr);   // the workspace layout does not depend on alignment
    ExpandLayout L{};
    L.ok = pl.ok ? 1 : 0;
    L.CH = pl.CH; L.nchunks = pl.nchunks; L.chunk_pad = pl.chunk_pad; L.tile_steps = pl.tile_steps;
    L.Cw2 = 2 * pl.S2; L.ws_bytes = pl.ws_bytes;
    return L;
}

static ExpandLayout bands_expand_layout(const Geom &g)
{
    const MfmaPlan pl = make_plan(g, nullptr);
    ExpandLayout L{};
    L.ok = pl.ok ? 1 : 0;
    L.CH = pl.CH; L.nchunks = pl.nchunks; L.chunk_pad = pl.chunk_pad; L.tile_steps = pl.tile_steps;
    L.Cw2 = 2 * pl.S2; L.ws_bytes = pl.ws_bytes;
    return L;
}

bool conv_mfma_bands_supports(const Geom &g)
{
    return make_plan(g, nullptr).ok;
}

// (enough for either kernel, so that a caller's one workspace serves whatever variant it asks for)
size_t conv_mfma_workspace_bytes(const Geom &g)
{
    const ExpandLayout L = conv_mfma_expand_layout(g);
    if (!L.ok) return 0;
    const ExpandLayout Lb = bands_expand_layout(g);
    return std::max(L.ws_bytes, Lb.ok ? Lb.ws_bytes : (size_t)0);
}

static hipError_t launch_expand_with(const ExpandLayout &L, const uint32_t *Wpk, const Geom &g, void *workspace,
                                     hipStream_t st)
{
    if (!L.ok) return hipErrorInvalidValue;
    const long long wx_items = (long long)(L.ws_bytes / sizeof(uint4));
    expand_filters_kernel<<<ceil_div(wx_items, 256), 256, 0, st>>>(
        Wpk, static_cast<uint4 *>(workspace), g.F, g.C, g.Cw, g.kh * g.kw, L.CH, L.nchunks, L.chunk_pad,
        L.tile_steps, L.Cw2, wx_items);
    return hipGetLastError();
}

hipError_t launch_expand_filters(const uint32_t *Wpk, const Geom &g, void *workspace, hipStream_t st)
{
    return launch_expand_with(conv_mfma_expand_layout(g), Wpk, g, workspace, st);
}

static hipError_t launch_mfma(const uint32_t *Ipk, const float *K, const float *A, const float *alpha,
                              const Geom &g, float *out, int32_t *dot, uint32_t *Opk, float *P,
                              const void *workspace, hipStream_t st, bool bands_kernel = false)
{
    if (!bands_kernel && use_persistent(g))
        return launch_conv_mfma_persistent(Ipk, K, A, alpha, g, out, dot, Opk, P, workspace, st);
    const MfmaPlan pl = make_plan(g, Ipk);
    if (!pl.ok) return hipErrorInvalidValue;
    const uint4 *Wx = static_cast<const uint4 *>(workspace);

    MfmaParams p{};
    p.Ipk = Ipk; p.Wx = Wx; p.K = K; p.A = A; p.alpha = alpha; p.out = out; p.dot = dot;
    p.Opk = Opk; p.P = P; p.Cwn = (g.F + 31) / 32; p.f_tiles = pl.f_tiles;
    p.N = g.N; p.C = g.C; p.H = g.H; p.W = g.W; p.F = g.F; p.kh = g.kh; p.kw = g.kw;
    p.sh = g.sh; p.sw = g.sw; p.ph = g.ph; p.pw = g.pw; p.OH = g.OH; p.OW = g.OW; p.Cw = g.Cw;
    p.TH = pl.TH;
    p.total_rows = g.N * g.OH;
    p.Wp = pl.Wp; p.RHfull = pl.RHfull; p.S2 = pl.S2; p.CH = pl.CH; p.nchunks = pl.nchunks;
    p.pitch16 = pl.pitch16;
    p.buf16 = pl.buf16;
    p.tab16 = pl.tab16;
    p.tab_len = pl.tab_len;
    p.kl16 = pl.kl16;
    p.chunk_pad = pl.chunk_pad;
    p.ragged = g.Cw % pl.CH != 0;
    // a band touches at most TH/OH + 2 images; a lane's offset also spans the tile's 32 planes
    p.near_out = ((long long)(pl.TH / g.OH + 2) * g.F + 32) * g.OH * g.OW * 4 < (1LL << 31);
    p.tile_steps = pl.tile_steps;
    p.dCHV = make_fastdiv(pl.CH / pl.vw);
    p.dWp = make_fastdiv(pl.Wp);
    p.dRH = make_fastdiv(pl.RHfull);
    p.dOW = make_fastdiv(g.OW);
    p.dOH = make_fastdiv(g.OH);

    p.nbands = ceil_div(p.total_rows, pl.TH);
    p.bands_per_xcd = ceil_div(p.nbands, kXcds);
    const dim3 grid(kXcds * p.bands_per_xcd * pl.f_tiles);
    auto launch = [&](auto kernel, int slot) -> hipError_t {
        // raise the kernel's dynamic-LDS limit to the hardware maximum once per device and kernel
        // (the call is slow on the host); the six template instances share one function type, so
        // each passes the slot of its own flag set
        static std::atomic<unsigned long long> raised[6];
        int dev = 0;
        hipError_t err = hipGetDevice(&dev);
        if (err != hipSuccess) return err;
        const unsigned long long bit = 1ull << (dev & 63);
        if (!(raised[slot].load(std::memory_order_acquire) & bit)) {
            err = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsMax);
            if (err != hipSuccess) return err;
            raised[slot].fetch_or(bit, std::memory_order_release);
        }
        kernel<<<grid, 256, pl.lds_bytes, st>>>(p);
        return hipGetLastError();
    };
    if (Opk) {
        switch (pl.vw) {
            case 4: return launch(conv_mfma_kernel<4, true>, 0);
            case 2: return launch(conv_mfma_kernel<2, true>, 1);
            default: return launch(conv_mfma_kernel<1, true>, 2);
        }
    }
    switch (pl.vw) {
        case 4: return launch(conv_mfma_kernel<4, false>, 3);
        case 2: return launch(conv_mfma_kernel<2, false>, 4);
        default: return launch(conv_mfma_kernel<1, false>, 5);
    }
}

hipError_t launch_conv_mfma_expanded(const uint32_t *Ipk, const float *K, const float *alpha,
                                     const Geom &g, float *out, int32_t *dot, const void *workspace,
                                     hipStream_t st)
{
    return launch_mfma(Ipk, K, nullptr, alpha, g, out, dot, nullptr, nullptr, workspace, st);
}

hipError_t launch_conv_mfma_expanded_from_A(const uint32_t *Ipk, const float *A, const float *alpha,
                                            const Geom &g, float *out, int32_t *dot,
                                            const void *workspace, hipStream_t st)
{
    return launch_mfma(Ipk, nullptr, A, alpha, g, out, dot, nullptr, nullptr, workspace, st);
}

// Eq. 10's channel mean for the next layer from the partial sums over groups of filters:
// A[pix] = sum_t P[pix][t] / F
__global__ __launch_bounds__(256) void chain_mean_kernel(const float *__restrict__ P, long long npix,
                                                         int f_tiles, int F, float *__restrict__ A)
{
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    if (i >= npix) return;
    double sum = 0.0;
    for (int t = 0; t < f_tiles; ++t) sum += (double)P[i * f_tiles + t];
    A[i] = (float)(sum / (double)F);
}

// partial sums of |out| per pixel that the chained epilogue leaves for chain_mean_kernel
static int chain_sum_parts(const Geom &g)
{
    return use_persistent(g) ? conv_mfma_persistent_sum_parts(g) : ceil_div(g.F, kFilterTile);
}

size_t conv_mfma_chain_workspace_bytes(const Geom &g)
{
    const size_t ws = conv_mfma_workspace_bytes(g);
    if (ws == 0) return 0;
    return ws + (size_t)g.N * g.OH * g.OW * chain_sum_parts(g) * sizeof(float);
}

hipError_t launch_conv_mfma_chain(const uint32_t *Ipk, const uint32_t *Wpk, const float *K, const float *A,
                                  const float *alpha, const Geom &g, uint32_t *Opk, float *A_next,
                                  void *workspace, hipStream_t st)
{
    const size_t ws = conv_mfma_workspace_bytes(g);
    if (ws == 0) return hipErrorInvalidValue;
    float *P = reinterpret_cast<float *>(static_cast<char *>(workspace) + ws);
    // (no Wpk: the caller has left the expanded filters at the start of the workspace)
    hipError_t e = Wpk ? launch_expand_filters(Wpk, g, workspace, st) : hipSuccess;
    if (e != hipSuccess) return e;
    e = launch_mfma(Ipk, K, A, alpha, g, nullptr, nullptr, Opk, P, workspace, st);   // K or A, the other null
    if (e != hipSuccess) return e;
    const long long npix = (long long)g.N * g.OH * g.OW;
    chain_mean_kernel<<<ceil_div(npix, 256), 256, 0, st>>>(P, npix, chain_sum_parts(g), g.F, A_next);
    return hipGetLastError();
}

}  // namespace xnor

namespace xnor {

hipError_t launch_conv_mfma(const uint32_t *Ipk, const uint32_t *Wpk, const float *K,
                            const float *alpha, const Geom &g, float *out, int32_t *dot,
                            void *workspace, hipStream_t st)
{
    // filters -> FP4 in A-operand order, then the convolution
    const hipError_t e = launch_expand_filters(Wpk, g, workspace, st);
    return e != hipSuccess ? e : launch_conv_mfma_expanded(Ipk, K, alpha, g, out, dot, workspace, st);
}

hipError_t launch_conv_mfma_bands(const uint32_t *Ipk, const uint32_t *Wpk, const float *K,
                                  const float *alpha, const Geom &g, float *out, int32_t *dot,
                                  void *workspace, hipStream_t st)
{
    // the same two steps with this file's kernel and its workspace layout, whatever the shape
    const hipError_t e = launch_expand_with(bands_expand_layout(g), Wpk, g, workspace, st);
    return e != hipSuccess ? e
                           : launch_mfma(Ipk, K, nullptr, alpha, g, out, dot, nullptr, nullptr, workspace, st, true);
}

}  // namespace xnor
