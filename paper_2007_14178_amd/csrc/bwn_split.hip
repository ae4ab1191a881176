// Binary-Weight-Network convolution (Sec. II-A, Eq. 1) on the bf16 matrix instruction, exact in its
// operands: every fp32 input value x is split into three bf16 terms x = hi + mid + lo (each term
// the leading eight significand bits of what the terms before it left over: the three differences
// are exact in fp32 and 3 x 8 bits are the whole significand), the weights are +-1 (exact in bf16),
// so the products are exact and the sum is accumulated in fp32 by v_mfma_f32_32x32x16_bf16: three
// matrix instructions per 16 channels where the fp32 matrix instruction needs eight, at 16 times
// its rate.
//
//   bwn_split_kernel: a workgroup (4 waves) owns 128 filters x up to 6 tiles of 32 consecutive
//   output pixels of one image; wave = 64 filters (two filter tiles) x half of the pixel tiles.
//   Per chunk of 16 channels the input rows under the pixels are fetched a chunk ahead (eight
//   channels of one position per granule), split, and staged in LDS as
//   [position][term][16 channels] bf16 (112 bytes per position: sixteen lanes' 16-byte reads or
//   writes at consecutive positions touch distinct banks), zeros where the image ends (that is the
//   zero padding).  The B operand of a matrix instruction is one 16-byte LDS read per lane (lane =
//   pixel, eight channels), used for both filter tiles; the A operand (lane = filter, eight
//   channels) is made in registers from eight bits of the filter's packed word (the words of the
//   next 32 channels come straight from memory into LDS while the current ones are in use).
//   Inputs that are not finite give NaN where the fp32 sum would give an infinity (inf - inf in the
//   split); the matrix instruction flushes a term below the normal range (2^-126), so an input value
//   contributes an error of up to 2^-125 (two of its terms) on top of the fp32 summation's.
#include <algorithm>
#include <atomic>
#include <type_traits>

#include "xnor_internal.hpp"

namespace xnor {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int kThreads = 256;
constexpr int kFiltersPerWg = 128;     // 2 wave columns x 2 filter tiles x 32
constexpr int kMaxTiles = 6;           // pixel tiles per workgroup: 2 wave rows x 3
constexpr int kChan = 16;              // channels per chunk = the reduction length of one matrix instruction
constexpr int kPosBytes = 112;         // 3 terms x 32 bytes + 16: see above
constexpr int kGran = 4;               // granules (8 channels of one position) a thread fetches ahead per chunk
constexpr int kMaxTaps = 64;
constexpr int kDumpBytes = 1024;       // 64 lanes x 8 bytes, the three terms 32 bytes apart
constexpr size_t kLdsBudget = 160 * 1024;  // all buffers of a workgroup (up to 80 KB: two workgroups per compute unit)

struct SplitParams {
    const float *I;
    const uint32_t *Wpk;
    const float *alpha;
    float *out;
    int N, C, H, W, F, kh, kw, sh, sw, ph, pw, OH, OW, Cw;
    int tiles, groups, fgroups;
    int tpr;                       // 0: a tile is 32 consecutive pixels of the image; else tiles per output row: a
                                   // tile is a 32-pixel segment of one row (the row's last one may be short)
    int rows_max, pitch, npos;     // staged rows, positions per row (W + 2*pw), rows_max * pitch
    uint32_t inv_pitch;            // ceil(2^32 / pitch), 0 for pitch 1
};

__device__ inline uint32_t quot(uint32_t n, uint32_t inv) { return inv == 0 ? n : __umulhi(n, inv); }
uint32_t reciprocal(unsigned long long d) { return d == 1 ? 0u : (uint32_t)(((1ULL << 32) + d - 1) / d); }

// x = hi + mid + lo, each the top 16 bits of an fp32 (a bf16): the leading bits by truncation, the
// rest by an exact subtraction.  Returned are x, x - hi and x - hi - mid: the terms are their top
// halves, which is all that pair16 takes of them.
__device__ inline void split3(float x, uint32_t &t0, uint32_t &t1, uint32_t &t2)
{
    t0 = __float_as_uint(x);
    const float r1 = x - __uint_as_float(t0 & 0xffff0000u);
    t1 = __float_as_uint(r1);
    const float r2 = r1 - __uint_as_float(t1 & 0xffff0000u);
    t2 = __float_as_uint(r2);
}
// the low 16 bits of x in both halves of a dword
__device__ inline uint32_t both_halves(uint32_t x) { return __builtin_amdgcn_perm(x, x, 0x01000100u); }
// the top halves of a and b in one dword, a's in the low half (one v_perm_b32)
__device__ inline uint32_t pair16(uint32_t a, uint32_t b) { return __builtin_amdgcn_perm(b, a, 0x07060302u); }

typedef unsigned short ushortx2 __attribute__((ext_vector_type(2)));

// Sixteen inverted filter signs (1 = -1.0), the same in both halves of `w2`, -> the eight bf16 +-1.0
// of this lane's channels: dword k holds channels 8*half + 2k (low) and 8*half + 2k + 1 (high).
// One packed 16-bit shift brings the two sign bits to bits 15 and 31; `sh[k]` holds the two counts
// (15 - 8*half - 2k in the low half, one less in the high half); `sign_mask` is 0x80008000 in a
// scalar and `ones` 0x3F803F80 in a vector register (an instruction takes one literal or one scalar
// register), so that the merge is one v_and_or_b32.
__device__ inline uint32_t sign_dword(uint32_t w2, uint32_t sh_k, uint32_t sign_mask, uint32_t ones)
{
    const ushortx2 y = __builtin_bit_cast(ushortx2, w2) << __builtin_bit_cast(ushortx2, sh_k);
    return (__builtin_bit_cast(uint32_t, y) & sign_mask) | ones;
}
__device__ inline bf16x8 signs_to_bf16(uint32_t w2, const uint32_t (&sh)[4], uint32_t sign_mask, uint32_t ones)
{
    return __builtin_bit_cast(bf16x8, make_uint4(sign_dword(w2, sh[0], sign_mask, ones), sign_dword(w2, sh[1], sign_mask, ones),
                                                  sign_dword(w2, sh[2], sign_mask, ones), sign_dword(w2, sh[3], sign_mask, ones)));
}

// The work of one wave with NT pixel tiles (0: it only takes part in the staging).
template <int NT>
__device__ __attribute__((always_inline)) void split_wave(const SplitParams &p, int n, int fbase, int t0,
                                                          int oy0, int oy1, int tile0, int wf)
{
    // LDS: two input buffers, taken in turn by the chunks, each [npos][3][16] bf16 at a 112-byte
    // pitch followed by a dump slot for the staging writes of threads without a position; then two
    // filter-word buffers, taken in turn by the 32-channel words (a word serves two chunks), each
    // [taps][128] packed words as they come.
    extern __shared__ unsigned char lds_raw[];
    const int tile_bytes = p.npos * kPosBytes + kDumpBytes;
    const int words_bytes = p.kh * p.kw * kFiltersPerWg * 4;
    unsigned char *const words_lds = lds_raw + 2 * tile_bytes;
    const int dump_off = p.npos * kPosBytes;

    const int lane = threadIdx.x & 63;
    const int col = lane & 31, half = lane >> 5;
    const int OHW = p.OH * p.OW;
    // the pixel of lane `col` in tile t of the image: its row and column (clamped to the image for
    // the reads) and whether it exists
    auto pixel_of = [&](int t, int &oy, int &ox) -> bool {
        if (p.tpr == 0) {
            const int px = t * 32 + col, pxc = min(px, OHW - 1);
            oy = pxc / p.OW;
            ox = pxc - oy * p.OW;
            return px < OHW;
        }
        oy = t / p.tpr;
        const int x = (t - oy * p.tpr) * 32 + col;
        ox = min(x, p.OW - 1);
        return x < p.OW;
    };
    const int iy0 = oy0 * p.sh - p.ph;
    const int rows = (oy1 - oy0) * p.sh + p.kh;         // <= rows_max
    const int taps = p.kh * p.kw;

    // per pixel tile: the lane's LDS byte offset of tap (0,0), its eight channels
    int base[NT > 0 ? NT : 1];
#pragma unroll
    for (int j = 0; j < NT; ++j) {
        int oy, ox;
        pixel_of(t0 + tile0 + j, oy, ox);
        base[j] = ((oy - oy0) * p.sh * p.pitch + ox * p.sw) * kPosBytes + half * 16;
    }

    uint32_t sign_mask;
    asm volatile("s_mov_b32 %0, 0x80008000" : "=s"(sign_mask));
    uint32_t ones;
    asm volatile("v_mov_b32 %0, 0x3f803f80" : "=v"(ones));
    uint32_t shifts[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const uint32_t lo = (uint32_t)(15 - 8 * half - 2 * k);
        shifts[k] = lo | ((lo - 1) << 16);
    }

    floatx16 acc[2][NT > 0 ? NT : 1];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const int nchunks = (p.C + kChan - 1) / kChan;
    const float *img = p.I + (size_t)n * p.C * p.H * p.W;
    const int HW = p.H * p.W;

    // Staging.  A granule is eight channels of one staged position: thread t takes the positions
    // q * 128 + t % 128 (q < kGran) of channel octet t / 128, which is the same for a whole wave, so
    // the address of a value is a scalar base (the channel's plane) plus a lane offset that does
    // not change from chunk to chunk (kept in registers, with one flag bit per granule: the position
    // lies in the image and under the band's rows).  Every load is unconditional (offset 0, channel
    // 0 where there is nothing to fetch) and nothing is done with its result until the commit, where
    // what is not there becomes zero: a select behind each load would make the compiler wait for it
    // before issuing the next.
    const int tl = threadIdx.x & 127;
    const int oct = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 7);
    uint32_t voff[kGran];
    int wr_off[kGran];         // where the granule goes in a buffer (a position past the last: the dump slot)
    uint32_t okbits = 0;
#pragma unroll
    for (int q = 0; q < kGran; ++q) {
        const int pos = q * 128 + tl;
        wr_off[q] = pos < p.npos ? pos * kPosBytes + oct * 16 : dump_off + (int)(threadIdx.x & 63) * 8;
        const uint32_t r = quot((uint32_t)pos, p.inv_pitch);
        const int xw = (int)((uint32_t)pos - r * (uint32_t)p.pitch);
        const int iy = iy0 + (int)r, ix = xw - p.pw;
        const bool ok = pos < p.npos && (int)r < rows && (unsigned)iy < (unsigned)p.H && (unsigned)ix < (unsigned)p.W;
        voff[q] = ok ? (uint32_t)(iy * p.W + ix) * 4u : 0u;
        okbits |= ok ? 1u << q : 0u;
    }
    // filter words: word i = q * 256 + t of [taps][128] is tap 2q + t / 128 (uniform) of filter t % 128

    float nxt[kGran][8];
    auto prefetch = [&](int ch) __attribute__((always_inline)) {
        const int c0 = ch * kChan + 8 * oct;
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int c = c0 + k < p.C ? c0 + k : 0;                             // (scalar)
            const char *plane_c = reinterpret_cast<const char *>(img + (size_t)c * HW);
#pragma unroll
            for (int q = 0; q < kGran; ++q) {
                if (q * 128 >= p.npos) break;                                    // uniform
                nxt[q][k] = *reinterpret_cast<const float *>(plane_c + voff[q]);
            }
        }
    };
    // Filter words.  Word cw (32 channels) serves chunks 2cw and 2cw + 1 and is brought in while
    // word cw - 1 is in use, straight from memory into its LDS buffer (global_load_lds_dword: a wave
    // instruction puts its 64 lanes' dwords side by side at the LDS address in M0, no registers in
    // between): instruction e of the 2 * taps of a word is tap e / 2, filters 64 * (e % 2) + lane;
    // wave w issues e = w, w + 4, ...  The loads are waited for before the barrier that ends the
    // chunk they were issued in.  (A filter past the last one gets the last one's signs: its outputs
    // are not stored.)
    auto words_stage = [&](int cw) __attribute__((always_inline)) {
        if (cw >= p.Cw) return;
        const int wave4 = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
        const int lane64 = threadIdx.x & 63;
        unsigned char *buf = words_lds + (cw & 1) * words_bytes;
        uint32_t off[2];
#pragma unroll
        for (int j = 0; j < 2; ++j)
            off[j] = (uint32_t)min(fbase + 64 * j + lane64, p.F - 1) * (uint32_t)(taps * p.Cw) * 4u;   // (below 2^31: the plan sees to it)
        for (int e = wave4; e < 2 * taps; e += 4) {
            const int t = e >> 1;                                               // (scalar)
            const char *wbase = reinterpret_cast<const char *>(p.Wpk + (size_t)t * p.Cw + cw);
            const uint32_t *src = reinterpret_cast<const uint32_t *>(wbase + off[e & 1]);
            __builtin_amdgcn_global_load_lds(src, (__attribute__((address_space(3))) void *)(buf + e * 256), 4, 0, 0);
        }
    };
    // The commit of chunk `ch` into buffer ch % 2 comes in kPieces pieces, so that each can be laid
    // among the matrix instructions of one step of the chunk before: pieces 0 .. 2*kGran - 1 split
    // and write one half (four channels) of granule s / 2, the last piece writes the filter words
    // fetched a chunk ago, fetches the next ones and issues the loads of chunk ch + 1 into the
    // registers just freed.
    constexpr int kPieces = 2 * kGran + 1;
    uint32_t th[4], tm[4], tl3[4];     // the three terms of a piece's four values, between its units
    auto commit_unit = [&](auto piece_c, auto unit_c, int ch) __attribute__((always_inline)) {
        constexpr int S = decltype(piece_c)::value, U = decltype(unit_c)::value;
        unsigned char *tile_w = lds_raw + (ch & 1) * tile_bytes;
        if constexpr (S < 2 * kGran) {
            constexpr int q = S >> 1, hf = S & 1;
            const int c0 = ch * kChan + 8 * oct + 4 * hf;
            // (no branch, uniform or not: the piece has to stay in the block of the step's matrix
            //  instructions; a position past the last one goes to the dump slot).  Units 0-3 split one
            // value each, unit 4 packs and writes: the caller lays one unit behind each matrix instruction.
            if constexpr (U < 4) {
                const bool ok = (okbits >> q) & 1u;
                split3((ok && c0 + U < p.C) ? nxt[q][4 * hf + U] : 0.f, th[U], tm[U], tl3[U]);
            } else if constexpr (U == 4) {
                uint2 *dst = reinterpret_cast<uint2 *>(tile_w + wr_off[q] + hf * 8);
                dst[0] = make_uint2(pair16(th[0], th[1]), pair16(th[2], th[3]));
                dst[4] = make_uint2(pair16(tm[0], tm[1]), pair16(tm[2], tm[3]));
                dst[8] = make_uint2(pair16(tl3[0], tl3[1]), pair16(tl3[2], tl3[3]));
            }
        } else if constexpr (U == 0) {
            // while an even chunk ch - 1 runs: the word after its own is brought in
            if (((ch - 1) & 1) == 0) words_stage(((ch - 1) >> 1) + 1);
            if (ch + 1 < nchunks) prefetch(ch + 1);
        }
    };
    auto commit_piece = [&](auto piece_c, int ch) __attribute__((always_inline)) {
        commit_unit(piece_c, std::integral_constant<int, 0>{}, ch);
        commit_unit(piece_c, std::integral_constant<int, 1>{}, ch);
        commit_unit(piece_c, std::integral_constant<int, 2>{}, ch);
        commit_unit(piece_c, std::integral_constant<int, 3>{}, ch);
        commit_unit(piece_c, std::integral_constant<int, 4>{}, ch);
    };
    // pieces `from` .. kPieces - 1 of chunk ch, one after the other
    auto commit_rest = [&](int from, int ch, bool last_too = true) __attribute__((always_inline)) {
        if (from <= 0) commit_piece(std::integral_constant<int, 0>{}, ch);
        if (from <= 1) commit_piece(std::integral_constant<int, 1>{}, ch);
        if (from <= 2) commit_piece(std::integral_constant<int, 2>{}, ch);
        if (from <= 3) commit_piece(std::integral_constant<int, 3>{}, ch);
        if (from <= 4) commit_piece(std::integral_constant<int, 4>{}, ch);
        if (from <= 5) commit_piece(std::integral_constant<int, 5>{}, ch);
        if (from <= 6) commit_piece(std::integral_constant<int, 6>{}, ch);
        if (from <= 7) commit_piece(std::integral_constant<int, 7>{}, ch);
        if (from <= 8 && last_too) commit_piece(std::integral_constant<int, 8>{}, ch);
        static_assert(kPieces == 9, "one line per piece");
    };

    // before the first chunk: word 0, chunk 0, and in flight: chunk 1
    words_stage(0);
    prefetch(0);
    commit_rest(0, 0, false);
    if (nchunks > 1) prefetch(1);
    __builtin_amdgcn_s_waitcnt(0x0F70);                  // vmcnt(0): the words are in LDS
    __syncthreads();
    for (int ch = 0; ch < nchunks; ++ch) {
        const bool more = ch + 1 < nchunks;
        int pc = more ? 0 : kPieces;                     // the next piece of chunk ch + 1 to commit
        if constexpr (NT > 0) {
            // The flat sequence of (tap, pixel tile) steps, six matrix instructions each.  A step's
            // three B operands are read two steps ahead, a tap's two filter words two taps ahead, a
            // tap's A operands are made among the matrix instructions of the tap before it, and
            // each of the chunk's first steps carries one piece of the next chunk's commit.
            const unsigned char *tile_r = lds_raw + (ch & 1) * tile_bytes;
            const uint32_t *wsrc = reinterpret_cast<const uint32_t *>(words_lds + ((ch >> 1) & 1) * words_bytes) + wf * 64 + col;
            const int bit0 = (ch & 1) * 16;              // the chunk's sixteen signs within the word
            // sixteen signs, inverted (1 = -1.0), in both halves of a dword
            auto signs2 = [&](uint32_t w) -> uint32_t { return both_halves(~(w >> bit0)); };
            auto read3 = [&](uint4 (&b)[3], int byte_off) __attribute__((always_inline)) {
                const uint4 *src = reinterpret_cast<const uint4 *>(tile_r + byte_off);
                b[0] = src[0];
                b[1] = src[2];
                b[2] = src[4];
            };
            // (off, kx): byte offset and window column of tap `tap` -> of the tap after it: one position
            // to the right, or to the start of the next window row; the last tap stays (reads beyond
            // it are not used).  (Selects, no branches.)
            const int row_step = (p.pitch - p.kw + 1) * kPosBytes;
            auto tap_after = [&](int &off, int &kx, int tap) {
                const bool further = tap + 1 < taps, wrap = kx + 1 == p.kw;
                off += further ? (wrap ? row_step : kPosBytes) : 0;
                kx = further ? (wrap ? 0 : kx + 1) : kx;
            };
            int off0 = 0;
            int off1 = 0, kx1 = 0;
            tap_after(off1, kx1, 0);
            int off2 = off1, kx2 = kx1;
            tap_after(off2, kx2, 1);
            const int t1 = min(1, taps - 1);
            uint32_t wn0 = wsrc[t1 * kFiltersPerWg], wn1 = wsrc[t1 * kFiltersPerWg + 32];
            bf16x8 a0 = signs_to_bf16(signs2(wsrc[0]), shifts, sign_mask, ones), a1 = signs_to_bf16(signs2(wsrc[32]), shifts, sign_mask, ones);
            uint4 bc[3], bn[3], bf[3];
            read3(bc, base[0] + off0);
            read3(bn, NT > 1 ? base[NT > 1 ? 1 : 0] + off0 : base[0] + off1);   // (step 1: the second tile, or the second tap)
            // one step: tile j of the current tap, with piece S of the commit (-1: none)
            // Behind each of its six matrix instructions a step lays one unit of the other work
            // (a fence after each keeps the order): a tap's first step the A operands of the next
            // tap, a step with a piece the piece's units.
            uint32_t an[2][4];
            uint32_t sg0 = 0, sg1 = 0;
            auto step = [&](auto piece_c, int j) __attribute__((always_inline)) {
                constexpr int S = decltype(piece_c)::value;
                const int j2 = (j + 2) % NT, ahead = (j + 2) / NT;          // (constants once unrolled)
                read3(bf, base[j2] + (ahead == 0 ? off0 : ahead == 1 ? off1 : off2));
                __builtin_amdgcn_sched_barrier(0);
                auto unit = [&](auto m_c) __attribute__((always_inline)) {
                    constexpr int M = decltype(m_c)::value;
                    const bf16x8 b = __builtin_bit_cast(bf16x8, bc[M >> 1]);
                    acc[M & 1][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16((M & 1) ? a1 : a0, b, acc[M & 1][j], 0, 0, 0);
                    if (j == 0) {
                        if constexpr (M == 0) { sg0 = signs2(wn0); an[0][0] = sign_dword(sg0, shifts[0], sign_mask, ones); an[0][1] = sign_dword(sg0, shifts[1], sign_mask, ones); }
                        if constexpr (M == 1) { an[0][2] = sign_dword(sg0, shifts[2], sign_mask, ones); an[0][3] = sign_dword(sg0, shifts[3], sign_mask, ones); }
                        if constexpr (M == 2) { sg1 = signs2(wn1); an[1][0] = sign_dword(sg1, shifts[0], sign_mask, ones); an[1][1] = sign_dword(sg1, shifts[1], sign_mask, ones); }
                        if constexpr (M == 3) { an[1][2] = sign_dword(sg1, shifts[2], sign_mask, ones); an[1][3] = sign_dword(sg1, shifts[3], sign_mask, ones); }
                    }
                    if constexpr (S >= 0 && M < 5) commit_unit(piece_c, std::integral_constant<int, M>{}, ch + 1);
                    __builtin_amdgcn_sched_barrier(0);
                };
                unit(std::integral_constant<int, 0>{});
                unit(std::integral_constant<int, 1>{});
                unit(std::integral_constant<int, 2>{});
                unit(std::integral_constant<int, 3>{});
                unit(std::integral_constant<int, 4>{});
                unit(std::integral_constant<int, 5>{});
#pragma unroll
                for (int t = 0; t < 3; ++t) { bc[t] = bn[t]; bn[t] = bf[t]; }
            };
            // one tap: its NT steps, the first of them with piece FIRST of the commit (-1: no pieces)
            auto tap_body = [&](auto first_c, int tap) __attribute__((always_inline)) {
                constexpr int FIRST = decltype(first_c)::value;
                const int t2 = min(tap + 2, taps - 1);
                const uint32_t wf0 = wsrc[t2 * kFiltersPerWg], wf1 = wsrc[t2 * kFiltersPerWg + 32];
                step(std::integral_constant<int, (FIRST >= 0 && FIRST < kPieces) ? FIRST : -1>{}, 0);
                if constexpr (NT > 1) step(std::integral_constant<int, (FIRST >= 0 && FIRST + 1 < kPieces) ? FIRST + 1 : -1>{}, 1);
                if constexpr (NT > 2) step(std::integral_constant<int, (FIRST >= 0 && FIRST + 2 < kPieces) ? FIRST + 2 : -1>{}, 2);
                static_assert(NT <= 3, "one line per step");
                a0 = __builtin_bit_cast(bf16x8, make_uint4(an[0][0], an[0][1], an[0][2], an[0][3]));
                a1 = __builtin_bit_cast(bf16x8, make_uint4(an[1][0], an[1][1], an[1][2], an[1][3]));
                wn0 = wf0; wn1 = wf1;
                off0 = off1; off1 = off2;
                tap_after(off2, kx2, tap + 2);
            };
            // the chunk's first taps carry the pieces (their code is laid out once per tap), the
            // other taps run in a loop
            int tap = 0;
            if (more) {
                if (tap < taps) { tap_body(std::integral_constant<int, 0>{}, tap); ++tap; }
                if constexpr (1 * NT < kPieces) if (tap < taps) { tap_body(std::integral_constant<int, 1 * NT>{}, tap); ++tap; }
                if constexpr (2 * NT < kPieces) if (tap < taps) { tap_body(std::integral_constant<int, 2 * NT>{}, tap); ++tap; }
                if constexpr (3 * NT < kPieces) if (tap < taps) { tap_body(std::integral_constant<int, 3 * NT>{}, tap); ++tap; }
                if constexpr (4 * NT < kPieces) if (tap < taps) { tap_body(std::integral_constant<int, 4 * NT>{}, tap); ++tap; }
                if constexpr (5 * NT < kPieces) if (tap < taps) { tap_body(std::integral_constant<int, 5 * NT>{}, tap); ++tap; }
                if constexpr (6 * NT < kPieces) if (tap < taps) { tap_body(std::integral_constant<int, 6 * NT>{}, tap); ++tap; }
                if constexpr (7 * NT < kPieces) if (tap < taps) { tap_body(std::integral_constant<int, 7 * NT>{}, tap); ++tap; }
                if constexpr (8 * NT < kPieces) if (tap < taps) { tap_body(std::integral_constant<int, 8 * NT>{}, tap); ++tap; }
                static_assert(kPieces <= 9, "one line per tap that carries pieces");
                pc = min(tap * NT, kPieces);
            }
            for (; tap < taps; ++tap) tap_body(std::integral_constant<int, -1>{}, tap);
        }
        // what the chunk's steps did not carry (few steps, or a wave without tiles)
        if (pc < kPieces) commit_rest(pc, ch + 1);
        // the words brought in during this chunk are in LDS once all but the loads issued after them
        // (the next prefetch: eight per granule in use) have come back
        if (more && (ch & 1) == 0 && (ch >> 1) + 1 < p.Cw) {
            if (ch + 2 >= nchunks) __builtin_amdgcn_s_waitcnt(0x0F70);           // vmcnt(0): no prefetch followed
            else if (p.npos <= 128) __builtin_amdgcn_s_waitcnt(0x0F78);          // vmcnt(8)
            else if (p.npos <= 256) __builtin_amdgcn_s_waitcnt(0x4F70);          // vmcnt(16)
            else if (p.npos <= 384) __builtin_amdgcn_s_waitcnt(0x4F78);          // vmcnt(24)
            else __builtin_amdgcn_s_waitcnt(0x8F70);                             // vmcnt(32)
        }
        __syncthreads();                                 // chunk ch has been read, chunk ch + 1 is written
    }

    // accumulator register r of a lane: filter row 8*(r/4) + 4*half + r%4 of the filter tile,
    // pixel column `col`
    float *dst = p.out + (size_t)n * p.F * OHW;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        float al[16];
        int fr[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            fr[r] = fbase + wf * 64 + i * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
            al[r] = fr[r] < p.F ? p.alpha[fr[r]] : 0.f;
        }
#pragma unroll
        for (int j = 0; j < NT; ++j) {
            int oy, ox;
            if (pixel_of(t0 + tile0 + j, oy, ox)) {
                const int px = oy * p.OW + ox;
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (fr[r] < p.F) dst[(size_t)fr[r] * OHW + px] = acc[i][j][r] * al[r];
            }
        }
    }
}

__global__ __launch_bounds__(kThreads, 2) void bwn_split_kernel(SplitParams p)
{
    int b = blockIdx.x;
    const int h = b % p.fgroups; b /= p.fgroups;
    const int g = b % p.groups;
    const int n = b / p.groups;
    const int OHW = p.OH * p.OW;
    const int total = p.tpr ? p.OH * p.tpr : (OHW + 31) >> 5;
    const int t0 = g * p.tiles, t1 = min(total, t0 + p.tiles);
    const int nt = t1 - t0;                              // tiles this workgroup really has (1..6)
    const int oy0 = p.tpr ? t0 / p.tpr : (t0 * 32) / p.OW;
    const int oy1 = p.tpr ? (t1 - 1) / p.tpr : (min(OHW, t1 * 32) - 1) / p.OW;
    const int fbase = h * kFiltersPerWg;
    // wave -> (filter half, pixel half).  Every wave passes
    // the same barriers whichever instance it runs (they count arrivals, not places in the code).
    const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
    const int wf = wave & 1, wp = wave >> 1;
    // (which half takes the odd tile alternates between the workgroups that share a compute unit:
    //  workgroup ids go round the 8 XCDs first)
    const int first = (nt + 1 - (int)((blockIdx.x >> 3) & 1)) >> 1;
    const int tile0 = wp ? first : 0;
    int my_nt = wp ? nt - first : first;
    if (fbase + wf * 64 >= p.F) my_nt = 0;                // no filters for this wave: staging only
    switch (my_nt) {
        case 0: split_wave<0>(p, n, fbase, t0, oy0, oy1, tile0, wf); break;
        case 1: split_wave<1>(p, n, fbase, t0, oy0, oy1, tile0, wf); break;
        case 2: split_wave<2>(p, n, fbase, t0, oy0, oy1, tile0, wf); break;
        default: split_wave<3>(p, n, fbase, t0, oy0, oy1, tile0, wf); break;
    }
}

struct SplitPlan {
    bool ok;
    int tiles, rows_max, pitch, tpr, total;
    size_t lds;
};

SplitPlan make_split_plan(const Geom &g, int cus = 0)
{
    SplitPlan pl{};
    const long long OHW = (long long)g.OH * g.OW;
    if (g.kh * g.kw > kMaxTaps || OHW > (1 << 24) || (long long)g.C * g.H * g.W >= (1LL << 30)) return pl;
    if ((long long)g.F * g.kh * g.kw * g.Cw >= (1LL << 29)) return pl;     // (32-bit byte offsets into Wpk)
    pl.pitch = g.W + 2 * g.pw;
    // Pixel tiles per workgroup T (the kernel gives every workgroup of an image T tiles and the last
    // one the rest).  A workgroup's time is about that of its busier pixel half, ceil(T / 2) tile
    // times, plus half a tile time of staging and epilogue, a tenth less where two workgroups fit a
    // compute unit (<= 80 KB of LDS each) and fill each other's gaps; a launch takes as many of those
    // as its busiest compute unit has workgroups.  Take the T with the smallest product; on a tie the
    // one with the smaller sum of busier halves over an image, then the larger one.  (Measured: 28 x
    // 28 outputs, 25 tiles, 6,6,6,6,1 against 5 x 5: 2 % faster; 56 x 56 with 16 images and 128
    // filters: 272 workgroups of six tiles are two rounds of one workgroup per unit, the second
    // nearly empty.)
    static std::atomic<int> cus_cached{0};
    if (cus <= 0) cus = cus_cached.load(std::memory_order_relaxed);
    if (cus <= 0) {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) {
            (void)hipGetLastError();
            cus = 256;
        } else {
            cus_cached.store(cus, std::memory_order_relaxed);
        }
    }
    // Two ways to cut an image into tiles: 32 consecutive pixels (no pixel slot idle but in an image's
    // last tile; a workgroup's pixels straddle rows, which costs a staged row), or 32-pixel segments
    // of single rows (the last segment of a row short; whole rows per workgroup, which on wide rows
    // lets more tiles share the staged rows).  Both go through the same cost.
    double best = -1.0;
    int best_half = 0;
    const int tpr_rows = ceil_div(g.OW, 32);
    for (int mode = 0; mode < 2; ++mode) {
        const int tpr = mode ? tpr_rows : 0;
        const int total = mode ? g.OH * tpr_rows : (int)((OHW + 31) / 32);
        if (mode && (long long)g.OH * tpr_rows > (1 << 24)) continue;
        auto half_tiles = [&](int T) {
            const int n = ceil_div(total, T), last = total - (n - 1) * T;
            return (n - 1) * ((T + 1) / 2) + (last + 1) / 2;
        };
        for (int T = std::min(kMaxTiles, total); T >= 1; --T) {
            // the output rows T tiles span at most
            int orows;
            if (!mode) orows = (int)((32LL * T + g.OW - 2) / g.OW + 1);
            else if (T % tpr == 0) orows = T / tpr;
            else if (tpr % T == 0) orows = 1;
            else orows = (T + tpr - 2) / tpr + 1;
            orows = std::min(orows, g.OH);
            const int rows = (orows - 1) * g.sh + g.kh;
            const long long npos = (long long)rows * pl.pitch;
            const size_t lds = 2 * ((size_t)npos * kPosBytes + kDumpBytes + (size_t)g.kh * g.kw * kFiltersPerWg * 4);
            if (npos > (long long)kGran * 128 || lds > kLdsBudget) continue;
            const long long wgs = (long long)g.N * ceil_div(g.F, kFiltersPerWg) * ceil_div(total, T);
            const double per_wg = ((T + 1) / 2 + 0.5) * (lds <= kLdsBudget / 2 ? 0.9 : 1.0);
            const double cost = (double)((wgs + cus - 1) / cus) * per_wg;
            const int ht = half_tiles(T);
            const bool better = best < 0.0 || cost < best * (1.0 - 1e-9) ||
                                (!mode && cost <= best * (1.0 + 1e-9) && ht < best_half);
            if (better) {
                best = cost;
                best_half = ht;
                pl.ok = true; pl.tiles = T; pl.rows_max = rows; pl.lds = lds; pl.tpr = tpr; pl.total = total;
            }
        }
    }
    return pl;
}

}  // namespace

bool bwn_split_supports(const Geom &g) { return make_split_plan(g).ok; }

bool bwn_split_plan(const Geom &g, int compute_units, int *tiles, int *row_segments, size_t *lds_bytes,
                    long long *workgroups)
{
    const SplitPlan pl = make_split_plan(g, compute_units);
    if (!pl.ok) return false;
    *tiles = pl.tiles;
    *row_segments = pl.tpr;
    *lds_bytes = pl.lds;
    *workgroups = (long long)g.N * ceil_div(g.F, kFiltersPerWg) * ceil_div(pl.total, pl.tiles);
    return true;
}

hipError_t launch_bwn_split(const float *I, const uint32_t *Wpk, const float *alpha, const Geom &g,
                            float *out, hipStream_t st)
{
    const SplitPlan pl = make_split_plan(g);
    if (!pl.ok) return hipErrorInvalidValue;
    SplitParams p;
    p.I = I; p.Wpk = Wpk; p.alpha = alpha; p.out = out;
    p.N = g.N; p.C = g.C; p.H = g.H; p.W = g.W; p.F = g.F; p.kh = g.kh; p.kw = g.kw;
    p.sh = g.sh; p.sw = g.sw; p.ph = g.ph; p.pw = g.pw; p.OH = g.OH; p.OW = g.OW; p.Cw = g.Cw;
    p.tiles = pl.tiles; p.rows_max = pl.rows_max; p.pitch = pl.pitch; p.npos = pl.rows_max * pl.pitch;
    p.inv_pitch = reciprocal((unsigned long long)pl.pitch);
    p.tpr = pl.tpr;
    p.groups = ceil_div(pl.total, pl.tiles);
    p.fgroups = ceil_div(g.F, kFiltersPerWg);
    const long long blocks = (long long)g.N * p.groups * p.fgroups;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    if (pl.lds > 64 * 1024) {
        // raise the kernel's dynamic-LDS limit once per device
        static std::atomic<unsigned long long> raised{0};
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess) return hipGetLastError();
        const unsigned long long bit = 1ull << (dev & 63);
        if (!(raised.load() & bit)) {
            const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&bwn_split_kernel),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsBudget);
            if (e != hipSuccess) return e;
            raised.fetch_or(bit);
        }
    }
    bwn_split_kernel<<<dim3((unsigned)blocks), dim3(kThreads), pl.lds, st>>>(p);
    return hipGetLastError();
}

}  // namespace xnor
