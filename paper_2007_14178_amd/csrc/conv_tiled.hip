// XNOR + popcount convolution on the vector ALU (Sec. III-A steps 1b-1d and 3, Eq. 11), tiled.
//
// Two lane-ops retire 32 binary MACs: v_xor_b32 with the filter word as a wave-uniform SGPR operand,
// then v_bcnt_u32_b32, which adds the popcount into its accumulator.  Everything else is arranged so that little more than those two
// instructions issues in the inner loop:
//   * a workgroup stages the packed words of a 2-D input tile (with halo) once in LDS and walks
//     over 4 waves x Q filters per pass with that tile resident;
//   * a lane owns P output pixels and Q filter accumulators per pass (P*Q independent v_bcnt chains);
//     each LDS read of 4 channel words feeds 4*Q xor/bcnt pairs;
//   * filter words are fetched with scalar loads (one s_load_dwordx4 per filter and word quad).
// Zero padding: a zero-filled halo word makes popcount(0 xor w) = popcount(w) instead of nothing, so
// after each tap the pixels for which it lies outside the image subtract that tap's popcount(w),
// which the scalar ALU sums on the side from the same scalar-loaded filter words.  Then
//   dot = C * (#in-image taps) - 2 * popcount,   out = float(dot) * K * alpha.
// P is chosen per layer (3, 4 or 7) so that whole tile rows fill the 64*P pixel slots well
// (28x28 -> 14 rows of 28 in 448 slots, 13x13 -> 169 of 192, 56x56 -> 8 rows of 56 in 448).
// The paper's kernel keeps one channel's 8x4 spatial tile per register and masks all but kh*kw
// bits of every popcount; here every bit of every word is a channel of the contraction.
#include <algorithm>

#include "xnor_internal.hpp"

namespace xnor {
namespace {

constexpr int kQ = 8;             // filters per wave and pass
constexpr int kPassFilters = 4 * kQ;
constexpr size_t kLdsBudget = 64 * 1024;

struct TiledParams {
    int N, C, H, W, F, kh, kw, sh, sw, ph, pw, OH, OW, Cw;
    int TH, TW;          // output tile
    int RH, RW;          // staged input rows / columns = (T-1)*stride + k
    int tiles_x, tiles_y;
    int pitch;           // LDS words per staged pixel
    int f_per_wg;        // filters handled by one workgroup (a multiple of kPassFilters)
};

template <int VW, int kP>
__global__ __launch_bounds__(256) void conv_tiled_kernel(
    // separate __restrict__ arguments (not struct members): only then may the compiler fetch the
    // filter words with scalar loads while the kernel also stores to `out`
    const uint32_t *__restrict__ Ipk, const uint32_t *__restrict__ Wpk, const float *__restrict__ K,
    const float *__restrict__ alpha, float *__restrict__ out, int32_t *__restrict__ dot, TiledParams p)
{
    extern __shared__ __align__(16) uint32_t smem[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int taps = p.kh * p.kw;

    // ---- tile ----
    int b = blockIdx.x;
    const int tx = b % p.tiles_x; b /= p.tiles_x;
    const int ty = b % p.tiles_y;
    const int n = b / p.tiles_y;
    const int oy0 = ty * p.TH, ox0 = tx * p.TW;
    const int iy0 = oy0 * p.sh - p.ph, ix0 = ox0 * p.sw - p.pw;
    const bool border = iy0 < 0 || ix0 < 0 || iy0 + p.RH > p.H || ix0 + p.RW > p.W;

    // ---- stage the input tile (packed words, zero outside the image) ----
    const uint32_t *img = Ipk + (long long)n * p.H * p.W * p.Cw;
    const int nslots = p.RH * p.RW;
    for (int it = tid; it < nslots * p.Cw; it += 256) {
        const int slot = it / p.Cw, w = it - slot * p.Cw;
        const int ry = slot / p.RW, rx = slot - ry * p.RW;
        const int iy = iy0 + ry, ix = ix0 + rx;
        uint32_t v = 0;
        if (iy >= 0 && iy < p.H && ix >= 0 && ix < p.W) v = img[((long long)iy * p.W + ix) * p.Cw + w];
        smem[slot * p.pitch + w] = v;
    }

    // ---- the lane's pixels ----
    int base[kP], oyv[kP], oxv[kP];
    int klo_y[kP], khi_y[kP], klo_x[kP], khi_x[kP];   // the taps of pixel k that lie inside the image
    bool ok[kP];
#pragma unroll
    for (int k = 0; k < kP; ++k) {
        const int q = lane + 64 * k;
        const int ly = q / p.TW, lx = q - ly * p.TW;
        oyv[k] = oy0 + ly;
        oxv[k] = ox0 + lx;
        ok[k] = ly < p.TH && oyv[k] < p.OH && oxv[k] < p.OW;
        base[k] = ok[k] ? (ly * p.sh * p.RW + lx * p.sw) * p.pitch : 0;
        klo_y[k] = max(0, p.ph - oyv[k] * p.sh); khi_y[k] = min(p.kh, p.H + p.ph - oyv[k] * p.sh);
        klo_x[k] = max(0, p.pw - oxv[k] * p.sw); khi_x[k] = min(p.kw, p.W + p.pw - oxv[k] * p.sw);
    }
    __syncthreads();   // staged tile ready

    const int f_wg0 = blockIdx.y * p.f_per_wg;
    for (int f_pass = f_wg0; f_pass < min(p.F, f_wg0 + p.f_per_wg); f_pass += kPassFilters) {
        const int f0 = f_pass + wave * kQ;   // this wave's filters (wave-uniform)
        uint32_t acc[kP][kQ];
#pragma unroll
        for (int k = 0; k < kP; ++k)
#pragma unroll
            for (int q = 0; q < kQ; ++q) acc[k][q] = 0;

        if (f0 < p.F) {
            // this wave's filters: words of filter q from fbase[q], [tap][Cw] contiguous; filters
            // past F re-read the last filter (their sums are never stored)
            const uint32_t *fbase[kQ];
#pragma unroll
            for (int q = 0; q < kQ; ++q) fbase[q] = Wpk + (long long)min(f0 + q, p.F - 1) * taps * p.Cw;
            typedef uint32_t wvec __attribute__((ext_vector_type(VW)));
            auto load_w = [&](int q, int woff) -> wvec { return *reinterpret_cast<const wvec *>(fbase[q] + woff); };
            // The filter words of step i+1 are requested (scalar loads) before the lane-ops of step
            // i are issued, so that their latency hides behind 2*P*Q*VW vector instructions.
            const int last_woff = taps * p.Cw - VW;
            wvec nxt[kQ];
#pragma unroll
            for (int q = 0; q < kQ; ++q) nxt[q] = load_w(q, 0);
            int woff = 0;
            for (int ky = 0; ky < p.kh; ++ky)
                for (int kx = 0; kx < p.kw; ++kx) {
                    const int toff = (ky * p.RW + kx) * p.pitch;
                    uint32_t spop[kQ];   // popcount of this tap's words of filter q (scalar ALU)
#pragma unroll
                    for (int q = 0; q < kQ; ++q) spop[q] = 0;
                    for (int w = 0; w < p.Cw; w += VW) {
                        uint32_t x[kP][VW];
#pragma unroll
                        for (int k = 0; k < kP; ++k) {
                            if constexpr (VW == 4) {
                                // (index arithmetic in 16-byte units: the type then carries the alignment
                                // that lets this be one ds_read_b128; pitch is a multiple of 4 words here)
                                const uint4 v = reinterpret_cast<const uint4 *>(smem)[(base[k] >> 2) + (toff >> 2) + (w >> 2)];
                                x[k][0] = v.x; x[k][1] = v.y; x[k][2] = v.z; x[k][3] = v.w;
                            } else {
                                x[k][0] = smem[base[k] + toff + w];
                            }
                        }
                        wvec cur[kQ];
                        woff = min(woff + VW, last_woff);
#pragma unroll
                        for (int q = 0; q < kQ; ++q) {
                            cur[q] = nxt[q];
                            nxt[q] = load_w(q, woff);
                        }
#pragma unroll
                        for (int q = 0; q < kQ; ++q) {
                            uint32_t wv[VW];
                            if constexpr (VW == 4) { wv[0] = cur[q].x; wv[1] = cur[q].y; wv[2] = cur[q].z; wv[3] = cur[q].w; }
                            else { wv[0] = cur[q][0]; }
#pragma unroll
                            for (int k = 0; k < kP; ++k)
#pragma unroll
                                for (int e = 0; e < VW; ++e) acc[k][q] += __popc(x[k][e] ^ wv[e]);
#pragma unroll
                            for (int e = 0; e < VW; ++e) spop[q] += __popc(wv[e]);
                        }
                    }
                    // Zero padding: the staged halo words are 0, so an out-of-image tap has just
                    // added popcount(0 xor w) = popcount(w); take it back for the pixels concerned
                    // (tiles that touch the image border only: 2 lane-ops per accumulator and tap
                    // against 2 * Cw in the loop above).
                    if (border) {
#pragma unroll
                        for (int k = 0; k < kP; ++k) {
                            const bool inside = ky >= klo_y[k] && ky < khi_y[k] && kx >= klo_x[k] && kx < khi_x[k];
#pragma unroll
                            for (int q = 0; q < kQ; ++q) acc[k][q] -= inside ? 0u : spop[q];
                        }
                    }
                }
        }

        // ---- step 3: dot, rescale ----
#pragma unroll
        for (int k = 0; k < kP; ++k) {
            if (!ok[k] || f0 >= p.F) continue;
            const int oy = oyv[k], ox = oxv[k];
            const int valid = max(0, khi_y[k] - klo_y[k]) * max(0, khi_x[k] - klo_x[k]);
            const float kv = K[((long long)n * p.OH + oy) * p.OW + ox];
#pragma unroll
            for (int q = 0; q < kQ; ++q) {
                const int f = f0 + q;
                if (f >= p.F) break;
                const int d = p.C * valid - 2 * (int)acc[k][q];
                const long long o = (((long long)n * p.F + f) * p.OH + oy) * p.OW + ox;
                out[o] = (float)d * (kv * alpha[f]);
                if (dot) dot[o] = d;
            }
        }
    }
}

struct TiledPlan {
    bool ok;
    int kp, TH, TW, RH, RW, tiles_x, tiles_y, pitch, vw, f_per_wg;
    size_t lds_bytes;
};

constexpr int kPixelsPerLane[] = {3, 4, 7};   // the instantiated values of P

TiledPlan make_plan(const Geom &g, const void *Ipk, const void *Wpk)
{
    TiledPlan best{};
    const uintptr_t al = reinterpret_cast<uintptr_t>(Ipk) | reinterpret_cast<uintptr_t>(Wpk);
    const int vw = (g.Cw % 4 == 0 && (al & 15) == 0) ? 4 : 1;
    // LDS words per staged pixel: an odd number of 16-byte units (VW = 4) or an odd number of words
    const int pitch = vw == 4 ? (g.Cw | 4) : (g.Cw | 1);
    double best_fill = 0.0;
    for (const int kp : kPixelsPerLane) {
        TiledPlan pl{};
        pl.kp = kp; pl.vw = vw; pl.pitch = pitch;
        pl.TW = std::min(g.OW, 64);
        pl.TH = std::max(1, std::min(g.OH, 64 * kp / pl.TW));
        pl.TH = ceil_div(g.OH, ceil_div(g.OH, pl.TH));   // same number of tiles, rows spread evenly
        // shrink the tile until it fits LDS (wide channels / big kernels)
        bool fits = true;
        for (;;) {
            pl.RH = (pl.TH - 1) * g.sh + g.kh;
            pl.RW = (pl.TW - 1) * g.sw + g.kw;
            pl.lds_bytes = (size_t)pl.RH * pl.RW * pitch * 4;
            if (pl.lds_bytes <= kLdsBudget) break;
            if (pl.TH > 1) pl.TH = (pl.TH + 1) / 2;
            else if (pl.TW > 1) pl.TW = (pl.TW + 1) / 2;
            else { fits = false; break; }   // one pixel's receptive field does not fit
        }
        if (!fits) continue;
        pl.tiles_x = ceil_div(g.OW, pl.TW);
        pl.tiles_y = ceil_div(g.OH, pl.TH);
        const long long tiles = (long long)g.N * pl.tiles_x * pl.tiles_y;
        if (tiles > 0x7fffffffLL) continue;
        // fraction of the pixel slots that hold an output pixel; ties go to the smaller P
        const double fill = (double)g.OH * g.OW / ((double)pl.tiles_x * pl.tiles_y * 64 * kp);
        if (fill <= best_fill + 1e-9) continue;
        // split the filters over workgroups until the grid has a few workgroups per CU
        const int passes = ceil_div(g.F, kPassFilters);
        int split = 1;
        while (split < passes && tiles * split < 4 * 256) ++split;
        pl.f_per_wg = ceil_div(passes, split) * kPassFilters;
        pl.ok = true;
        best = pl;
        best_fill = fill;
    }
    return best;
}

}  // namespace

bool conv_tiled_supports(const Geom &g) { return make_plan(g, nullptr, nullptr).ok; }

hipError_t launch_conv_tiled(const uint32_t *Ipk, const uint32_t *Wpk, const float *K,
                             const float *alpha, const Geom &g, float *out, int32_t *dot,
                             hipStream_t st)
{
    const TiledPlan pl = make_plan(g, Ipk, Wpk);
    if (!pl.ok) return hipErrorInvalidValue;
    TiledParams p{};
    p.N = g.N; p.C = g.C; p.H = g.H; p.W = g.W; p.F = g.F; p.kh = g.kh; p.kw = g.kw;
    p.sh = g.sh; p.sw = g.sw; p.ph = g.ph; p.pw = g.pw; p.OH = g.OH; p.OW = g.OW; p.Cw = g.Cw;
    p.TH = pl.TH; p.TW = pl.TW; p.RH = pl.RH; p.RW = pl.RW;
    p.tiles_x = pl.tiles_x; p.tiles_y = pl.tiles_y;
    p.pitch = pl.pitch; p.f_per_wg = pl.f_per_wg;
    const dim3 grid(g.N * pl.tiles_x * pl.tiles_y, ceil_div(g.F, pl.f_per_wg));
    auto launch = [&](auto kernel) {
        kernel<<<grid, 256, pl.lds_bytes, st>>>(Ipk, Wpk, K, alpha, out, dot, p);
        return hipGetLastError();
    };
    if (pl.vw == 4) {
        switch (pl.kp) {
            case 3: return launch(conv_tiled_kernel<4, 3>);
            case 4: return launch(conv_tiled_kernel<4, 4>);
            default: return launch(conv_tiled_kernel<4, 7>);
        }
    }
    switch (pl.kp) {
        case 3: return launch(conv_tiled_kernel<1, 3>);
        case 4: return launch(conv_tiled_kernel<1, 4>);
        default: return launch(conv_tiled_kernel<1, 7>);
    }
}

}  // namespace xnor
