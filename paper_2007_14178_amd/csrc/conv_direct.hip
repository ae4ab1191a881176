// XNOR + popcount convolution, one thread per output element (Sec. III-A steps 1b-1d and 3,
// Eq. 11).  Runs every shape; it is the fallback for shapes the tiled kernels do not take and the
// in-library cross-check for them.
//
// With bit 1 = +1 and bit 0 = -1 (step 1c), a word pair contributes 32 - 2*popcount(a xor b) to the
// sign dot product, and zero tail bits in both operands contribute popcount 0, so
//   dot = C * (#in-image taps) - 2 * sum popcount(Ipk xor Wpk).
// Out-of-image taps are skipped, which is the zero padding of the +-1 tensor.
#include "xnor_internal.hpp"

namespace xnor {

__global__ __launch_bounds__(256) void conv_direct_kernel(const uint32_t *__restrict__ Ipk,
                                                          const uint32_t *__restrict__ Wpk,
                                                          const float *__restrict__ K,
                                                          const float *__restrict__ alpha, Geom g,
                                                          long long total, float *__restrict__ out,
                                                          int32_t *__restrict__ dot)
{
    const long long o = (long long)blockIdx.x * 256 + threadIdx.x;
    if (o >= total) return;
    const int ox = (int)(o % g.OW);
    long long t = o / g.OW;
    const int oy = (int)(t % g.OH);
    t /= g.OH;
    const int f = (int)(t % g.F);
    const long long n = t / g.F;

    const uint32_t *img = Ipk + n * (long long)g.H * g.W * g.Cw;
    const uint32_t *flt = Wpk + (long long)f * g.kh * g.kw * g.Cw;
    int pop = 0, taps = 0;
    for (int ky = 0; ky < g.kh; ++ky) {
        const int iy = oy * g.sh - g.ph + ky;
        if (iy < 0 || iy >= g.H) continue;
        for (int kx = 0; kx < g.kw; ++kx) {
            const int ix = ox * g.sw - g.pw + kx;
            if (ix < 0 || ix >= g.W) continue;
            const uint32_t *a = img + ((long long)iy * g.W + ix) * g.Cw;
            const uint32_t *b = flt + (ky * g.kw + kx) * g.Cw;
            for (int w = 0; w < g.Cw; ++w) pop += __popc(a[w] ^ b[w]);
            ++taps;
        }
    }
    const int d = g.C * taps - 2 * pop;
    if (dot) dot[o] = d;
    out[o] = (float)d * (K[(n * g.OH + oy) * g.OW + ox] * alpha[f]);
}

hipError_t launch_conv_direct(const uint32_t *Ipk, const uint32_t *Wpk, const float *K,
                              const float *alpha, const Geom &g, float *out, int32_t *dot,
                              hipStream_t st)
{
    const long long total = (long long)g.N * g.F * g.OH * g.OW;
    conv_direct_kernel<<<ceil_div(total, 256), 256, 0, st>>>(Ipk, Wpk, K, alpha, g, total, out, dot);
    return hipGetLastError();
}

}  // namespace xnor
