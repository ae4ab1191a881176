/*
 * Plain CPU oracle for the XNOR-Net binary convolution forward pass.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct statement of what the
 * forward pass computes; it exists so that the GPU library can be checked against something that
 * shares no code with it.  Only the tests, the smoke check and the bench's cpu_baseline leg may
 * call it.  It is never a fallback for the product path.
 *
 * What it follows (paper = "Optimization of XNOR Convolution for Binary Convolutional Neural
 * Networks on GPU"):
 *   - binarisation B = sign(W), H = sign(X)            : Sec. II, Eq. 3 and Eq. 8
 *   - per-filter scale alpha = ||W||_1 / n             : Sec. II-A, Eq. 5
 *   - scaling map K = A * k, A = sum_c |I_c| / c,
 *     k_ij = 1 / (w*h)                                 : Sec. II-B, Eq. 10
 *   - output = (sign(I) (*) sign(W)) . K . alpha       : Sec. II-B, Eq. 11
 *   - pipeline order (binarise, xnor, sum with 0 == -1,
 *     to float, channel sum, K*alpha, multiply)        : Sec. III-A step list
 *   - bit encoding: bit 1 <=> +1, bit 0 <=> -1         : Sec. III-A step 1c
 *   - Binary-Weight-Network layer, real input and
 *     binary weights: (I (+) B) alpha, B = sign(W)     : Sec. II-A, Eq. 1 (with Eq. 5 for alpha)
 *   - real-valued convolution, the float comparison
 *     of the timings (sum of I * W, nothing binarised) : Sec. IV, Table I
 *
 * The method reaches its target exactly (the bit encoding is a trick, not an approximation of the
 * sign convolution), so the oracle is the plain definition: a direct float convolution on +-1
 * values, no packing, no blocking, no reordering.  OpenMP is used over independent (image, filter)
 * planes only.
 *
 * Readings of points the paper leaves open (all listed again in the design notes):
 *   - sign(0) = +1, implemented as (x >= 0): -0.0 -> +1, NaN -> -1.
 *   - zero padding pads the +-1 tensor with 0: out-of-image taps contribute nothing.
 *   - K uses the same kernel size, stride and padding as the convolution; A is zero outside the
 *     image and the divisor kh*kw is constant (Eq. 10 read literally as a fixed-kernel filter).
 *   - "convolution" is cross-correlation (no kernel flip), as Alg. 2 applies the weights unflipped.
 *   - batch: N independent images, K per image, alpha per filter.
 *
 * Precision: the sign convolution is accumulated in float (every partial sum is an integer far
 * below 2^24, so it is exact) and returned as int32.  K, alpha and the final product are
 * accumulated in double and rounded once to float.
 *
 * Parity pins: every function here is pinned by tests/test_oracle_pins.py (brute force, the
 * XNOR-popcount identity, closed forms, invariants, library special cases, a hand-worked fixture).
 */
#include <stdint.h>
#include <stddef.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int N, C, H, W;      /* input   I  [N][C][H][W]       */
    int F, kh, kw;       /* filters Wt [F][C][kh][kw]     */
    int sh, sw, ph, pw;  /* stride, zero padding          */
} oracle_shape;

/* Threads the (image, filter) loop of oracle_dot will use. */
int oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static int out_dim(int in, int pad, int k, int stride) { return (in + 2 * pad - k) / stride + 1; }

int oracle_out_dims(const oracle_shape *s, int *OH, int *OW)
{
    if (!s || s->N <= 0 || s->C <= 0 || s->H <= 0 || s->W <= 0 || s->F <= 0 || s->kh <= 0 ||
        s->kw <= 0 || s->sh <= 0 || s->sw <= 0 || s->ph < 0 || s->pw < 0)
        return -1;
    if (s->H + 2 * s->ph < s->kh || s->W + 2 * s->pw < s->kw) return -1;
    *OH = out_dim(s->H, s->ph, s->kh, s->sh);
    *OW = out_dim(s->W, s->pw, s->kw, s->sw);
    return 0;
}

/* Eq. 3 / Eq. 8 with sign(0) = +1. */
static inline float sgn(float x) { return x >= 0.0f ? 1.0f : -1.0f; }

/* Step 1a (Sec. III-A): element-wise sign, as +-1.0f. */
void oracle_sign(const float *x, size_t n, float *s)
{
    for (size_t i = 0; i < n; ++i) s[i] = sgn(x[i]);
}

/*
 * Step 1a in the channel-packed encoding used at the library boundary: for a tensor
 * x[N][C][H][W], word (n, y, x, w) holds channels 32w .. 32w+31 of pixel (y, x); bit j is 1 iff
 * sign(x[n][32w+j][y][x]) = +1; bits of channels >= C are 0.  Output [N][H][W][ceil(C/32)].
 */
void oracle_pack(const float *x, int N, int C, int H, int W, uint32_t *packed)
{
    const int Cw = (C + 31) / 32;
    for (int n = 0; n < N; ++n)
        for (int y = 0; y < H; ++y)
            for (int xx = 0; xx < W; ++xx)
                for (int w = 0; w < Cw; ++w) {
                    uint32_t word = 0;
                    for (int j = 0; j < 32; ++j) {
                        const int c = 32 * w + j;
                        if (c < C && sgn(x[(((size_t)n * C + c) * H + y) * W + xx]) > 0.0f)
                            word |= (uint32_t)1 << j;
                    }
                    packed[(((size_t)n * H + y) * W + xx) * Cw + w] = word;
                }
}

/*
 * Steps 1b-1d (Sec. III-A) and the first factor of Eq. 11: dot = sign(I) (*) sign(W), direct loop.
 * Out-of-image taps are skipped.  dot[N][F][OH][OW], int32.
 */
int oracle_dot(const float *I, const float *Wt, const oracle_shape *s, int32_t *dot)
{
    int OH, OW;
    if (oracle_out_dims(s, &OH, &OW)) return -1;
    const int N = s->N, C = s->C, H = s->H, W = s->W, F = s->F, kh = s->kh, kw = s->kw;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int f = 0; f < F; ++f)
            for (int oy = 0; oy < OH; ++oy)
                for (int ox = 0; ox < OW; ++ox) {
                    float acc = 0.0f;
                    for (int c = 0; c < C; ++c)
                        for (int ky = 0; ky < kh; ++ky) {
                            const int iy = oy * s->sh - s->ph + ky;
                            if (iy < 0 || iy >= H) continue;
                            for (int kx = 0; kx < kw; ++kx) {
                                const int ix = ox * s->sw - s->pw + kx;
                                if (ix < 0 || ix >= W) continue;
                                acc += sgn(I[(((size_t)n * C + c) * H + iy) * W + ix]) *
                                       sgn(Wt[(((size_t)f * C + c) * kh + ky) * kw + kx]);
                            }
                        }
                    dot[(((size_t)n * F + f) * OH + oy) * OW + ox] = (int32_t)acc;
                }
    return 0;
}

/* Eq. 10, first half: A[n][y][x] = (sum_c |I[n][c][y][x]|) / C, in double. */
void oracle_A(const float *I, int N, int C, int H, int W, double *A)
{
    for (int n = 0; n < N; ++n)
        for (int y = 0; y < H; ++y)
            for (int x = 0; x < W; ++x) {
                double sum = 0.0;
                for (int c = 0; c < C; ++c) {
                    const double v = (double)I[(((size_t)n * C + c) * H + y) * W + x];
                    sum += v < 0.0 ? -v : v;
                }
                A[((size_t)n * H + y) * W + x] = sum / (double)C;
            }
}

/*
 * Eq. 10: K = A * k with k_ij = 1/(kh*kw), evaluated at the convolution's output positions
 * (same stride and padding), A taken as 0 outside the image.  K[N][OH][OW], float.
 * `A_scratch` must hold N*H*W doubles.
 */
int oracle_K(const float *I, const oracle_shape *s, double *A_scratch, float *K)
{
    int OH, OW;
    if (oracle_out_dims(s, &OH, &OW)) return -1;
    const int N = s->N, H = s->H, W = s->W;
    oracle_A(I, N, s->C, H, W, A_scratch);
    for (int n = 0; n < N; ++n)
        for (int oy = 0; oy < OH; ++oy)
            for (int ox = 0; ox < OW; ++ox) {
                double sum = 0.0;
                for (int ky = 0; ky < s->kh; ++ky) {
                    const int iy = oy * s->sh - s->ph + ky;
                    if (iy < 0 || iy >= H) continue;
                    for (int kx = 0; kx < s->kw; ++kx) {
                        const int ix = ox * s->sw - s->pw + kx;
                        if (ix < 0 || ix >= W) continue;
                        sum += A_scratch[((size_t)n * H + iy) * W + ix];
                    }
                }
                K[((size_t)n * OH + oy) * OW + ox] = (float)(sum / (double)(s->kh * s->kw));
            }
    return 0;
}

/* Eq. 5: alpha[f] = (sum |Wt[f]|) / (C*kh*kw), in double, rounded once. */
void oracle_alpha(const float *Wt, int F, int C, int kh, int kw, float *alpha)
{
    const size_t n = (size_t)C * kh * kw;
    for (int f = 0; f < F; ++f) {
        double sum = 0.0;
        for (size_t i = 0; i < n; ++i) {
            const double v = (double)Wt[(size_t)f * n + i];
            sum += v < 0.0 ? -v : v;
        }
        alpha[f] = (float)(sum / (double)n);
    }
}

/* Eq. 11 / step 3 (Sec. III-A): O = dot * K * alpha, product in double, rounded once. */
void oracle_out(const int32_t *dot, const float *K, const float *alpha, int N, int F, int OH,
                int OW, float *O)
{
    for (int n = 0; n < N; ++n)
        for (int f = 0; f < F; ++f)
            for (int p = 0; p < OH * OW; ++p) {
                const size_t o = ((size_t)n * F + f) * OH * OW + p;
                O[o] = (float)((double)dot[o] * (double)K[(size_t)n * OH * OW + p] *
                               (double)alpha[f]);
            }
}

/*
 * Binary-Weight-Network convolution (Sec. II-A, Eq. 1): the input keeps its real values, the
 * weights are B = sign(W), and the convolution, free of multiplications, adds or subtracts each
 * input value according to its weight's sign; the per-filter alpha of Eq. 5 scales the sum:
 *     O[n][f][oy][ox] = alpha[f] * sum_{in-image taps, c} (B = +1 ? +I : -I).
 * No K: the input is not binarised.  Same padding, stride and cross-correlation readings as the
 * XNOR path.  Accumulated in double in the plain loop order (c, ky, kx), multiplied by alpha in
 * double, rounded once to float.  S (optional) receives sum |I| over the same taps, in double: the
 * scale against which a float implementation's summation error is measured.
 */
int oracle_bwn(const float *I, const float *Wt, const oracle_shape *s, const float *alpha, float *O,
               double *S)
{
    int OH, OW;
    if (oracle_out_dims(s, &OH, &OW)) return -1;
    const int N = s->N, C = s->C, H = s->H, W = s->W, F = s->F, kh = s->kh, kw = s->kw;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int f = 0; f < F; ++f)
            for (int oy = 0; oy < OH; ++oy)
                for (int ox = 0; ox < OW; ++ox) {
                    double acc = 0.0, mag = 0.0;
                    for (int c = 0; c < C; ++c)
                        for (int ky = 0; ky < kh; ++ky) {
                            const int iy = oy * s->sh - s->ph + ky;
                            if (iy < 0 || iy >= H) continue;
                            for (int kx = 0; kx < kw; ++kx) {
                                const int ix = ox * s->sw - s->pw + kx;
                                if (ix < 0 || ix >= W) continue;
                                const double v = (double)I[(((size_t)n * C + c) * H + iy) * W + ix];
                                if (Wt[(((size_t)f * C + c) * kh + ky) * kw + kx] >= 0.0f)
                                    acc += v;
                                else
                                    acc -= v;
                                mag += v < 0.0 ? -v : v;
                            }
                        }
                    O[(((size_t)n * F + f) * OH + oy) * OW + ox] = (float)(acc * (double)alpha[f]);
                    if (S && f == 0) S[((size_t)n * OH + oy) * OW + ox] = mag;
                }
    return 0;
}

/*
 * Real-valued ("vanilla") convolution: the float comparison that Sec. IV's Table I sets the XNOR
 * convolution against.  Input and weights keep their values:
 *     O[n][f][oy][ox] = sum_{c, in-image taps} I[n][c][iy][ix] * Wt[f][c][ky][kx],
 * cross-correlation (no kernel flip), zero padding and stride as in the XNOR path, no alpha and no
 * K.  Every product of two floats is exact in double; they are added in double in the plain loop
 * order (c, ky, kx) and the sum is rounded once to float.  S (optional) receives sum |I * Wt| over
 * the same terms, in double: the scale against which a float implementation's summation error is
 * measured.
 */
int oracle_conv_fp32(const float *I, const float *Wt, const oracle_shape *s, float *O, double *S)
{
    int OH, OW;
    if (oracle_out_dims(s, &OH, &OW)) return -1;
    const int N = s->N, C = s->C, H = s->H, W = s->W, F = s->F, kh = s->kh, kw = s->kw;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int f = 0; f < F; ++f)
            for (int oy = 0; oy < OH; ++oy)
                for (int ox = 0; ox < OW; ++ox) {
                    double acc = 0.0, mag = 0.0;
                    for (int c = 0; c < C; ++c)
                        for (int ky = 0; ky < kh; ++ky) {
                            const int iy = oy * s->sh - s->ph + ky;
                            if (iy < 0 || iy >= H) continue;
                            for (int kx = 0; kx < kw; ++kx) {
                                const int ix = ox * s->sw - s->pw + kx;
                                if (ix < 0 || ix >= W) continue;
                                const double t = (double)I[(((size_t)n * C + c) * H + iy) * W + ix] *
                                                 (double)Wt[(((size_t)f * C + c) * kh + ky) * kw + kx];
                                acc += t;
                                mag += t < 0.0 ? -t : t;
                            }
                        }
                    const size_t o = (((size_t)n * F + f) * OH + oy) * OW + ox;
                    O[o] = (float)acc;
                    if (S) S[o] = mag;
                }
    return 0;
}
