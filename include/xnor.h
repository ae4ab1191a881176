/*
 * xnor.h -- C ABI of the MI355X (gfx950) XNOR-Net binary convolution forward pass.
 *
 * The calls are the steps of the binary-convolution pipeline of "Optimization of XNOR Convolution
 * for Binary Convolutional Neural Networks on GPU" (Sec. III-A step list):
 *
 *   xnor_binarize_pack  step 1a   sign-binarise and bit-pack along channels      (Eq. 3, Eq. 8)
 *   xnor_scale_K        step 2a   scaling map K = box filter of mean_c |I|       (Eq. 10)
 *   xnor_alpha                    per-filter scale alpha = mean |W|              (Eq. 5)
 *   xnor_conv2d_fwd     steps 1b-1d, 2b, 3: XNOR + popcount convolution, then
 *                       out = dot * K * alpha                                    (Eq. 11)
 *
 * Problem statement (Sec. II): input I of C channels x H x W per image, filters of C x kh x kw with
 * one alpha each, zero padding.  A batch is N independent images; K is per image.
 *
 * Conventions shared by every call
 *   - Every data pointer is a DEVICE pointer owned by the caller.  The library allocates nothing,
 *     frees nothing and keeps no state between calls.  Inputs are never written; outputs are
 *     overwritten in full.  Outputs must not alias inputs.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls enqueue their
 *     kernels on it and return without synchronising; buffers must stay alive until the stream
 *     has passed them.
 *   - Tensors are dense, row-major, in the index order written in each comment.
 *   - sign(x) = +1 if x >= 0 else -1 (so +0.0 and -0.0 are +1, NaN is -1).  Bit 1 stands for +1,
 *     bit 0 for -1 (Sec. III-A step 1c).
 *   - Packed layout: for a tensor x[N][C][H][W] the packed form is uint32 [N][H][W][Cw],
 *     Cw = ceil(C/32); bit j of word w of a pixel is the sign bit of channel 32w+j; bits of
 *     channels >= C are 0.  Filters Wt[F][C][kh][kw] are packed by the same call as F "images" of
 *     kh x kw pixels, giving [F][kh][kw][Cw].
 *   - Return value: XNOR_OK (0) or a negative xnor_status.  Arguments are validated on the host
 *     before anything is enqueued; on an error nothing has been launched.  XNOR_E_HIP reports a
 *     launch failure (text via xnor_strerror / xnor_last_hip_error).
 */
#ifndef XNOR_H
#define XNOR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    XNOR_OK = 0,
    XNOR_E_NULL = -1,        /* a required pointer is NULL                                        */
    XNOR_E_SHAPE = -2,       /* a dimension <= 0, stride <= 0, pad < 0, empty output, or a tensor
                                too large for the kernels' 31-bit pixel / 63-bit byte indexing     */
    XNOR_E_ALIGN = -3,       /* a pointer is not aligned as the call requires                     */
    XNOR_E_HIP = -4,         /* the HIP runtime refused a launch                                  */
    XNOR_E_UNSUPPORTED = -5, /* the requested algorithm cannot run this shape                     */
    XNOR_E_WORKSPACE = -6    /* the requested algorithm needs a (larger) workspace                */
} xnor_status;

/* Geometry of one layer (Sec. II problem statement; stride/padding as in Sec. III-B step 1). */
typedef struct {
    int N, C, H, W;     /* input   I  [N][C][H][W]  fp32                                          */
    int F, kh, kw;      /* filters Wt [F][C][kh][kw] fp32                                         */
    int sh, sw;         /* stride  >= 1                                                           */
    int ph, pw;         /* zero padding >= 0 (padded taps contribute nothing to dot or K)         */
} xnor_shape;

/* Which convolution kernel xnor_conv2d_fwd_algo runs. */
typedef enum {
    XNOR_ALGO_AUTO = 0,     /* pick per shape (what xnor_conv2d_fwd does)                         */
    XNOR_ALGO_DIRECT = 1,   /* one thread per output, v_xor + v_bcnt, any shape                   */
    XNOR_ALGO_TILED = 2,    /* LDS-staged packed halo, wave-uniform filter words, register tile   */
    XNOR_ALGO_MFMA = 3,     /* +-1 expanded to FP4 in LDS, v_mfma_f32_32x32x64_f8f6f4: persistent
                               workgroups where the shape allows, else as XNOR_ALGO_MFMA_BANDS    */
    XNOR_ALGO_MFMA_BANDS = 4, /* the same arithmetic with one workgroup per band of output rows
                               (xnor_conv2d_fwd_algo only; tests and measurements)                */
    XNOR_ALGO_MFMA_SPLIT = 5 /* xnor_bwn_conv2d_fwd_algo only: the fp32 input split exactly into
                               three bf16 terms, v_mfma_f32_32x32x16_bf16 against +-1 weights     */
} xnor_algo;

/* Host helpers (no GPU work). */
int xnor_out_dim(const xnor_shape *s, int *OH, int *OW); /* OH = (H+2ph-kh)/sh+1, OW likewise      */
int xnor_packed_words(int C);                            /* ceil(C/32), or XNOR_E_SHAPE if C <= 0  */
const char *xnor_strerror(int status);                   /* static string, never NULL              */
const char *xnor_last_hip_error(void);                   /* text of the last XNOR_E_HIP on this
                                                            thread ("" if none)                    */

/*
 * Step 1a (Sec. III-A): packed[n][y][x][w] bit j = (x[n][32w+j][y][x] >= 0).
 *   x       in   fp32 [N][C][H][W]
 *   packed  out  uint32 [N][H][W][ceil(C/32)], 4-byte aligned
 * Used for the input (N images) and for the filters (x = Wt, N = F, H = kh, W = kw).
 */
int xnor_binarize_pack(const float *x, int N, int C, int H, int W, uint32_t *packed, void *stream);

/*
 * Eq. 10: A[n][y][x] = (1/C) sum_c |I[n][c][y][x]|, then
 * K[n][oy][ox] = (1/(kh*kw)) * sum over in-image taps of A[n][oy*sh-ph+ky][ox*sw-pw+kx]
 * (A is 0 outside the image; the divisor is constant; K uses the convolution's stride and pad).
 *   I       in   fp32 [N][C][H][W]
 *   A_work  out  fp32 [N][H][W]   caller-owned workspace; holds A on return
 *   K       out  fp32 [N][OH][OW]
 */
int xnor_scale_K(const float *I, const xnor_shape *s, float *A_work, float *K, void *stream);

/*
 * Eq. 5: alpha[f] = (1/(C*kh*kw)) sum |Wt[f][c][ky][kx]|.
 *   Wt     in   fp32 [F][C][kh][kw]
 *   alpha  out  fp32 [F]
 */
int xnor_alpha(const float *Wt, int F, int C, int kh, int kw, float *alpha, void *stream);

/*
 * Step 1a and Eq. 10 in one pass over I (each input element is read from HBM once): the packed
 * input of xnor_binarize_pack(I) and the A and K of xnor_scale_K(I), same definitions, same layouts.
 * The paper computes the bit path and the scale path as separate kernels (Sec. III-C).
 *   I       in   fp32 [N][C][H][W]
 *   Ipk     out  uint32 [N][H][W][ceil(C/32)]
 *   A_work  out  fp32 [N][H][W]   caller-owned workspace; holds A on return
 *   K       out  fp32 [N][OH][OW], or NULL: then only Ipk and A are produced (for
 *                xnor_conv2d_fwd_expanded given A, which forms K itself)
 */
int xnor_input_prepare(const float *I, const xnor_shape *s, uint32_t *Ipk, float *A_work, float *K,
                       void *stream);

/*
 * xnor_input_prepare, xnor_filter_prepare and (with a workspace) xnor_filter_expand, all declared
 * below, as ONE call, for a layer whose input and filters are both new (the benchmark step; a first
 * inference).  Same outputs, same definitions; but for extreme shapes (more than 256 taps or 16384
 * channels, filters too large for one workgroup's LDS) all of it runs in a single launch, the filter
 * blocks beside the HBM-bound input blocks (a second launch forms K where it is asked for).  K may
 * be NULL as in xnor_input_prepare.  workspace may be NULL; if given
 * it is filled for xnor_conv2d_fwd_expanded* (XNOR_E_UNSUPPORTED / XNOR_E_WORKSPACE as in
 * xnor_filter_expand).
 */
int xnor_prepare(const float *I, const float *Wt, const xnor_shape *s, uint32_t *Ipk, float *A_work,
                 float *K, uint32_t *Wpk, float *M_work, float *alpha, void *workspace,
                 size_t workspace_bytes, void *stream);

/*
 * Per-model filter preparation in one pass over Wt: the packed filters of xnor_binarize_pack(Wt)
 * (step 1a, Eq. 3) and the alpha of xnor_alpha(Wt) (Eq. 5).
 *   Wt      in   fp32 [F][C][kh][kw]
 *   Wpk     out  uint32 [F][kh][kw][ceil(C/32)]
 *   M_work  out  fp32 [F][kh][kw]  caller-owned workspace; holds mean_c |Wt| per tap on return
 *   alpha   out  fp32 [F]
 */
int xnor_filter_prepare(const float *Wt, int F, int C, int kh, int kw, uint32_t *Wpk, float *M_work,
                        float *alpha, void *stream);

/*
 * Steps 1b-1d and 3 (Sec. III-A), Eq. 11:
 *   dot[n][f][oy][ox] = sum over in-image taps (ky,kx) and channels c of
 *                       sign(I[n][c][oy*sh-ph+ky][ox*sw-pw+kx]) * sign(Wt[f][c][ky][kx])
 *                     = N_valid - 2 * popcount(Ipk xor Wpk)   over the same taps,
 *                       N_valid = C * (number of in-image taps)
 *   out = float(dot) * K[n][oy][ox] * alpha[f]
 *
 *   Ipk    in   uint32 [N][H][W][Cw]     from xnor_binarize_pack(I)
 *   Wpk    in   uint32 [F][kh][kw][Cw]   from xnor_binarize_pack(Wt)
 *   K      in   fp32   [N][OH][OW]
 *   alpha  in   fp32   [F]
 *   out    out  fp32   [N][F][OH][OW]
 *   dot    out  int32  [N][F][OH][OW], or NULL when the raw binary dot products are not wanted
 *   workspace        caller-owned device scratch of `workspace_bytes` bytes, 16-byte aligned, or
 *                    NULL.  The matrix-core kernel expands the filter bits into it on every call
 *                    (its contents mean nothing afterwards).  With NULL, or fewer bytes than
 *                    xnor_conv2d_workspace_bytes reports, the call runs a kernel that needs none.
 * Packed pointers must be 4-byte aligned (16-byte alignment lets the kernels use wider loads).
 */
int xnor_conv2d_fwd(const uint32_t *Ipk, const uint32_t *Wpk, const float *K, const float *alpha,
                    const xnor_shape *s, float *out, int32_t *dot, void *workspace,
                    size_t workspace_bytes, void *stream);

/* Bytes of workspace with which xnor_conv2d_fwd can run its fastest kernel on this shape
 * (0 if no kernel for this shape uses a workspace).  Host only. */
int xnor_conv2d_workspace_bytes(const xnor_shape *s, size_t *bytes);

/*
 * The matrix-core kernel of xnor_conv2d_fwd in two calls, for callers whose filters stay the same
 * over many inputs (inference): xnor_filter_expand is per-model work like xnor_filter_prepare,
 * xnor_conv2d_fwd_expanded is the per-input convolution (steps 1b-1d and 3, Eq. 11) and computes
 * exactly what xnor_conv2d_fwd computes.
 *   xnor_filter_expand        writes the filters' +-1 values in the kernel's operand order into
 *                             `workspace` (xnor_conv2d_workspace_bytes bytes, 16-byte aligned);
 *                             the contents stay valid for this shape until overwritten.
 *   xnor_conv2d_fwd_expanded  reads that workspace instead of Wpk; it must have been filled for the
 *                             same shape.  Exactly one of K and A is given (the other NULL, else
 *                             XNOR_E_NULL): K [N][OH][OW] as in xnor_conv2d_fwd, or the channel mean
 *                             A [N][H][W] (Eq. 10, first half), from which each workgroup forms the
 *                             K of its own output pixels while its first operands are on their way
 *                             (same sum, order and rounding as xnor_box_filter_K, so the outputs
 *                             are bit-identical), which saves the box-filter launch between the
 *                             input pass and the convolution.  Other arguments as in
 *                             xnor_conv2d_fwd.
 * Both return XNOR_E_UNSUPPORTED where xnor_conv2d_workspace_bytes reports 0 and XNOR_E_WORKSPACE
 * for a workspace that is too small.
 */
int xnor_filter_expand(const uint32_t *Wpk, const xnor_shape *s, void *workspace,
                       size_t workspace_bytes, void *stream);
int xnor_conv2d_fwd_expanded(const uint32_t *Ipk, const void *workspace, size_t workspace_bytes,
                             const float *K, const float *A, const float *alpha, const xnor_shape *s,
                             float *out, int32_t *dot, void *stream);

/*
 * Chained layers (the paper's closing proposal, Sec. V: hand the next kernel the binary outputs
 * themselves, with no conversion to integers in between).  When the consumer of this layer's output O (Eq. 11) is
 * another binary convolution, all it needs of O is what xnor_input_prepare would compute from it:
 * the packed signs of O along its channels (= this layer's filters) and the channel mean of |O|
 * (Eq. 10).  xnor_conv2d_fwd_chain produces exactly these and never writes the fp32 O:
 *   Opk     out  uint32 [N][OH][OW][ceil(F/32)]  = xnor_binarize_pack(O): bit = (O >= 0) with
 *                O = float(dot) * (K * alpha) formed in fp32 as in xnor_conv2d_fwd; tail bits 0
 *   A_next  out  fp32   [N][OH][OW]              = (1/F) sum_f |O[n][f][oy][ox]|
 *   workspace    caller-owned, 16-byte aligned, xnor_conv2d_chain_workspace_bytes bytes (filter
 *                expansion plus per-filter-tile partial sums); contents mean nothing afterwards.
 *   K, A         exactly one is given (the other NULL, else XNOR_E_NULL): K [N][OH][OW], or this
 *                layer's channel mean A [N][H][W] (what the previous chained layer left as its
 *                A_next), from which K is formed inside the kernel as in xnor_conv2d_fwd_expanded,
 *                so that a chain of layers needs no xnor_box_filter_K calls in between.
 *                Bit-identical results.
 *   Wpk          the packed filters, expanded into the workspace by a launch of this call; or NULL
 *                for filters that do not change from call to call (every layer of a chained
 *                network at inference): the caller has run xnor_filter_expand (or xnor_prepare) on
 *                this same workspace, whose first xnor_conv2d_workspace_bytes bytes therefore hold
 *                the expanded filters and are only read here; the rest (up to
 *                xnor_conv2d_chain_workspace_bytes) is the scratch for the per-filter-tile sums.
 *                Same results bit for bit, one launch less per layer.
 * The next layer continues with A_next as its A (or with xnor_box_filter_K(A_next, its shape, K))
 * and a convolution on Opk.
 * Runs on the matrix-core kernel only: XNOR_E_UNSUPPORTED where
 * xnor_conv2d_chain_workspace_bytes reports 0, XNOR_E_WORKSPACE for a workspace that is too small.
 */
int xnor_conv2d_chain_workspace_bytes(const xnor_shape *s, size_t *bytes);
int xnor_conv2d_fwd_chain(const uint32_t *Ipk, const uint32_t *Wpk, const float *K, const float *A,
                          const float *alpha, const xnor_shape *s, uint32_t *Opk, float *A_next,
                          void *workspace, size_t workspace_bytes, void *stream);

/*
 * Second half of Eq. 10 on its own: K = box filter of a given A (taps 1/(kh*kw), zero outside the
 * image, the convolution's stride and padding), for callers that already hold A (chained layers).
 *   A  in   fp32 [N][H][W]      K  out  fp32 [N][OH][OW]      (s->C and s->F are not used)
 */
int xnor_box_filter_K(const float *A, const xnor_shape *s, float *K, void *stream);

/*
 * The whole forward pass in one call for images with few channels: first layers, and the workload
 * the paper times (Sec. IV, Tables I-III: one channel, a 3x3 filter, 256^2 ... 2048^2 pixels).
 * Computes exactly what xnor_input_prepare + xnor_conv2d_fwd compute -- the signs of I (step 1a),
 * K (Eq. 10, steps 2a-2b), the binary dot products over spatially packed windows (Sec. III-B,
 * steps 1b-1d) and the rescale (step 3, Eq. 11) -- from one read of the fp32 image, with nothing
 * intermediate written to memory.
 *   I      in   fp32 [N][C][H][W]
 *   Wpk    in   uint32 [F][kh][kw][1]   packed filter signs (xnor_filter_prepare / xnor_binarize_pack)
 *   alpha  in   fp32 [F]
 *   out    out  fp32 [N][F][OH][OW]
 *   dot    out  int32 [N][F][OH][OW] or NULL
 * Takes 1 <= C <= 4, kh = kw in {3, 5, 7}, any stride and padding; XNOR_E_UNSUPPORTED otherwise
 * (xnor_forward_image_supported: 1 if the shape is taken, 0 if not, negative status for a bad shape).
 * K is formed in fp32 from fp32 partial sums (row sums, then their sum): within kw*C + kh roundings
 * of the exact value.
 */
int xnor_forward_image_supported(const xnor_shape *s);
int xnor_forward_image(const float *I, const uint32_t *Wpk, const float *alpha, const xnor_shape *s,
                       float *out, int32_t *dot, void *stream);

/*
 * Binary-Weight-Network convolution (Sec. II-A, Eq. 1, with alpha from Eq. 5): real-valued input,
 * binary weights B = sign(W), so the convolution needs no multiplications:
 *     out[n][f][oy][ox] = alpha[f] * sum over in-image taps and channels of (B = +1 ? +I : -I).
 * The input is not binarised and there is no K.  Zero padding, stride and cross-correlation as in
 * xnor_conv2d_fwd.
 *   I      in   fp32 [N][C][H][W]
 *   Wpk    in   uint32 [F][kh][kw][ceil(C/32)]   packed filter signs, bit 1 = +1
 *   alpha  in   fp32 [F]
 *   out    out  fp32 [N][F][OH][OW]
 * The sum is formed in fp32 (fp32 matrix-core accumulation, or a short chain of fp32 partial sums
 * in the one-thread-per-output kernel); its rounding error is relative to alpha * sum |I| over the
 * window, not to |out|.  No workspace.  xnor_bwn_conv2d_fwd_algo: XNOR_ALGO_AUTO (the first of
 * MFMA_SPLIT, MFMA, DIRECT that takes the shape), XNOR_ALGO_DIRECT (any shape), XNOR_ALGO_MFMA (fp32
 * matrix instruction with +-1.0 as one operand; XNOR_E_UNSUPPORTED where the input rows under 32
 * output pixels do not fit in 128 KB of LDS, or kh*kw > 64) or XNOR_ALGO_MFMA_SPLIT (every input
 * value split into three bf16 terms whose sum is the value, bf16 matrix instruction with +-1
 * weights, fp32 accumulation: the same products, three instructions at 16 times the rate instead of
 * eight; an input that is not finite gives NaN, not an infinity, and a term below the normal range
 * is flushed, which adds at most alpha * 2^-125 per input value under the window to the error;
 * XNOR_E_UNSUPPORTED where the input rows under 32 output pixels are more than 512 staged
 * positions or do not fit, twice over and with two sets of filter words, in 160 KB of LDS, or
 * kh*kw > 64); other values XNOR_E_UNSUPPORTED.
 */
int xnor_bwn_conv2d_fwd(const float *I, const uint32_t *Wpk, const float *alpha, const xnor_shape *s,
                        float *out, void *stream);
int xnor_bwn_conv2d_fwd_algo(const float *I, const uint32_t *Wpk, const float *alpha,
                             const xnor_shape *s, float *out, int algo, void *stream);

/* The algorithm XNOR_ALGO_AUTO resolves to in xnor_bwn_conv2d_fwd_algo for this shape (an
 * xnor_algo), or a negative status.  Host only. */
int xnor_bwn_pick_algo(const xnor_shape *s);

/*
 * The launch XNOR_ALGO_MFMA_SPLIT makes for this shape on a GPU of `compute_units` units (0: the
 * current device's, 256 where there is none).  Host only; for tests and for reading a timing.
 *   *tiles         32-pixel tiles of one image a workgroup takes (1..6; an image's last workgroup
 *                  the rest)
 *   *row_segments  0: a tile is 32 consecutive output pixels; k > 0: a tile is one of the k
 *                  32-pixel segments of one output row (the row's last one short)
 *   *lds_bytes     dynamic LDS per workgroup (<= 160 KB; <= 80 KB lets two share a unit)
 *   *workgroups    the grid: N x ceil(F/128) x ceil(tiles of an image / *tiles)
 * XNOR_E_UNSUPPORTED where XNOR_ALGO_MFMA_SPLIT would return it; XNOR_E_SHAPE for compute_units < 0.
 */
int xnor_bwn_split_plan(const xnor_shape *s, int compute_units, int *tiles, int *row_segments,
                        size_t *lds_bytes, long long *workgroups);

/*
 * Real-valued ("vanilla") convolution: the float comparison that the paper's timings set the XNOR
 * convolution against (Sec. IV, Table I).  Nothing is binarised and there are no scaling factors:
 *     out[n][f][oy][ox] = sum over in-image taps and channels of I * Wt
 * with zero padding, stride and cross-correlation as in xnor_conv2d_fwd.
 *   I      in   fp32 [N][C][H][W]
 *   Wt     in   fp32 [F][C][kh][kw]
 *   out    out  fp32 [N][F][OH][OW]
 * Products and sums are fp32 (fp32 matrix-core accumulation, or chains of fp32 partial sums in the
 * one-thread-per-output kernel); the rounding error is relative to sum |I * Wt| over the window,
 * not to |out|.  No workspace.  xnor_conv2d_fp32_fwd_algo: XNOR_ALGO_AUTO (the matrix-core kernel
 * where it takes the shape and the layer has at least 8 filters and 4 channels), XNOR_ALGO_DIRECT
 * (any shape) or XNOR_ALGO_MFMA (XNOR_E_UNSUPPORTED where the staged input rows and the chunk's
 * weights, kh*kw x 8 channels x 128 filters, do not fit in 128 KB of LDS, or kh*kw > 64); other
 * values XNOR_E_UNSUPPORTED.
 */
int xnor_conv2d_fp32_fwd(const float *I, const float *Wt, const xnor_shape *s, float *out, void *stream);
int xnor_conv2d_fp32_fwd_algo(const float *I, const float *Wt, const xnor_shape *s, float *out, int algo,
                              void *stream);

/* Same as xnor_conv2d_fwd, with the kernel chosen by the caller (tests and measurements run every
 * variant).  Returns XNOR_E_UNSUPPORTED if `algo` cannot run this shape, XNOR_E_WORKSPACE if it
 * needs more workspace than given; XNOR_ALGO_DIRECT runs every shape without workspace. */
int xnor_conv2d_fwd_algo(const uint32_t *Ipk, const uint32_t *Wpk, const float *K,
                         const float *alpha, const xnor_shape *s, float *out, int32_t *dot,
                         void *workspace, size_t workspace_bytes, int algo, void *stream);

/*
 * For callers that cannot allocate device memory and have no workspace to hand in (code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc): xnor_conv2d_fwd_algo with
 * XNOR_ALGO_MFMA, its workspace (the filters expanded to matrix-core operands) taken from an array
 * of XNOR_STATIC_SCRATCH_BYTES that the library holds on every GPU it runs on until the process
 * ends.  Same arguments, layouts and results as xnor_conv2d_fwd_algo; the call allocates nothing.
 * Returns XNOR_E_UNSUPPORTED for shapes the matrix-core kernel does not take and XNOR_E_WORKSPACE
 * for shapes whose expanded filters exceed the array (xnor_conv2d_workspace_bytes(s) >
 * XNOR_STATIC_SCRATCH_BYTES).  All calls on one GPU share that GPU's array and each rewrites it:
 * calls that overlap on one GPU (different streams, or threads) race; calls on one stream do not.
 */
#define XNOR_STATIC_SCRATCH_BYTES (4u << 20)
int xnor_conv2d_fwd_static(const uint32_t *Ipk, const uint32_t *Wpk, const float *K,
                           const float *alpha, const xnor_shape *s, float *out, int32_t *dot,
                           void *stream);

/* The algorithm XNOR_ALGO_AUTO resolves to for this shape when given `workspace_bytes` of
 * workspace (an xnor_algo), or a negative status. */
int xnor_conv2d_pick_algo(const xnor_shape *s, size_t workspace_bytes);

/*
 * Measurement probes (no part of the forward pass): what the GPU at hand sustains on the resources
 * the kernels above are priced against, for reading a roofline fraction against a measured
 * ceiling beside the published one.  Each enqueues one kernel on `stream` and returns; the caller
 * times it with events.
 *   xnor_probe_mfma_fp4      `workgroups` x 4 waves each run `iters` x 8 register-only
 *                            v_mfma_f32_32x32x64_f8f6f4 (both operands FP4 +-1, the convolution's
 *                            instruction); *flops receives the flops issued (2 per multiply-add)
 *   xnor_probe_mfma_bf16     the same with `iters` x 6 v_mfma_f32_32x32x16_bf16 (the Binary-Weight-
 *                            Network kernel's instruction): A operands +-1.0, B operands +-1.0
 *                            (random_b = 0) or bf16 values with random significands (random_b != 0;
 *                            the rate the chip holds depends on the operand values)
 *   xnor_probe_xor_popcount  `workgroups` x 256 lanes each run `iters` x 8 register-only
 *                            v_xor_b32 + v_bcnt_u32_b32 pairs; *binary_macs receives 32 per lane
 *                            and pair
 *   xnor_probe_copy          copies `bytes` (a multiple of 16; both pointers 16-byte aligned) from
 *                            src to dst, 16 bytes per lane
 *   xnor_probe_read          reads `bytes` (a multiple of 16, 16-byte aligned) of src, 16 bytes per
 *                            lane, and writes nothing
 *   xnor_probe_store_beside_mfma   what a wave's global stores cost while another wave of its SIMD
 *                            runs matrix instructions (the convolution's epilogue beside the other
 *                            wave group's loop): `workgroups` x 8 waves; waves 0-3 of each run a
 *                            register-only FP4 matrix loop (matrix_loop 1: back to back, 2: the pipe
 *                            idle an eighth of the time, 0: no loop), waves 4-7 each store `reps` x
 *                            32 KB to dst as 16-byte (wide != 0) or 4-byte stores per lane and write
 *                            the shader-clock cycles they took to cycles[workgroup][4] (device,
 *                            8-byte aligned).  dst (device, 16-byte aligned) holds workgroups x reps
 *                            x 128 KB, every byte of which is written; sink here is 8 bytes
 * `sink` (device, 4 bytes) is never written in practice; it keeps the loops alive.  `flops` and
 * `binary_macs` are host pointers.  XNOR_E_SHAPE for counts <= 0 or beyond 2^20 workgroups /
 * 2^24 iterations (store probe: 4096 workgroups, 64 repetitions, matrix_loop outside 0..2, dst_bytes
 * too small), or a byte count that is 0 or no multiple of 16.
 */
int xnor_probe_mfma_fp4(int workgroups, int iters, float *sink, double *flops, void *stream);
int xnor_probe_mfma_bf16(int workgroups, int iters, int random_b, float *sink, double *flops, void *stream);
int xnor_probe_xor_popcount(int workgroups, int iters, uint32_t *sink, double *binary_macs, void *stream);
int xnor_probe_copy(const void *src, void *dst, size_t bytes, void *stream);
int xnor_probe_read(const void *src, size_t bytes, uint32_t *sink, void *stream);
int xnor_probe_store_beside_mfma(int workgroups, int reps, int wide, int matrix_loop, float *dst, size_t dst_bytes,
                                 unsigned long long *cycles, float *sink, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* XNOR_H */
