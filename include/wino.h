/*
 * libwino — Winograd-algorithm 2-D convolution (3x3 filter, stride 1, zero pad 1,
 * dilation 1, groups 1) for AMD Instinct MI355X (gfx950).
 *
 * The operator is the 2-D convolution that the paper's Section "Techniques"
 * replaces by a Winograd path with three steps: (i) preprocess of the filter and
 * of the activation, (ii) element-wise multiplication of the preprocessed
 * tensors (summed over input channels, i.e. alpha^2 batched matrix products),
 * (iii) postprocess of the intermediate result.  Tensor orders follow the header
 * of the paper's Table 1 (filter [KW,KH,IC,OC], activation [IW,IH,IC,N], fastest
 * dimension first): w[K][C][3][3], x[N][C][H][W], y[N][K][H][W].
 *
 *     y[n,k,i,j] = bias[k] + sum_{c,r,s} xhat[n,c,i+r-1,j+s-1] * w[k,c,r,s]
 *     xhat = x inside the image, 0 outside            (cross-correlation, no flip)
 *
 * Notation: m = output tile edge (2 or 4), alpha = m+2, th = ceil(H/m),
 * tw = ceil(W/m), T = N*th*tw tiles, tile index t = (n*th+ti)*tw+tj,
 * xi*alpha+nu in [0, alpha^2) = position inside the transformed tile.
 *
 * General conventions
 *  - Every pointer named x, w, w_t->data, bias, y, U, V, M or workspace is DEVICE
 *    memory owned by the caller; the library keeps nothing after a call returns
 *    (wino_conv2d borrows its workspace from the stream-ordered allocator and
 *    returns it on the same stream).  wino_filter is a HOST struct.
 *  - All work is enqueued on `stream` (a hipStream_t passed as void*; NULL = the
 *    default stream).  No call synchronises with the host.
 *  - Arguments are validated on the host before anything is launched; errors come
 *    back as a wino_status and nothing is enqueued.  No exceptions, no abort.
 *  - Device pointers must be 16-byte aligned.  x and y must not overlap.
 *  - bias is always fp32 [K] and may be NULL.  Accumulation is always fp32.
 *  - Results are deterministic run to run (no atomics).
 *  - fp16 range: the F4 activation transform can grow values by up to 100x, so
 *    |x| must stay below ~650 on the fp16 F4 path (F2: 4x, ~16000).  bf16 and fp32
 *    have the range of fp32.
 */
#ifndef WINO_H
#define WINO_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum wino_status {
    WINO_OK = 0,
    WINO_ERR_NULL = 1,       /* a required pointer is NULL                         */
    WINO_ERR_DIM = 2,        /* a dimension is < 1, mismatches w_t, or overflows   */
    WINO_ERR_DTYPE = 3,      /* dtype enum out of range or unsupported here        */
    WINO_ERR_VARIANT = 4,    /* variant enum out of range or unsupported here      */
    WINO_ERR_ALIGN = 5,      /* a device pointer is not 16-byte aligned            */
    WINO_ERR_WORKSPACE = 6,  /* workspace NULL or smaller than wino_workspace_bytes*/
    WINO_ERR_ALIAS = 7,      /* x and y byte ranges overlap                        */
    WINO_ERR_HIP = 8,        /* a HIP call (launch, allocation) failed             */
    WINO_ERR_LAYOUT = 9,     /* layout enum out of range or unsupported here       */
    WINO_ERR_SCRATCH = 10    /* wino_conv2d_static: needs more than wino_static_scratch_bytes() */
} wino_status;

/* Storage type of x, w, y and of the transformed tensors U and V.  Accumulation is fp32 for all three.
 * Relative L2 error against an exact result on unit-variance data, from the rounding of U, V and y alone:
 *   fp32  <= 1e-5;   fp16  F(2x2) ~5e-4, F(4x4) ~3e-3, direct ~2e-4  (<= 5e-3);
 *   bf16  F(2x2) ~4e-3 (<= 8e-3), F(4x4) ~2.5e-2 (<= 4e-2; WINO_AUTO never picks it), direct ~1.7e-3 (<= 3e-3). */
typedef enum wino_dtype { WINO_F32 = 0, WINO_F16 = 1, WINO_BF16 = 2 } wino_dtype;

/*
 * WINO_F2 / WINO_F4: Winograd F(2x2,3x3) / F(4x4,3x3), three kernels (activation
 * transform, batched MFMA GEMM, output transform).  WINO_AUTO: the library picks F2,
 * F4 or one of the fused variants per shape and storage type (wino_resolve_variant).  WINO_DIRECT: direct correlation; a filter prepared with it
 * (wino_filter_transform) makes wino_conv2d / wino_conv2d_ex run the implicit-GEMM
 * MFMA kernel described at the end of this header (no transformed tensors, output
 * rounding only; faster than the Winograd path where there are few channels and
 * many pixels, see wino_recommend_variant).  wino_direct_conv2d is a third thing:
 * a one-lane-per-output checking kernel.
 * WINO_FUSED_F2: F(2x2,3x3) with steps (ii) and (iii) in ONE kernel (two launches per convolution
 * instead of three).  Step (iii) is linear in the product, so a workgroup that owns a block of
 * (output channels x tiles) walks the 16 positions in turn, keeps one product block in the MFMA
 * accumulators and adds it at once, with its +-1 coefficients, into four output accumulators; the
 * product M is never stored (the paper's locality argument: dependent steps stay on chip).  Same U and
 * V as WINO_F2, same error (~5e-4 for fp16); workspace = V only.
 * WINO_FUSED_F4: the same for F(4x4,3x3), two-byte storage types only (WINO_ERR_DTYPE for fp32).  An output tile has 16 values,
 * so step (iii) is folded in one dimension at a time: four row sums per row of the transformed tile, added into the 16 output
 * accumulators when the row is complete.  Same U and V as WINO_F4, same error (~3e-3 for fp16); workspace = V only.  Meant for
 * large images, where the unfused path is bound by writing and re-reading the product.
 */
typedef enum wino_variant { WINO_AUTO = 0, WINO_DIRECT = 1, WINO_F2 = 2, WINO_F4 = 4, WINO_FUSED_F2 = 12, WINO_FUSED_F4 = 14 } wino_variant;

/* Layout of x and y only (w is always [K][C][3][3]); NHWC = x[N][H][W][C], y[N][H][W][K]. */
typedef enum wino_layout { WINO_NCHW = 0, WINO_NHWC = 1 } wino_layout;

/* Host-side descriptor of a transformed filter.  `data` is the caller's device
 * buffer; the blob holds no pointers and can be copied or saved by the caller. */
typedef struct wino_filter {
    void *data;      /* device, U[alpha^2][K][Cp] in `dtype`, Cp = C rounded up to 8 */
    int K, C;
    int dtype;       /* wino_dtype   */
    int variant;     /* wino_variant, resolved: WINO_F2, WINO_F4, WINO_FUSED_F2, WINO_FUSED_F4 or WINO_DIRECT */
} wino_filter;

int wino_version(void);                         /* major*10000 + minor*100 + patch */
const char *wino_status_string(int status);     /* static string, never NULL       */

/* WINO_AUTO -> WINO_F2, WINO_F4, WINO_FUSED_F2 or WINO_FUSED_F4 for this shape and storage type, by measured speed within
 * the type's error bound (F4 from 64 tiles on; fp32 with C > 640 and bf16 stay on F(2x2); the fused variants where they
 * measured faster: 2-byte storage, K >= 32, and F(2x2) with >= 4096 tiles, or F(4x4) with >= 4096 tiles, at most 512
 * input and output channels and at least 512 blocks of 64 output channels x 64 tiles).  Other values are returned as they are; -1 on bad arguments (a variant that does not exist
 * for the storage type included). */
int wino_resolve_variant(int N, int C, int H, int W, int K, int dtype, int variant);

/* A Winograd variant or WINO_DIRECT, whichever was measured faster for 3x3 / stride 1 on shapes like this one
 * (the direct path where sqrt(C*K) is small and the image large but WINO_AUTO does not resolve to the fused F(4x4)
 * variant - e.g. 64 channels at 256x256, or bf16 with 256 channels at 512x512 - and for at most four output channels
 * on images of 512x512 pixels and more, which have a kernel of their own there); -1 on bad arguments.
 * wino_resolve_variant(WINO_AUTO) keeps to the Winograd variants. */
int wino_recommend_variant(int N, int C, int H, int W, int K, int dtype);

/* Sizes (elements, not bytes) of the transformed tensors for a resolved variant:
 * *Cp = C rounded up to a multiple of 8 (zero-filled), *T = N*ceil(H/m)*ceil(W/m).
 * Returns WINO_OK or an error; outputs may be NULL. */
int wino_transformed_dims(int N, int C, int H, int W, int K, int variant, int *alpha, int *Cp, int *T);

/* Bytes of the device buffer that holds U (WINO_DIRECT: the re-laid filter).  0 on bad arguments / AUTO. */
size_t wino_filter_bytes(int K, int C, int dtype, int variant);

/* Bytes of scratch (V then M, each 256-byte aligned; WINO_DIRECT: the re-laid copy of x and any
 * partial sums) that wino_conv2d_ex needs for a resolved variant; 0 on bad arguments. */
size_t wino_workspace_bytes(int N, int C, int H, int W, int K, int dtype, int variant);

/*
 * Step (i), filter:  U[xi,nu,k,c] = (G g[k,c] G^T)[xi,nu], computed in fp32 and
 * rounded once to `dtype`.  Done once per weight tensor.
 *   w         device, [K][C][3][3] in `dtype`
 *   w_t_data  device, at least wino_filter_bytes(K,C,dtype,variant) bytes
 *   variant   WINO_F2, WINO_F4, WINO_FUSED_F2, WINO_FUSED_F4 (the fused variants share U with their tile size; WINO_FUSED_F4 with
 *             fp32 is WINO_ERR_DTYPE) or WINO_DIRECT; WINO_AUTO is rejected: the shape is not known here
 *   out       host, filled on success
 */
int wino_filter_transform(const void *w, void *w_t_data, int K, int C, int dtype, int variant,
                          wino_filter *out, void *stream);

/*
 * The whole path (steps (i) activation, (ii), (iii) + bias) with the variant held
 * in w_t.  x[N][C][H][W] and y[N][K][H][W] (NCHW) in w_t->dtype; y is fully overwritten.
 * Borrows wino_workspace_bytes() of scratch from hipMallocAsync on `stream` and
 * returns it with hipFreeAsync on `stream`.
 */
int wino_conv2d(const void *x, const wino_filter *w_t, const float *bias, void *y,
                int N, int C, int H, int W, int K, void *stream);

/* Same, scratch supplied by the caller; allocates nothing.  `layout` is a wino_layout
 * and applies to both x and y. */
int wino_conv2d_ex(const void *x, const wino_filter *w_t, const float *bias, void *y,
                   int N, int C, int H, int W, int K, int layout,
                   void *workspace, size_t workspace_bytes, void *stream);

/*
 * wino_conv2d_ex for callers that cannot allocate and have no workspace to hand over: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  The scratch (V and M; for a
 * WINO_DIRECT filter the re-laid x and partial sums) lives in a device array inside the library,
 * wino_static_scratch_bytes() = 64 MiB per GPU, held from the time the library is loaded until the
 * process ends.  The call allocates nothing and frees nothing; its first call on a device looks up
 * that device's copy of the array (no allocation either).  Same kernels, same results as
 * wino_conv2d_ex, bit for bit.  Problems whose wino_workspace_bytes() exceed the array are refused
 * with WINO_ERR_SCRATCH and nothing is launched (layer sizes up to about N=2, C=K=320, 64x64 in
 * fp16 fit).  All calls on one GPU share the one array: calls that may overlap in time (different
 * streams, different threads) race on it, so serialise them on one stream.
 */
size_t wino_static_scratch_bytes(void);
int wino_conv2d_static(const void *x, const wino_filter *w_t, const float *bias, void *y,
                       int N, int C, int H, int W, int K, int layout, void *stream);

/*
 * The three stages on their own (the same kernels wino_conv2d_ex chains), for
 * stage-by-stage checks and per-kernel measurement.  Layouts, `e` = dtype:
 *   V[alpha^2][T][Cp]  e     step (i), activation: V[xi,nu,t,c] = (B^T d[c,t] B)[xi,nu],
 *                            d = alpha x alpha window of xhat at rows m*ti-1.., cols m*tj-1..;
 *                            entries with c >= C are written as zero
 *   U[alpha^2][K][Cp]  e     as produced by wino_filter_transform
 *   M[alpha^2][K][T]   fp32  step (ii): M[xi,nu,k,t] = sum_c U[xi,nu,k,c] * V[xi,nu,t,c]
 *   y[N][K][H][W]      e     step (iii): y tile = A^T M[.,.,k,t] A (+ bias[k]), cropped to HxW
 * Channel-last (WINO_NHWC): the product is kept transposed, M[alpha^2][T][K], so that the channel
 * index stays contiguous from x to y.  wino_batched_gemm is symmetric in its two operands: called
 * as (V, U, M, T, C, K) it writes exactly that tensor, and wino_output_transform with
 * layout = WINO_NHWC reads it (and only it).  wino_conv2d_ex does the same internally.
 */
int wino_input_transform(const void *x, void *V, int N, int C, int H, int W,
                         int dtype, int variant, int layout, void *stream);
int wino_batched_gemm(const void *U, const void *V, float *M, int K, int C, int T,
                      int dtype, int variant, void *stream);
int wino_output_transform(const float *M, const float *bias, void *y, int N, int K, int H, int W,
                          int dtype, int variant, int layout, void *stream);

/*
 * Steps (ii) and (iii) + bias in one kernel, the second launch of WINO_FUSED_F2 (F(2x2,3x3) only):
 *   U[16][K][Cp], V[16][T][Cp] as above  ->  y[N][K][H][W] (WINO_NCHW) or y[N][H][W][K] (WINO_NHWC) in `dtype`.
 * block_shape = -1 lets the library choose the workgroup's block; 0..6 name one (rows x columns of the
 * block, rows = output channels for NCHW and tiles for NHWC): 0 = 64x64, 1 = 64x128, 2 = 128x64,
 * 3 = 128x128 with four waves, 4 = 128x128, 5 = 128x64, 6 = 64x128 with eight waves.  The shapes differ
 * only in which fp32 partial sums are added first (results agree to fp32 rounding); the argument exists so
 * that tests and measurements can reach each kernel instantiation on small inputs.  WINO_ERR_VARIANT for
 * other values.  Reduction lengths that are not a multiple of 64 (fp32: 32) always run the 64x64 block.
 */
int wino_fused_gemm_output(const void *U, const void *V, const float *bias, void *y,
                           int N, int C, int H, int W, int K, int dtype, int layout, int block_shape, void *stream);

/* The same for F(4x4,3x3), the second launch of WINO_FUSED_F4: U[36][K][Cp], V[36][T][Cp] -> y, two-byte `dtype` only.
 * block_shape: -1 = the library's choice, 0 = 64x64 (eight waves), 1 = 32x64 (four waves); reduction lengths that are
 * not a multiple of 64 always run the 32x64 block. */
int wino_fused_f4_gemm_output(const void *U, const void *V, const float *bias, void *y,
                              int N, int C, int H, int W, int K, int dtype, int layout, int block_shape, void *stream);

/*
 * wino_batched_gemm with a named block shape instead of the library's choice, so that every instantiation
 * of the step (ii) kernel can be reached on small, ragged inputs (tests, measurements):
 *   0 = 128x128, 1 = 128x64, 2 = 64x128, 3 = 64x64 (4 waves, 2 ring slots), 4 = 256x256 (16 waves),
 *   5 = 128x32, 6 = 32x128 (3 slots), 7 = 128x128 with 3 slots, 8 = 256x128 (8 waves, 3 slots);
 * rows x columns = rows of the first operand x rows of the second.  WINO_ERR_VARIANT outside 0..8.
 */
int wino_batched_gemm_shape(const void *U, const void *V, float *M, int K, int C, int T,
                            int dtype, int variant, int block_shape, void *stream);

/*
 * The operators on either side of the convolution inside a residual block, fused into the
 * transforms so that the activation is not rewritten to memory in between (the paper's Section
 * "Techniques" argues for keeping dependent steps local; it names none of these operators, the
 * textbook definitions apply):
 *   on the way in   x' = SiLU(GroupNorm(x)), GroupNorm over gn_groups equal channel groups per image
 *                   with affine gamma/beta; zero padding applies to x'.  Active iff gn_stats != NULL.
 *   upsample != 0   the convolution reads x' through a 2x nearest-neighbour upsampling (the step before
 *                   the 3x3 convolution in the UNet's and the VAE decoder's up-sampling blocks): x holds
 *                   [H/2][W/2] pixels per channel, H and W (the arguments of the call, the size of y)
 *                   must be even, and GroupNorm statistics, if used, are those of the stored x.
 *   on the way out  y = conv(x') + bias + addvec[n][k] + residual.  Each part optional.
 *   product_fp16    opt-in, fp16 storage only: the product M of step (ii) is written and read back as fp16
 *                   instead of fp32, which halves the largest tensor of the path (1.2-1.4x on layers with
 *                   large images).  Accumulation stays fp32.  The relative L2 error of F(4x4) grows from
 *                   about 3.1e-3 to 3.8-4.2e-3 (F(2x2): 5e-4 to 6.4e-4), and |M| must stay below 65504.
 *                   Ignored where the reduction is split into partial products, for fp32 storage, and by
 *                   the fused variants (which have no stored product).
 * A filter prepared with WINO_DIRECT is accepted too: the direct path reads x through the upsampling by address
 * arithmetic, adds in its epilogue, and applies GroupNorm + SiLU while it re-lays x into its workspace (the activated
 * tensor is rounded once to the storage type there; a channel-last x is then copied once instead of read in place).
 * All pointers are device memory.  residual has the layout, dtype and shape of y and may be y
 * itself (in-place accumulate) but must not otherwise overlap it.
 */
typedef struct wino_fusion {
    const float *gn_stats;   /* [N][gn_groups][2] = (mean, 1/sqrt(var+eps)), from wino_groupnorm_stats */
    const float *gn_gamma;   /* fp32 [C] */
    const float *gn_beta;    /* fp32 [C] */
    int gn_groups;           /* must divide C */
    const float *addvec;     /* fp32 [N][K], or NULL */
    const void *residual;    /* like y, or NULL */
    int upsample;            /* 0, or 1 = read x through a 2x nearest-neighbour upsampling */
    int product_fp16;        /* 0, or 1 = keep the intermediate product M in fp16 (see below) */
} wino_fusion;

/* Bytes of the buffer wino_groupnorm_stats writes (statistics first, then its partial sums);
 * 0 on bad arguments. */
size_t wino_groupnorm_stats_bytes(int N, int groups);

/* Statistics of x (NCHW or NHWC, `dtype`) for the fused GroupNorm: mean and 1/sqrt(biased
 * variance + eps) per (image, group), fp32, at the start of `stats` (16-byte aligned, at least
 * wino_groupnorm_stats_bytes(N, groups)).  Deterministic. */
int wino_groupnorm_stats(const void *x, float *stats, int N, int C, int H, int W, int groups, float eps,
                         int dtype, int layout, void *stream);

/* wino_conv2d_ex with the fused operators of `f` (host struct, read during the call). */
int wino_conv2d_fused(const void *x, const wino_filter *w_t, const float *bias, void *y,
                      int N, int C, int H, int W, int K, int layout, const wino_fusion *f,
                      void *workspace, size_t workspace_bytes, void *stream);

/* Direct correlation on the GPU from the untransformed filter (fp32 accumulate),
 * one thread per output; a checking fallback, not a fast path. */
int wino_direct_conv2d(const void *x, const void *w, const float *bias, void *y,
                       int N, int C, int H, int W, int K, int dtype, void *stream);

/*
 * The convolution flavours of a Stable-Diffusion UNet / VAE that the Winograd path does not cover
 * (1x1 projections, 3x3 with stride 2), as an implicit GEMM on the MFMA units with fp32 accumulation,
 * so that the library can stand in for the whole 2-D convolution operator that the paper's Section
 * "Techniques" replaces (the paper defines none of these flavours; the textbook definition applies):
 *
 *     y[n,k,i,j] = bias[k] + sum_{c,r,s} xhat[n,c,i*stride+r-pad,j*stride+s-pad] * w[k,c,r,s]
 *     R x R filter with R in {1, 3}, stride in {1, 2}, pad = (R-1)/2, Ho = (H+2*pad-R)/stride+1, Wo likewise
 *
 * The filter is re-laid once per weight tensor (wino_igemm_filter_repack: w[K][C][R][R] ->
 * Wr[R*R][K][Cp] plus one row of zeros, wino_igemm_filter_bytes() bytes).  x[N][C][H][W] -> y[N][K][Ho][Wo]
 * (WINO_NCHW) or x[N][H][W][C] -> y[N][Ho][Wo][K] (WINO_NHWC), all in `dtype`; bias fp32 [K] or NULL.
 * The workspace (wino_igemm_workspace_bytes(), may be 0: channel-last x with C a multiple of 8 is read
 * in place) holds x re-laid with the channel index contiguous and, for shapes with few output pixels and
 * a long reduction, fp32 partial sums of a reduction that is cut into ranges.  Same conventions as above: device
 * pointers 16-byte aligned, arguments validated on the host, work enqueued on `stream`, deterministic.
 * One shape class takes a kernel of its own behind the same call, with the same result up to summation order: 3x3 / stride 1
 * with K <= 4 output channels in fp16 on images of at least 512 tiles of 8 x 64 pixels (one pass over x on the vector ALU, no
 * re-layout, no workspace use; C a multiple of 16, and W a multiple of 8 for WINO_NCHW - otherwise the general kernels run).
 */
size_t wino_igemm_filter_bytes(int K, int C, int R, int dtype);
int wino_igemm_filter_repack(const void *w, void *w_r, int K, int C, int R, int dtype, void *stream);
size_t wino_igemm_workspace_bytes(int N, int C, int H, int W, int K, int R, int stride, int dtype, int layout);
int wino_igemm_conv2d(const void *x, const void *w_r, const float *bias, void *y,
                      int N, int C, int H, int W, int K, int R, int stride, int dtype, int layout,
                      void *workspace, size_t workspace_bytes, void *stream);

/*
 * The same direct convolution with 8-bit floating-point operands (OCP E4M3: 4 exponent and 3 mantissa bits, largest
 * value 448), fp32 accumulation on the 8-bit MFMA path of the chip.  The paper only remarks that its stack supports
 * quantised operators and defines no scheme; this one is the plainest: one power-of-two scale per tensor,
 *
 *     xq = e4m3(clamp(x' * scale_x, +-448)),  wq = e4m3(clamp(w * scale_w, +-448)),
 *     y  = conv(xq, wq) / (scale_x * scale_w) + bias (+ addvec + residual),        x' = x or SiLU(GroupNorm(x))
 *
 * with scales chosen by the caller (largest power of two that keeps max|.| * scale <= 448; activations after
 * GroupNorm + SiLU are bounded, which makes a fixed scale safe).  Relative L2 error against the exact convolution on
 * unit-variance data: about 3.8e-2 (tolerance of this path: 6e-2).  x and y are in `dtype` (any of the three storage
 * types), NCHW or NHWC; R in {1, 3}, stride in {1, 2}.  The filter is quantised once (wino_fp8_filter_quantize, re-laid
 * as for the implicit-GEMM path, wino_fp8_filter_bytes() bytes); the workspace (wino_fp8_workspace_bytes()) holds xq and
 * any partial sums.  `f` may be NULL; its fused operators work as with a WINO_DIRECT filter (product_fp16 is ignored).
 */
size_t wino_fp8_filter_bytes(int K, int C, int R);
int wino_fp8_filter_quantize(const void *w, void *w_q, int K, int C, int R, int dtype, float scale_w, void *stream);
size_t wino_fp8_workspace_bytes(int N, int C, int H, int W, int K, int R, int stride);
int wino_fp8_conv2d(const void *x, const void *w_q, const float *bias, void *y,
                    int N, int C, int H, int W, int K, int R, int stride, int dtype, int layout,
                    float scale_x, float scale_w, const wino_fusion *f,
                    void *workspace, size_t workspace_bytes, void *stream);

/*
 * The Winograd path with 8-bit integer transformed tensors: F(2x2,3x3), U and V held as symmetric integer codes with one
 * quantisation step per row of each of the 16 matrix products of step (ii), exact int32 accumulation on the chip's 8-bit
 * integer MFMA path.  The paper's Section "Techniques" only remarks that its stack supports quantised operators; the scheme
 * is this library's, chosen by a CPU error model first (F(4x4) and 8-bit floating point amplify the rounding too much):
 *
 *     U = G g G^T,  V = (B^T d) B                            b = xi*4 + nu, the position inside the transformed tile
 *     mU[b][k] = max_c |U[b][k][c]|,  Uq = rint(U * (127 / mU)),  dU = mU / 127      (codes -127..127, ties to even;
 *     mV[b][t] = max_c |V[b][t][c]|,  Vq = rint(V * (127 / mV)),  dV = mV / 127       a zero row has codes 0 and step 0)
 *     M[b][k][t] = float(sum_c Uq[b][k][c] * Vq[b][t][c]) * dU[b][k] * dV[b][t],     y = A^T M A + bias
 *
 * The filter side is decided in fp64 (U is exact there) once per weight tensor; the activation side in fp32 on every call,
 * row combination B^T d first, so that every entry is one IEEE operation and the codes are reproducible bit for bit.  The
 * steps follow the data (no calibration, no scale arguments).  Halves the bytes of U and V: meant for the layers whose
 * step (ii) streams a large U against few tiles (8x8 and 16x16 images with 640-2560 channels).  Relative L2 error against
 * the exact convolution on unit-variance data: 1.4e-2 ... 2.0e-2 (tolerance of this path: 3e-2) - an opt-in, never chosen
 * by WINO_AUTO.  x and y are in `dtype` (any storage type), NCHW or NHWC; C <= 65536.
 *   u_q        device, wino_i8_filter_bytes(K, C): Uq[16][K][Cq] int8 (Cq = C rounded up to 16, padding zero), then,
 *              256-byte aligned, dU[16][K] fp32
 *   workspace  device, wino_i8_workspace_bytes(): Vq[16][T][Cq], dV[16][T], M (each 256-byte aligned), T = N*ceil(H/2)*ceil(W/2)
 * wino_i8_input_transform and wino_i8_batched_gemm are the first two stages on their own (the third is
 * wino_output_transform with WINO_F2); block_shape as for wino_batched_gemm_shape, -1 = the library's choice.
 */
size_t wino_i8_filter_bytes(int K, int C);
int wino_i8_filter_transform(const void *w, void *u_q, int K, int C, int dtype, void *stream);
size_t wino_i8_workspace_bytes(int N, int C, int H, int W, int K);
int wino_i8_conv2d(const void *x, const void *u_q, const float *bias, void *y,
                   int N, int C, int H, int W, int K, int dtype, int layout,
                   void *workspace, size_t workspace_bytes, void *stream);
int wino_i8_input_transform(const void *x, void *Vq, float *dV, int N, int C, int H, int W,
                            int dtype, int layout, void *stream);
int wino_i8_batched_gemm(const void *Uq, const float *dU, const void *Vq, const float *dV, float *M,
                         int K, int C, int T, int block_shape, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* WINO_H */
