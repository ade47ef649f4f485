/*
 * iconv.h - C ABI of the implicit-im2col convolution library for AMD MI355X (gfx950).
 *
 * The operation is the 2-D convolution layer of the paper's section 2.1 (C_I input maps of
 * H_I x W_I, a sliding H_F x W_F kernel, C_O output maps, batch N), evaluated as the GEMM
 * that im2col lowering defines there (M = N*P*Q output pixels, N_gemm = K filters,
 * K_gemm = C*R*S taps) with the lowered dimension ordered tap-row, tap-column, channel
 * (channel fastest: the "channel-first" order of section 3.1) and formed on the fly inside
 * each output tile's K loop (block-level channel-first im2col, section 5), so the lowered
 * matrix never exists in device memory.
 *
 * Notation: N batch, H x W input map, C input channels, K filters, R x S filter, P x Q output
 * map (the paper's N, H_I x W_I, C_I, C_O, H_F x W_F, H_O x W_O).
 *
 *   y[n,p,q,k] = sum_{r,s,c} x[n, p*stride + r*dilation - pad, q*stride + s*dilation - pad, c]
 *                            * w[k,r,s,c]
 *
 * x is read as zero outside the map (symmetric zero padding), the filter is not flipped,
 *   P = floor((H + 2*pad - dilation*(R-1) - 1) / stride) + 1,   Q alike with W and S.
 *
 * Layouts (dense, no strides):  x[((n*H+h)*W+w)*C+c]   (NHWC)
 *                               w[((k*R+r)*S+s)*C+c]   (KRSC)
 *                               y[((n*P+p)*Q+q)*K+k]   (NPQK, i.e. row-major M x K)
 *
 * Ownership and execution: every tensor pointer is a DEVICE pointer owned by the caller and
 * must be 16-byte aligned.  x and w are only read; y is overwritten in full (no accumulate, no
 * bias, one group).  The library allocates nothing, frees nothing and never synchronises: the
 * kernels are enqueued on `stream` (a hipStream_t passed as void*, NULL = the default stream)
 * and the results are valid once the caller has synchronised that stream.  Calls are
 * thread-safe: every entry point is a function of its arguments alone, and the library keeps
 * no mutable state beyond one-time, idempotent caches of device properties (number of compute
 * units, LDS limits raised once per kernel).  Measurement helpers and the per-call kernel
 * override used by tests and sweeps live in iconv_bench.h, not here.
 *
 * Errors are reported by the return value only (never abort, never throw):
 */
#ifndef ICONV_H
#define ICONV_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ICONV_OK                 0
#define ICONV_ERR_NULL          -1  /* a required pointer is NULL                               */
#define ICONV_ERR_SHAPE         -2  /* a dimension <= 0, stride < 1, dilation < 1, pad < 0,
                                       or an empty output (P < 1 or Q < 1)                      */
#define ICONV_ERR_UNSUPPORTED   -3  /* unknown dtype/algo, or a tensor of 2^31 elements or more */
#define ICONV_ERR_ALIGN         -4  /* a tensor pointer is not 16-byte aligned                  */
#define ICONV_ERR_WORKSPACE     -5  /* explicit variant only: workspace missing or too small    */
#define ICONV_ERR_LAUNCH        -6  /* the HIP runtime refused a launch                         */

/* dtype: element type of x and w / of y.  Products and sums are always fp32. */
#define ICONV_F32_F32    0  /* fp32 in, fp32 out (plain FMA path; correctness configuration)  */
#define ICONV_BF16_F32   1  /* bf16 in, fp32 out (MFMA; the measured path)                    */
#define ICONV_F16_F32    2  /* fp16 in, fp32 out (MFMA)                                       */
#define ICONV_BF16_BF16  3  /* bf16 in, bf16 out (fp32 accumulators rounded to nearest even)  */
#define ICONV_F16_F16    4  /* fp16 in, fp16 out                                              */

/* algo, for iconv_workspace_bytes */
#define ICONV_ALGO_IMPLICIT 0
#define ICONV_ALGO_EXPLICIT 1

/* Output map size for one spatial axis pair (formula above).  Host pointers P, Q.
 * Returns ICONV_OK, ICONV_ERR_NULL or ICONV_ERR_SHAPE. */
int iconv_out_shape(int H, int W, int R, int S, int stride, int pad, int dilation, int *P, int *Q);

/* Implicit channel-first im2col convolution (paper sections 3 and 5).  Needs no workspace.
 * Any C and K are accepted; C % 8 == 0 takes the MFMA path with 16-byte channel runs, C == 4
 * takes the merged-tap path for low-channel first layers (the multi-tile idea of section 4.3),
 * anything else (and ICONV_F32_F32) takes a plain direct kernel. */
int iconv_fwd(const void *x_nhwc, const void *w_krsc, void *y_npqk,
              int N, int H, int W, int C, int K, int R, int S,
              int stride, int pad, int dilation, int dtype, void *stream);

/* Device bytes the caller must provide as workspace.  ICONV_ALGO_IMPLICIT: always 0.
 * ICONV_ALGO_EXPLICIT: the lowered matrix of section 2.1, M x (R*S*C) input elements.  When
 * R*S*C is not a multiple of 8 and the inputs are 16-bit, the rows of the lowered matrix are
 * padded with zeros to the next multiple of 8 elements (the matrix cores read 16-byte runs),
 * the total is rounded up to 16 bytes, and a copy of the K x (R*S*C) filter matrix with rows
 * of the same padded length follows it: M*pitch*2 (rounded) + K*pitch*2 bytes.
 * Returns 0 also for invalid arguments. */
size_t iconv_workspace_bytes(int algo, int N, int H, int W, int C, int K, int R, int S,
                             int stride, int pad, int dilation, int dtype);

/* Channel-last implicit im2col (sections 2.3 and 3.1): the conventional design the paper's
 * channel-first method is compared with, built as a second in-run comparison for the stride
 * study.  Same operation and result contract as iconv_fwd (y in NPQK, fully overwritten, fp32
 * accumulation), but the lowered columns are ordered channel, tap row, tap column, so the
 * tensors arrive in the layouts that order reads contiguously:
 *   x_nchw[((n*C + c)*H + h)*W + w]     w_kcrs[((k*C + c)*R + r)*S + s]
 * dtype: the 16-bit input codes only (ICONV_BF16_F32, ICONV_F16_F32, ICONV_BF16_BF16,
 * ICONV_F16_F16); ICONV_F32_F32 returns ICONV_ERR_UNSUPPORTED.  No workspace; errors as iconv_fwd. */
int iconv_fwd_channel_last(const void *x_nchw, const void *w_kcrs, void *y_npqk,
                           int N, int H, int W, int C, int K, int R, int S,
                           int stride, int pad, int dilation, int dtype, void *stream);

/* Explicit im2col followed by a GEMM (section 2.2): the comparison the paper argues against.
 * Kernel 1 writes the lowered M x (R*S*C) matrix (columns in tap-row, tap-column, channel
 * order) into `workspace`; kernel 2 multiplies it with the filter matrix using the same MFMA
 * GEMM core (as a 1x1 convolution over the lowered matrix).  `workspace` is a device pointer,
 * 16-byte aligned, of at least iconv_workspace_bytes(ICONV_ALGO_EXPLICIT, ...) bytes; its
 * contents are overwritten.  Same result contract as iconv_fwd. */
int iconv_fwd_explicit(const void *x_nhwc, const void *w_krsc, void *y_npqk,
                       void *workspace, size_t workspace_bytes,
                       int N, int H, int W, int C, int K, int R, int S,
                       int stride, int pad, int dilation, int dtype, void *stream);

/* iconv_fwd_explicit for callers that cannot allocate device memory (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc) and therefore have no workspace
 * to pass: the lowered matrix goes into a buffer of ICONV_NOALLOC_WORKSPACE_BYTES that is part of
 * the library's device image (one per GPU, held until the process ends).  The call allocates and
 * frees nothing and runs the same two kernels as iconv_fwd_explicit, with the same result contract.
 * Layers whose lowered matrix, iconv_workspace_bytes(ICONV_ALGO_EXPLICIT, ...), exceeds that size
 * return ICONV_ERR_WORKSPACE and launch nothing.  Every call on a GPU uses that GPU's one buffer:
 * calls that overlap on the same GPU (two streams, two threads) race on it and must be ordered by
 * the caller; calls on different GPUs are independent.  The buffer's address is looked up on the
 * first call on each device (no allocation; make that first call outside a graph capture). */
#define ICONV_NOALLOC_WORKSPACE_BYTES (16u << 20)
int iconv_fwd_explicit_noalloc(const void *x_nhwc, const void *w_krsc, void *y_npqk,
                               int N, int H, int W, int C, int K, int R, int S,
                               int stride, int pad, int dilation, int dtype, void *stream);

/* Only the first half of the explicit variant (the lowering kernel), for timing it alone;
 * `workspace_bytes` must cover the lowered matrix (the padded rows, see above). */
int iconv_im2col(const void *x_nhwc, void *workspace, size_t workspace_bytes,
                 int N, int H, int W, int C, int R, int S,
                 int stride, int pad, int dilation, int dtype, void *stream);

/* Which kernel iconv_fwd runs for a layer: the name of a kernel-table entry (see
 * iconv_variant_name in iconv_bench.h), "stem" for the merged-tap kernel of 4-channel first layers (the
 * multi-tile idea of section 4.3) or "direct" for the plain kernel.  Host logic only: no device
 * work, no pointers; the choice depends on the tile counts of the block-level decomposition of
 * section 5 against the number of compute units (256 is assumed when no device is present).
 * Returns a static string, or NULL for arguments iconv_fwd would reject (shape, dtype, size). */
const char *iconv_kernel_for(int N, int H, int W, int C, int K, int R, int S,
                             int stride, int pad, int dilation, int dtype);

/* Static string for a status code. */
const char *iconv_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* ICONV_H */
