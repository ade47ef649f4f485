/*
 * iconv_bench.h - test and measurement entry points of libiconv_mi355.so.
 *
 * None of these belong to the convolution contract of iconv.h; they exist so that tests can
 * reach every kernel of the table and so that the benchmark can price the kernels against what
 * the device sustains.  All of them are functions of their arguments alone (no process-wide
 * switch is left behind by any call), all pointers are DEVICE pointers owned by the caller and
 * 16-byte aligned, nothing is allocated or synchronised, errors are ICONV_* return codes.
 */
#ifndef ICONV_BENCH_H
#define ICONV_BENCH_H

#include <stddef.h>

#include "iconv.h"

#ifdef __cplusplus
extern "C" {
#endif

/* iconv_fwd with the kernel choice and the launch width in the caller's hands, for this call only.
 *   variant        -1 = the library's own choice (what iconv_fwd does); otherwise an index into the
 *                  kernel table (iconv_num_variants entries, names from iconv_variant_name).  An
 *                  entry that cannot run the layer (shape limits of the patch-reuse and
 *                  resident-filter kernels, C % 8 != 0, fp32 input) falls back to the library's
 *                  choice, so the result is always the convolution.
 *   max_workgroups 0 = fill the device; n > 0 caps the workgroups of the persistent kernels at n,
 *                  so that each walks through more output tiles (tests of the tile-to-tile
 *                  hand-over); kernels with one workgroup per tile ignore it.
 * Returns ICONV_ERR_UNSUPPORTED for variant < -1, variant >= iconv_num_variants() or
 * max_workgroups < 0; otherwise as iconv_fwd. */
int iconv_fwd_ex(const void *x_nhwc, const void *w_krsc, void *y_npqk,
                 int N, int H, int W, int C, int K, int R, int S,
                 int stride, int pad, int dilation, int dtype,
                 int variant, int max_workgroups, void *stream);

/* The kernel table: the MFMA paths (block-level channel-first im2col, paper section 5, in its
 * per-tap, patch-reuse, resident-filter and pixel-resident forms) for channel counts that are
 * multiples of eight, then the forms of the merged-tap kernel for four-channel layers (paper
 * section 4.3).  iconv_variant_name returns "auto" outside 0 .. iconv_num_variants() - 1. */
int iconv_num_variants(void);
const char *iconv_variant_name(int variant);

/* Whether kernel-table entry `variant` can run the layer itself (1), or iconv_fwd_ex would fall
 * back to the library's choice for it (0: the entry's shape limits, C % 8 != 0, fp32 input,
 * invalid arguments, no such entry).  Host logic only. */
int iconv_variant_accepts(int variant, int N, int H, int W, int C, int K, int R, int S,
                          int stride, int pad, int dilation, int dtype);

/* A plain device-to-device copy kernel of `bytes` bytes (a multiple of 16), used to calibrate
 * memory-traffic counters and to measure the achievable copy bandwidth. */
int iconv_probe_copy(void *dst, const void *src, size_t bytes, void *stream);

/* The same copy with the store instructions of the convolution kernels' epilogues (whole 128-byte lines per
 * instruction, written through at system scope): the achievable read + write bandwidth for data that is
 * written once.  bytes < 2^32 (ICONV_ERR_UNSUPPORTED otherwise); other errors as iconv_probe_copy. */
int iconv_probe_copy_wt(void *dst, const void *src, size_t bytes, void *stream);

/* A register-only loop of `iters` x 8 bf16 32x32x16 MFMAs per wave on 1024 workgroups of four
 * waves (no memory traffic in the loop), for the achievable matrix-core rate:
 * 1024 * 4 * iters * 8 * 32768 flop per launch.  random_operands = 0 multiplies one fixed pair of
 * small-integer operands (few bits toggle, the highest clock the chip sustains);
 * random_operands != 0 alternates four pairs of pseudo-random operands, the rate the matrix cores
 * sustain on real data under the board's power limit.  `out` is a device buffer of at least
 * 1024 * 256 * 4 bytes that receives one float per thread (so that the loop is not optimised
 * away).  Returns ICONV_ERR_NULL, ICONV_ERR_SHAPE (iters < 1), ICONV_ERR_WORKSPACE (out too small). */
int iconv_probe_mfma(void *out, size_t out_bytes, int iters, int random_operands, void *stream);

/* A loop of `iters` x 8 LDS instructions per wave with one fixed 64-lane address pattern and nothing else, on
 * the MFMA probe's grid (1024 workgroups of four waves, i.e. 128 * iters instructions per compute unit on 256
 * compute units): what an LDS instruction costs, and what the bank-conflict counter reads for it.
 *   pattern 0  ds_read_b128, lane l at byte 16 * l (conflict-free reference)
 *   pattern 1  ds_write_b128, lane l at byte 16 * l
 *   pattern 2  ds_read_b128 of the MFMA operand shape (lane l: tile row l % 32, 16-byte chunk l / 32) on
 *              64-byte tile rows without a swizzle
 *   pattern 3  the same through the kernels' swizzle of 64-byte rows
 *   pattern 4  the same on 128-byte rows through the kernels' swizzle of 128-byte rows
 *   pattern 5  ds_write_b128, the deposit of the kernels' output staging: 32 of the 64 lanes (16 pixels x 2
 *              pieces) write 16-byte piece c of pixel i at iconv_lds_stage_offset(i, c)
 *   pattern 6  the same with all 64 lanes (32 pixels), the deposit of the merged-tap kernel
 *   pattern 7  as pattern 6 with piece c of pixel i at i * 128 + ((c ^ (i >> 1 & 7)) << 4): conflict-free as a
 *              read, two lanes per bank in every pass as a write (reference for the counter)
 * `out` as for iconv_probe_mfma.  Returns ICONV_ERR_UNSUPPORTED for another pattern, otherwise as
 * iconv_probe_mfma. */
int iconv_probe_lds(void *out, size_t out_bytes, int iters, int pattern, void *stream);

/* The chunk position the MFMA kernels give 16-byte chunk `chunk` of tile row `row` in LDS rows of
 * `chunks_per_row` (4, 8, 16 or 32) chunks - the very function the kernels compile, evaluated on the host, so that
 * the layout can be checked against the bank model without a GPU.  Returns -1 for other arguments. */
int iconv_lds_swizzle(int chunks_per_row, int row, int chunk);

/* Byte offset of 16-byte piece `piece` (0..7) of pixel `pixel` in the kernels' output staging areas, again the
 * function the kernels compile.  Returns -1 for a piece outside 0..7 or a negative pixel. */
int iconv_lds_stage_offset(int pixel, int piece);

#ifdef __cplusplus
}
#endif
#endif /* ICONV_BENCH_H */
