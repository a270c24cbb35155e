/*
 * shiftattn_probe.h - measurement aids exported by libshiftattn.so for benchmark reports.
 *
 * Not part of the attention path and not part of the product interface (shiftattn.h): four kernels
 * that show what the chip attains on the resources the path's kernels are priced against, to print
 * beside the datasheet peaks.  Each call validates its arguments, enqueues one kernel on `stream`
 * (a hipStream_t as void*) and returns SHIFTATTN_OK or a negative code of shiftattn.h; the caller
 * times it.  All buffer pointers are device pointers, 16-byte aligned.
 *
 * ceiling_mfma_bf16: every wavefront of a chip-filling grid issues iters x 32 independent
 *   16x16x32 bf16 MFMAs (the form that sustains the higher rate at the chip's power limit) on the
 *   operand values found in `operands` (2 KiB = 128 lanes x 8 bf16; random values give the clock
 *   real data gives).  *flops (host) receives the flops of the launch.  sink: 4 bytes, never
 *   written in practice.
 * ceiling_mfma_bf16_fresh: the same loop (iters x 64 MFMAs per wavefront) with operands that differ
 *   from one MFMA to the next, as in a product of real matrices: `operands` holds eight A and eight
 *   B fragments per lane (16 KiB = 16 x 64 lanes x 8 bf16), MFMA m takes A fragment m % 8 and B
 *   fragment (m / 8) % 8.  Inputs that toggle cost power, which the chip gives up in clock: the
 *   rate a GEMM-shaped kernel can be held against.
 * ceiling_hbm_read: streams `bytes` (rounded down to 16 KiB) of `src` through every wavefront
 *   with 16-byte non-temporal loads.  *bytes_read (host) receives the bytes requested.
 * ceiling_hbm_copy: copies `bytes` (rounded down to 16 KiB) from src to dst with 16-byte
 *   non-temporal loads and stores, 16 KiB in flight per wavefront: a read + write stream with no
 *   index arithmetic.  *bytes_copied (host) receives the bytes copied (as many are read as written).
 */
#ifndef SHIFTATTN_PROBE_H
#define SHIFTATTN_PROBE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

int shiftattn_ceiling_mfma_bf16(const void *operands, void *sink, int32_t iters, int64_t *flops, void *stream);
int shiftattn_ceiling_mfma_bf16_fresh(const void *operands, void *sink, int32_t iters, int64_t *flops, void *stream);
int shiftattn_ceiling_hbm_read(const void *src, size_t bytes, void *sink, int64_t *bytes_read, void *stream);
int shiftattn_ceiling_hbm_copy(const void *src, void *dst, size_t bytes, int64_t *bytes_copied, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* SHIFTATTN_PROBE_H */
