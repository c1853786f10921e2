/*
 * hipattn_aux - test and measurement aids that ship beside the HiP attention library (libhipattn_aux.so).
 *
 * Nothing here is part of the method or of the product ABI (include/hipattn.h): the GPU tests use the LDS
 * poisoner, the benchmark uses the probes to quote what this GPU sustains next to the published peaks.
 * Every pointer is a DEVICE pointer owned by the caller; a call enqueues one kernel on `stream` (a
 * hipStream_t passed as void*, NULL = the default stream) and returns 0, a negative argument error
 * (-1 NULL pointer, -2 bad size, -7 alignment) or -1000 - hipError_t for a failed launch.  The caller
 * times the kernels with events on `stream`.
 */
#ifndef HIPATTN_AUX_H
#define HIPATTN_AUX_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Fills the LDS of every compute unit with `pattern`, so that a kernel that wrongly reads LDS it never
 * wrote sees that value instead of whatever an earlier kernel left there. */
int hip_attn_poison_lds(uint32_t pattern, void *stream);

/* Copies `bytes` (a multiple of 16) from `src` to `dst` (both 16-byte aligned, not overlapping):
 * HBM traffic = 2 * bytes. */
int hip_attn_probe_copy(void *dst, const void *src, size_t bytes, void *stream);

/* Reads `bytes` (a multiple of 16) from `src` (16-byte aligned) and writes the XOR of the words each lane
 * saw to `out` [HIP_ATTN_PROBE_READ_WORDS uint32]: HBM traffic = bytes (+ 8 MiB written). */
#define HIP_ATTN_PROBE_READ_WORDS (256 * 32 * 256)
int hip_attn_probe_read(uint32_t *out, const void *src, size_t bytes, void *stream);

/* `workgroups` workgroups of 4 waves; every wave issues iters * 4 independent 32x32x16 bf16 matrix
 * instructions (2*32*32*16 flop each) on register operands and writes one float per lane to
 * `out` [workgroups * 256]. */
int hip_attn_probe_mfma(float *out, int32_t workgroups, int32_t iters, void *stream);

/* The gather pattern of the attention kernels without their arithmetic.  `src` (16-byte aligned, `bytes`
 * long) is taken as `slices` equal slices of 256-byte rows; workgroup w (4 waves) works on slice
 * w % slices; every wave reads `tiles` (a multiple of 4) tiles of 32 rows, each tile being 32 / run_rows
 * runs of `run_rows` (a power of two up to 32) consecutive rows at pseudo-random places of the slice, with
 * 16 lanes per row and four tiles in flight, and writes one word per lane to `out` [workgroups * 256].
 * Bytes gathered = workgroups * 4 * tiles * 8192. */
int hip_attn_probe_gather(uint32_t *out, const void *src, size_t bytes, int32_t slices, int32_t run_rows,
                          int32_t workgroups, int32_t tiles, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* HIPATTN_AUX_H */
