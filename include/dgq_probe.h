/*
 * dgq_probe.h -- machine ceilings measured by the benchmark beside the datasheet peaks.
 *
 * These calls are not part of the method: they run the bare instruction the contraction is
 * built on and plain streaming kernels, so that a reported throughput can be set against what
 * the very box it was measured on delivers (sustained clocks under matrix load are well below
 * the clock the published peaks are quoted at).  Each call only enqueues one kernel on
 * `stream` (a hipStream_t as void*); the caller times it.  Return: DGQ_OK or a negative
 * dgq_status (dgq.h).
 */
#ifndef DGQ_PROBE_H
#define DGQ_PROBE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * A loop of nothing but v_mfma_i32_32x32x32_i8 (the int8 x int8 -> int32 matrix instruction of
 * dgq_linear) on constant operands: `blocks` workgroups of 4 wavefronts, every wavefront runs
 * `iters` rounds of 4 independent accumulator chains.  Integer operations issued:
 *   blocks * 4 * iters * 4 * 2 * 32 * 32 * 32.
 * sink: device int32 [blocks * 256], receives one accumulator register per lane (keeps the
 * loop alive; its value is 32 * iters for the operands used).
 */
int dgq_probe_mfma_i8(int32_t blocks, int32_t iters, int32_t *sink, void *stream);

/*
 * Streaming kernels over `bytes` (a multiple of 16 KiB) with 16-byte accesses:
 *   mode 0  read:  src is read once; sink (device uint32 [1]) receives a checksum nobody needs
 *   mode 1  write: dst is filled with a constant, every workgroup one contiguous 16 KiB piece
 *   mode 2  copy:  dst = src
 * src, dst: device, 16-byte aligned; unused ones may be NULL.
 */
int dgq_probe_stream(const void *src, void *dst, size_t bytes, int32_t mode, uint32_t *sink,
                     void *stream);

/*
 * The store pattern of dgq_linear's epilogue with nothing before it: dst fp32 [rows,
 * out_channels] (both multiples of 128) is written in 128 x 128 tiles by workgroups of 8
 * wavefronts, one dword per lane and instruction (two 128-byte row pieces), non-temporal.
 * What this reaches is the ceiling of a layer whose time is its fp32 output.
 */
int dgq_probe_write_tiles(float *dst, int64_t rows, int32_t out_channels, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* DGQ_PROBE_H */
