/*
 * w4a8_measure.h -- bench aids of libw4a8.so: the measured ceilings of the machine that the
 * benchmark prints beside the nominal peaks.  No function here is a step of the method, and none
 * belongs to the product ABI of w4a8.h (whose conventions -- status codes, `stream`, no allocation,
 * no synchronization -- they share).
 */
#ifndef W4A8_MEASURE_H
#define W4A8_MEASURE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* w4a8_measure_stream_read reads `bytes` bytes of device memory once (16-byte loads, 512 x 512 lanes,
 * four loads in flight per lane) and writes nothing; w4a8_measure_mfma_i8 runs `iters` rounds of eight
 * independent v_mfma_i32_32x32x32_i8 per wave on register operands (512 workgroups of four waves) and
 * stores the number of integer operations issued (2 per multiply-accumulate) to *ops.
 *   buf: DEVICE pointer, 16-byte aligned, bytes % 16 == 0; sink: DEVICE uint32 or NULL (never written in
 *   practice: it only keeps the work alive); ops: HOST pointer or NULL, written by the call itself
 *   before it returns; iters <= 2^24.
 * w4a8_measure_ktile_mix runs `iters` rounds of the instruction mix of one k-tile of the group-wise tile
 * kernel per wave (16 such MFMAs in four chains, six independent vector instructions behind each, then one
 * convert and one multiply-add per accumulator register; 512 workgroups of four waves); fragment_reads != 0:
 * each MFMA's second operand is read from LDS first (one 16-byte-per-lane read per MFMA, conflict free), as
 * in the kernel; 0: it stays in a register.  iters <= 2^24.
 * All three only enqueue work on `stream`; the caller times them. */
int w4a8_measure_stream_read(const void *buf, int64_t bytes, uint32_t *sink, void *stream);
int w4a8_measure_mfma_i8(int64_t iters, uint32_t *sink, int64_t *ops, void *stream);
int w4a8_measure_ktile_mix(int64_t iters, int fragment_reads, uint32_t *sink, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* W4A8_MEASURE_H */
