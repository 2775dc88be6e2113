/* C ABI of libarkv_measure.so: bandwidth measurement kernels that bench.py and the counter calibration use.
 * Not part of the method (nothing of the paper is computed here) and not part of libarkv.so. */
#ifndef ARKV_MEASURE_H
#define ARKV_MEASURE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ARKV_MEASURE_OK      0
#define ARKV_MEASURE_EINVAL -1   /* bad argument */
#define ARKV_MEASURE_EHIP   -4   /* a HIP runtime call failed */

/* A plain streaming read (16 bytes per lane, nothing else) of bytes_per_launch bytes
 * per kernel launch, `launches` launches back to back on the stream, walking through the DEVICE buffer
 * buf of buf_bytes bytes and wrapping around.  pattern 0: fully coalesced (a wave reads 1 KB contiguous
 * per instruction; kernel k_stream_read); pattern 1: the MFMA-operand layout the attention kernel uses
 * for keys (rows of 256 bytes, lane = row lane%16, 16-byte chunk lane/16 of each 64 bytes; kernel
 * k_stream_read_operand); pattern 2: plain copy that reads the first half of each window and WRITES the
 * second half (kernel k_stream_copy; buf is modified).  Returns the average time of one launch in microseconds (HIP events;
 * synchronises).  This is the practical bandwidth ceiling of the box for a launch of that size, and a
 * kernel of known traffic for calibrating hardware counters.  bytes_per_launch must be a multiple of
 * 524288 and <= buf_bytes. */
int arkv_measure_stream_read(void* buf, uint64_t buf_bytes, uint64_t bytes_per_launch, int32_t launches,
                             int32_t pattern, void* hip_stream, float* avg_us);

#ifdef __cplusplus
}
#endif
#endif
