/* pipad_ceilings.h - measurement kernels that bound what the aggregation can reach on this GPU.
 *
 * Not part of the aggregation path: small kernels with the aggregation kernel's access shapes
 * (16 bytes per lane, four row gathers in flight per lane), used by `bench.py --ceilings` and by
 * bench.py's roofline block to state the attainable bound
 *      max( algorithmic bytes / streaming rate ,  gathered bytes / gather rate )
 * next to the plain HBM-roofline fraction (Section 3.2 "Memory access inefficiency" is about
 * exactly this gap between moved and useful bytes).  They allocate nothing and only enqueue work.
 * Same conventions as pipad.h: device pointers on the current device, `stream` is a hipStream_t,
 * return 0 or a negative pipad_status.
 */
#ifndef PIPAD_CEILINGS_H_
#define PIPAD_CEILINGS_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Streams `bytes` (a multiple of 16) of `src` through the chip once, 16 bytes per lane, and
 * writes one float per workgroup to `sink` (at least `pipad_ceiling_sink_floats()` floats) so
 * that the loads cannot be dropped. */
int pipad_ceiling_stream_read(const float *src, size_t bytes, float *sink, void *stream);

/* Copies `bytes` (a multiple of 16) from `src` to `dst` (both 16-byte aligned, not overlapping),
 * 16 bytes per lane.  Besides the copy rate it gives the traffic counters of a profiler a kernel
 * whose memory traffic is known exactly: `bytes` read and `bytes` written. */
int pipad_ceiling_stream_copy(const float *src, float *dst, size_t bytes, void *stream);

/* Gathers `count` rows of a row-major float table in the aggregation kernel's access shape and
 * sums them (one float4 per lane team and wave goes to `sink`).
 *   table        device, `rows` rows of `row_floats` floats (16, 32 or 64: a lane team of
 *                row_floats / 4 lanes reads one row with 16-byte loads), row stride
 *                `stride_floats` >= row_floats, a multiple of 4; rows * stride_floats * 4 < 4 GiB
 *   index        device, int32[count], every value in [0, rows); entry e is gathered by the wave
 *                that owns position e, so the order of `index` is the order in time
 *   xcd_classes  0: every workgroup takes the next chunk of `index`.  8: `index` holds 8
 *                consecutive sections of count / 8 entries and workgroup b only takes chunks of
 *                section b mod 8 - with the workgroups dealt round-robin to the 8 XCDs, XCD x then
 *                only ever gathers section x (count must be a multiple of 8 * 4096).
 *   count        a multiple of 4096 (entries per workgroup)
 */
int pipad_ceiling_gather(const float *table, int64_t rows, int32_t row_floats, int64_t stride_floats,
                         const int32_t *index, int64_t count, int32_t xcd_classes, float *sink,
                         void *stream);

/* Floats the `sink` argument of the calls above must hold. */
size_t pipad_ceiling_sink_floats(void);

#ifdef __cplusplus
}
#endif
#endif /* PIPAD_CEILINGS_H_ */
