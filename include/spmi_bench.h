/* spmi_bench.h: measurement hooks of the spmi library.  Not part of the product interface (include/spmi.h): they exist
 * so that a benchmark can time the library's own kernels on the stream they run on and scale its bandwidth figures by a
 * plain copy.  Same conventions as spmi.h: plain pointers marked HOST or DEVICE, status codes only. */
#ifndef SPMI_BENCH_H
#define SPMI_BENCH_H

#include "spmi.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Key for sp_tensor_tune: value 1 switches kernel timing on for the tensor, 0 off. */
enum { SP_TUNE_PROFILE = 4 };

/* Kernel timing for measurements.  After sp_tensor_tune(t, SP_TUNE_PROFILE, 1) every sp_matmul on
 * t brackets its main kernel (the one that streams A; not the zero fill, not the fix-up; both passes of
 * the binned SpMV, all three launches of the column-segmented one) with a
 * pair of HIP events on the caller's stream.  sp_profile_read waits for those events, returns
 * the summed kernel time in milliseconds and the number of launches, and clears the record.
 * Profiling costs two event records per call; leave it off in production. */
sp_status sp_profile_read(sp_tensor *t, double *ms_total /* HOST */, int64_t *launches /* HOST */);

/* dst[i] = src[i] for `bytes` bytes (multiple of 16), a plain streaming copy kernel: the
 * yardstick the benchmark scales its bandwidth figures and hardware counters by. */
sp_status sp_stream_copy(void *dst /* DEVICE */, const void *src /* DEVICE */, size_t bytes, void *stream);

/* Reads `bytes` bytes (multiple of 16) at src and writes nothing (sink: 4 DEVICE bytes that are practically never
 * written): the read-only streaming rate, the yardstick for kernels whose traffic is mostly reads. */
sp_status sp_stream_read(const void *src /* DEVICE */, size_t bytes, void *sink /* DEVICE */, void *stream);

/* Which sort the storage builder (sp_pack, sp_pack_sum) uses from now on, process-wide: 0 = it chooses (the default: most
 * significant digit first with an LDS finishing pass for a million entries or more whose top key bits are spread evenly
 * enough, least significant digit first otherwise), 1 = always least significant digit first, 2 = always most significant
 * digit first (any size below 2^31 entries: how the tests reach its rare paths with small inputs).  Both sorts are stable
 * and give the same storage bit for bit.  Returns SP_ERR_UNSUPPORTED for another value. */
sp_status sp_pack_sort_mode(int mode);

#ifdef __cplusplus
}
#endif
#endif /* SPMI_BENCH_H */
