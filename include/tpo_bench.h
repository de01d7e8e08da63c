/*
 * tpo_bench.h -- C ABI of libtpo_bench.so: the measurement aid of the benchmark.  It is no part
 * of the operator library (libtpo.so, tpo.h) and implements no passage of the paper: it gives
 * the plain streaming rate the operator kernels are compared with, and a kernel of exactly
 * known HBM traffic against which hardware counters are calibrated.
 */
#ifndef TPO_BENCH_H
#define TPO_BENCH_H

#include "tpo.h" /* status codes, TPO_F64 / TPO_F32 */

#ifdef __cplusplus
extern "C" {
#endif

/*
 * tpo_stream_scale -- enqueue the plain streaming kernel v[i] = u[i] * D[i], i < count, over flat
 * DEVICE arrays of `dtype` on `stream` (a hipStream_t, NULL for the default stream); returns
 * without synchronising.  It moves the operator's algorithmic traffic (two reads and one write
 * per word) and nothing else, so the benchmark uses its time as the streaming ceiling and its
 * HBM counters to calibrate those of the operator's kernels.  Pointers must be 16-byte aligned
 * and stay owned by the caller; no aliasing check is made (v == u is fine).  Needs no
 * tpo_create and no libtpo.so.  Errors: TPO_ERR_INVALID_ARG (dtype, negative count, null or
 * misaligned pointer), TPO_ERR_UNSUPPORTED (more than 2^31-1 workgroups), TPO_ERR_DEVICE.
 */
int tpo_stream_scale(const void *u, const void *D, void *v, long long count, int dtype,
                     void *stream);

#ifdef __cplusplus
}
#endif
#endif /* TPO_BENCH_H */
