/*
 * vq_bench.h -- measurement aid of the benchmark (libvq_bench.so).  NOT part of the product:
 * libvq.so neither exports nor uses it.
 */
#ifndef VQ_BENCH_H_
#define VQ_BENCH_H_

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Reads `bytes` bytes (a multiple of 16, 16-byte aligned device memory) once with the same
 * non-temporal 128-bit loads the GEMV kernels stream their indices with, and discards them.
 * Timing it over a buffer much larger than the caches gives the HBM read rate this GPU
 * actually sustains, which the bench reports next to the nominal peak.  `stream` is a
 * hipStream_t.  Returns 0, or the negative code of the same meaning as in vq.h
 * (-1 null pointer, -4 alignment, -5 launch refused, -6 bad size).
 */
__attribute__((visibility("default")))
int vq_bench_stream_read(const void* buf, size_t bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* VQ_BENCH_H_ */
