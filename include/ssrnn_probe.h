/* Measurement aids of libssrnn.so that are not part of the method's interface
 * (include/ssrnn.h): kernels that only read, against which bench.py prices the
 * stage kernels next to the published peaks.  Same conventions as ssrnn.h
 * (device pointers, work queued on `stream`, ssrnn_status return values). */
#ifndef SSRNN_PROBE_H
#define SSRNN_PROBE_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

/* One launch that reads bufs[0 .. n) (a HOST array of n <= 8 device pointers,
 * each `bytes` long, 16-byte aligned, bytes a multiple of 16) once with
 * streaming 16-byte loads and keeps nothing.  The grid has the shape of a
 * stage launch that holds n stages: blockIdx.y picks the buffer, `groups`
 * workgroups of 512 threads share each buffer (0: 256).  n = 1 prices a
 * one-stage launch, n = 8 the eight-stage launches of the wavefront schedule;
 * a buffer that fits the caches, read again and again, prices the
 * cache-resident configurations.  sink: 4 bytes of device memory the kernel may
 * write. */
int ssrnn_read_probe(const void* const* bufs, int n, size_t bytes, int groups,
                     void* sink, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SSRNN_PROBE_H */
