/*
 * csketch_probe.h -- a measurement aid exported by libcsketch.so beside the C ABI of
 * csketch.h.  No part of the method and not for callers of the library: bench.py uses it to
 * time a plain read of the worker vectors on the machine it runs on, the rate that the
 * bandwidth-bound kernels of the path are reported against.
 */
#ifndef CSKETCH_PROBE_H
#define CSKETCH_PROBE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Reads the W vectors x_w[w][0..d) once, as plainly as the hardware allows (16-byte loads, two
 * in flight per thread, one stream per vector), and adds the sum of all values to out[0]
 * (device float, accumulated into, fp32 in no fixed order) so that the loads cannot be dropped.
 * x_w: HOST array of W device pointers to float[d].  W >= 1, d >= 0.  Returns 0, or the
 * negative cs_status of csketch.h.  `stream` as in csketch.h. */
int cs_probe_stream_read(const float* const* x_w, int32_t W, int64_t d, float* out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* CSKETCH_PROBE_H */
