/*
 * spec_probe.h - measurement aid shipped next to libspectree, in a library of its own (libspecprobe): not
 * part of the method and not needed to use it. bench.py times it beside the attention kernels.
 */
#ifndef SPEC_PROBE_H
#define SPEC_PROBE_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Reads `bytes` (a multiple of 16 is used) from the DEVICE buffer `buf` once with non-temporal 16-byte loads,
 * a contiguous piece per workgroup, and writes nothing (`sink`: 16 device bytes that are never written in
 * practice). Enqueued on `hip_stream` (hipStream_t as void*), no synchronisation. Timed over a buffer much
 * larger than the on-chip caches it gives the read bandwidth this machine sustains for a launch of that
 * size: the practical ceiling next to the published HBM peak. Returns 0, -1 (bad argument) or -4 (launch
 * failed).
 */
int spec_probe_read_stream(const void* buf, size_t bytes, void* sink, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* SPEC_PROBE_H */
