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

/*
 * The memory requests of one fused append + attention launch (Section 4.2: the tree's K/V rows appended, every
 * node attending to prefix and tree) without any arithmetic, for bf16 rows of 128 elements and equal prefix
 * lengths: B * H workgroups, one per (request, head) pair, each streaming rows [0, P + N) of its K and V through
 * LDS. All pointers are DEVICE pointers, 16-byte aligned, contiguous: k_cache, v_cache [B, H, S_cap, 128] bf16;
 * q, k_new, v_new, out [B, N, H, 128] bf16. `flags` (any combination) adds to the K/V stream:
 *   QUERIES   the N query rows of the pair are read first;
 *   NEW_ROWS  rows [P, P + N) come from k_new / v_new instead of the caches;
 *   APPEND    rows [P, P + N) of both caches are written (with what was loaded for them);
 *   OUTPUTS   N rows of `out` are written at the end (with whatever the LDS holds).
 * Requires 1 <= N <= 128, P >= 0, P + N <= S_cap. Enqueued on `hip_stream`, no synchronisation. The time of a
 * launch is what the traffic of that attention launch costs in this access pattern, the floor for a kernel that
 * also has to compute. Returns 0, -1 (bad argument) or -4 (launch failed).
 */
#define SPEC_PROBE_TRAFFIC_QUERIES 1
#define SPEC_PROBE_TRAFFIC_NEW_ROWS 2
#define SPEC_PROBE_TRAFFIC_APPEND 4
#define SPEC_PROBE_TRAFFIC_OUTPUTS 8
int spec_probe_attention_traffic(int B, int H, int N, int P, int S_cap, void* k_cache, void* v_cache, const void* q,
                                 const void* k_new, const void* v_new, void* out, int flags, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* SPEC_PROBE_H */
