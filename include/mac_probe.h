/* Read-only streaming probe for MI355X (gfx950): what a kernel that only loads can pull out of HBM with the access
 * pattern of a paged KV cache.  Measurement aid beside the MAC-Attention library (libmacattn.so, mac_attn.h): it
 * computes nothing of the method.  The decode-attention kernel reads every K/V byte once (Sec. 2: the sum over all
 * cached keys), in runs of one (page, K|V, head) block -- 4 KiB for 16-token pages of 128 bf16 -- at page addresses
 * that are random in HBM; this probe reads the same bytes the same way without any arithmetic, which gives the
 * ceiling to hold the kernel's achieved bandwidth against (the roofline fraction itself is quoted against the
 * published 8 TB/s).
 */
#ifndef MAC_PROBE_H
#define MAC_PROBE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Streams `n_segments` segments of `segment_bytes` each out of `buffer` (device memory, 16-byte aligned, at least
 * (max(order) + 1) * segment_bytes long) `iterations` times on `hip_stream` and returns the average duration of one
 * pass in microseconds in *us_per_pass (HIP events around all passes; the call synchronises the stream).
 *   order          device pointer, int32[n_segments]: segment index read i-th (a permutation for a random walk, the
 *                  identity for a linear one).  Wave w of the launch reads order[w * k .. (w + 1) * k), k =
 *                  n_segments / (4 * work_groups); n_segments must be a multiple of 8 * work_groups.
 *   segment_bytes  2048, 4096, 8192 or 16384.
 *   non_temporal   1: loads carry the non-temporal hint (as the attention kernel's K/V loads do); 0: plain loads.
 *   work_groups    256-thread work-groups launched (1 .. 65536).
 * Nothing is allocated and nothing is written except 4 bytes at `sink` (device pointer, never actually stored to
 * unless the data has one particular checksum; it keeps the compiler from dropping the loads).
 * Returns 0, -1 for a bad argument, -2 for a HIP error.
 */
int mac_probe_stream(const void* buffer, const int32_t* order, int64_t n_segments, int32_t segment_bytes,
                     int32_t non_temporal, int32_t work_groups, int32_t iterations, void* sink, void* hip_stream,
                     float* us_per_pass);

#ifdef __cplusplus
}
#endif
#endif
