/*
 * def_probe.h -- plain streaming kernels of exactly known traffic (non-temporal
 * dwordx4 accesses), in the launch shape of the library's streaming pass (one-wave
 * workgroups, one float4 per lane, residency capped through an LDS reservation) or
 * in a few other shapes.
 *
 * They are measurement aids, not part of the method (arXiv 2004.05298 has no such
 * step): the benchmark runs them beside the DEF step to show what a pure read, a
 * pure write, a copy and an in-place update sustain on the same GPU in the same
 * run, and hardware counters are scaled by what they read for these launches.
 */
#ifndef DEF_PROBE_H_
#define DEF_PROBE_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum def_probe_kind {
    DEF_PROBE_READ = 0,     /* reads src[0..n): 4n bytes read, nothing written               */
    DEF_PROBE_WRITE = 1,    /* dst[i] = value: 4n bytes written, nothing read                */
    DEF_PROBE_COPY = 2,     /* dst[i] = src[i]: 4n read, 4n written                          */
    DEF_PROBE_UPDATE = 3    /* dst[i] = dst[i] * value: 4n read and 4n written in place      */
} def_probe_kind;

/*
 * Enqueue one probe launch on `stream` (hipStream_t of the current GPU; NULL = null stream).
 *   src, dst     DEVICE, 16-byte aligned, n floats each (src unused for WRITE and UPDATE, dst
 *                unused for READ, where it may be NULL); n a multiple of 256, 0 < n < 2^39.
 *   value        the fill value / scale factor.
 *   threads      workgroup size, 64 or 256.
 *   quads        float4 groups per lane, 1, 2 or 4 (lane t of a workgroup takes groups
 *                t, t + threads, ...: every wave instruction covers 1 KiB of consecutive bytes).
 *   lds_reserve  bytes of LDS reserved per workgroup (never touched; caps residency: 10240 with
 *                one-wave workgroups -> 16 waves per compute unit, 0 -> as many as fit); <= 65536.
 * Returns DEF_OK, DEF_EINVAL (nothing launched) or DEF_EHIP.  Asynchronous.
 */
int def_probe_stream(int kind, const float *src, float *dst, uint64_t n, float value, uint32_t threads,
                     uint32_t quads, uint32_t lds_reserve, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* DEF_PROBE_H_ */
