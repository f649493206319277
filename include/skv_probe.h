/*
 * Measuring sticks for the benchmark: plain streaming kernels that are no part of the method (they
 * compute nothing of Sec. 2-3) and live in a library of their own, libskv_probe.so, so that the
 * product library exports the method only.  C ABI, device pointers, work enqueued on `stream`;
 * return values are skv_status codes.
 */
#ifndef SKV_PROBE_H
#define SKV_PROBE_H

#include <stddef.h>
#include <stdint.h>

#include "skv.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * One launch that only READS.  The first *bytes_read <= bytes bytes of src (whole multiples of
 * workgroups * 16 KiB) are streamed, each workgroup a contiguous slice, and nothing is written.  Timing it
 * tells what a plain streaming read of that size reaches on the machine at hand, the yardstick the decode
 * range kernels (which read every row of the compressed cache once, Sec. 2.1 Eq. 2 inside App. A.1 Eq. 18)
 * are compared with.
 *   src        device, 16-byte aligned, at least `bytes` long
 *   streaming  nonzero: streaming (non-temporal) loads, as the range kernels use for rows that no cache
 *              will hold; 0: ordinary loads
 *   sink       device float32 [workgroups]: never written in practice, must be valid
 * Errors: NULL, ALIGN, SHAPE (workgroups outside [1, 65535], or bytes below workgroups * 16 KiB), HIP.
 */
skv_status skv_probe_stream_read(const void* src, size_t bytes, int32_t workgroups, int32_t streaming,
                                 void* sink, size_t* bytes_read, void* stream);

/*
 * One launch that reads two buffers and writes a third (c = a ^ b), two bytes read for each byte written:
 * the traffic mix of the chunk append (Sec. 2.1 Eq. 1 at r_k + r_v = head size).  The first *bytes_each <=
 * bytes bytes of each buffer take part (whole multiples of workgroups * 16 KiB), each workgroup a
 * contiguous slice.
 *   a, b  device, 16-byte aligned, at least `bytes` long, read
 *   c     device, 16-byte aligned, at least `bytes` long, overwritten; must not overlap a or b
 * Errors: NULL, ALIGN, SHAPE (workgroups outside [1, 65535], or bytes below workgroups * 16 KiB), HIP.
 */
skv_status skv_probe_stream_mix(const void* a, const void* b, void* c, size_t bytes, int32_t workgroups,
                                size_t* bytes_each, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SKV_PROBE_H */
