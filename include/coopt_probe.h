/*
 * coopt_probe.h -- C ABI of libcoopt_probe.so, a measurement aid that ships beside the paged
 * decode-attention library (coopt_attn.h) and is no part of the method: the benchmark uses it to
 * quote the decode kernels' bandwidth beside the rate this GPU sustains for a kernel that only
 * reads.  Conventions (device pointers, hip_stream, return values) as in coopt_attn.h.
 */
#ifndef COOPT_PROBE_H
#define COOPT_PROBE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Reads `bytes` of device memory at `buf` (16-byte aligned) once with 16-byte streaming loads from
 * `workgroups` workgroups of 256 lanes and writes nothing (one word of `sink`, device memory of at
 * least 4 bytes, only if the XOR of the data hits an arbitrary constant).  Timed by the caller.
 * Returns 0, -1 for a NULL pointer, -2 for workgroups outside [1, 2^20] or a misaligned buffer,
 * -4 if the HIP runtime refused the launch.
 */
int coopt_stream_read_probe(const void* buf, size_t bytes, int32_t workgroups, void* sink,
                            void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* COOPT_PROBE_H */
