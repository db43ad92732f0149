/*
 * chai_probe.h -- measurement aids of libchai.so.  NOT part of the method's boundary (that is chai.h): two kernels
 * that do no useful work and exist so that the benchmark can quote the library's kernels against what the device
 * at hand reaches with nothing in the way -- a bare streaming read (the practical ceiling of the HBM-bound decode
 * kernels) and the matrix pipe alone (the practical ceiling of the prefill and projection kernels).  Conventions
 * (device pointers, streams, status codes) as in chai.h.
 */
#ifndef CHAI_PROBE_H
#define CHAI_PROBE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Measurement aid, not a step of the method: a bare streaming read of
 * `bytes` bytes (a multiple of 16, 16-byte aligned) of device memory with the
 * load pattern of the decode kernels (16-byte non-temporal loads, eight in
 * flight per lane) in the best launch shape a sweep found on MI355X: one
 * workgroup per CU from 256 MiB up, 128 KiB per workgroup below that.  The rate it reaches is the
 * practical ceiling for the HBM-bound kernels above on the device at hand;
 * the benchmark quotes its kernels against it next to the nominal peak.
 *   sink        one fp32 on the device (written practically never; it keeps
 *               the loads alive)
 *   start/stop  hipEvent_t handles as void* stamped with the kernel's begin
 *               and end (either may be NULL)
 */
int chai_stream_read_probe(const void *buf, size_t bytes, float *sink, void *stream, void *start_event,
                           void *stop_event);

/*
 * Measurement aid, not a step of the method: the matrix pipe alone.  Every
 * wave of a chip-filling launch (two waves per SIMD) takes six bf16 operand
 * fragments from `buf` (device memory, at least 16 bytes, 16-byte aligned;
 * read modulo its length) and issues `rounds` rounds of eight independent
 * v_mfma_f32_32x32x16_bf16 with nothing else in the loop.  The rate depends
 * on the operand values (switching activity moves the clocks), so pass the
 * data of the workload at hand.  *flops (HOST pointer, may be NULL) receives
 * the floating-point operations of one launch; sink and the events as for
 * chai_stream_read_probe.  The benchmark quotes the prefill and projection
 * kernels against this rate next to the nominal peak.
 */
int chai_mfma_rate_probe(const void *buf, size_t bytes, int rounds, float *sink, double *flops, void *stream,
                         void *start_event, void *stop_event);

#ifdef __cplusplus
}
#endif

#endif /* CHAI_PROBE_H */
