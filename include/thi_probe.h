/*
 * thi_probe.h -- measurement probes for the benchmark, in a library of their own (libthi_probe.so):
 * they compute nothing useful and are not part of the product library.  What the GPU sustains for the
 * two resources the kernels of libthi are bound by, to be reported next to the nominal peaks.
 * Status codes are those of thi.h.  Device pointers; the calls enqueue on `hip_stream` and return.
 */
#ifndef THI_PROBE_H
#define THI_PROBE_H

#include <stddef.h>

#include "thi.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * thi_probe_stream_read: reads `bytes` (>= 16 MiB, device memory, 16-byte aligned) once with the
 * access pattern of an ideal weight-streaming kernel.  bytes / elapsed = attainable HBM read rate.
 * thi_probe_mfma_f16: `workgroups` x 8 waves each issue iters x 8 v_mfma_f32_32x32x16_f16 on
 * register operands taken from `operands` (64 KiB of fp16 device memory: constant or random values --
 * the clock under load depends on operand toggling).  flops = workgroups * 8 * iters * 8 * 32768.
 * `sink` is 4 bytes of device memory that is (practically) never written.
 */
int thi_probe_stream_read(const void* buffer, size_t bytes, void* sink, void* hip_stream);
int thi_probe_mfma_f16(const void* operands, int iters, int workgroups, void* sink, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* THI_PROBE_H */
