// Calibration entry points of librd.so that are not part of the method's interface (include/rd.h):
// the benchmark uses them to measure the machine's own floor beside the kernels' times.
#pragma once
#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * rd_debug_stream_read — calibration aid, not part of the method: one launch in which `workgroups`
 * workgroups of 256 threads read `bytes` bytes at `src` (device memory, 16-byte aligned; a trailing
 * part of less than 16 bytes is ignored) once, as contiguous slabs with 16-byte loads, and discard
 * them.  Timing it over the bytes an rd_tree_attn launch has to read gives the machine's floor for
 * that launch, which the benchmark reports beside the kernel's own time.  `sink`: device word that
 * is written only if the folded data happens to equal one magic value, or NULL.
 */
int rd_debug_stream_read(const void *src, size_t bytes, int workgroups, uint32_t *sink, void *stream);

#ifdef __cplusplus
}
#endif
