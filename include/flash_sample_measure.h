/*
 * flash_sample_measure.h -- measurement aids that ship in the same shared library as the sampler
 * (include/flash_sample.h) but are no part of the method: a streaming kernel of known traffic to
 * scale profiler counters with, and the launcher's kernel choice as pure host logic.  The
 * benchmark and the tests use them; a serving stack does not need this header.
 */
#ifndef FLASH_SAMPLE_MEASURE_H
#define FLASH_SAMPLE_MEASURE_H

#include <stddef.h>
#include <stdint.h>

#include "flash_sample.h"

#ifdef __cplusplus
extern "C" {
#endif

/* A plain streaming kernel of known size on device memory.
 * dst == NULL: read `bytes` bytes from src (the read-bandwidth ceiling of the device);
 * dst != NULL: copy src to dst.  bytes must be a multiple of 16, pointers 16-byte aligned.
 * `sink` is a 4-byte device location the read variant may write to.  Asynchronous on `stream`. */
fs_status flash_measure_stream_probe(void* dst, const void* src, size_t bytes, uint32_t* sink,
                                     void* stream);

/* Which stage-1 kernel the automatic choice takes for a bf16 problem (B, D, V) on a device with
 * `compute_units` CUs: 0 = the split-K kernel, otherwise the tile shape number of
 * FS_TUNE_TILE_SHAPE.  Pure host logic (no device call); -1 for an invalid shape. */
int flash_measure_kernel_choice(int B, int D, int V, int compute_units);

#ifdef __cplusplus
}
#endif
#endif /* FLASH_SAMPLE_MEASURE_H */
