/*
 * svdcache_probes.h -- memory-system probes for MI355X (gfx950), built as libsvdcache_probes.so.
 *
 * Not part of the SVD-Cache computation: these kernels move bytes and compute nothing.  The benchmark times them
 * (python bench.py --probes) to put measured ceilings next to the published 8 TB/s when it reports what fraction
 * of the memory roofline the step kernels reach: what a plain copy gets on this machine, what a copy with a step
 * kernel's access skeleton gets, and what a re-read out of the Infinity Cache is worth.
 *
 * All pointers are DEVICE pointers, 16-byte aligned; sizes in bytes, multiples of 16.  Calls enqueue one kernel on
 * `stream` (hipStream_t as void*, NULL = default stream) and return 0, or -1 for bad arguments, -7 if the launch
 * failed.  The caller owns all memory.
 */
#ifndef SVDCACHE_PROBES_H
#define SVDCACHE_PROBES_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* dst[i] = src[i]: one 16-byte load and one 16-byte store per lane, one piece per thread, consecutive lanes on
 * consecutive addresses (the plainest streaming copy). */
int32_t svdc_probe_copy(void* dst, const void* src, size_t bytes, void* stream);

/* Read-only stream over src (four 16-byte loads per thread); `sink` (4 bytes) is written only if an impossible
 * value shows up, which keeps the loads alive.  Run twice on <= 256 MB to time a re-read out of the Infinity Cache. */
int32_t svdc_probe_read(const void* src, size_t bytes, void* sink, void* stream);

/* Copy of a [rows x 6144 bytes] row-major matrix with the access skeleton of the cached-step kernel at 3072 bf16
 * channels: a load instruction of a wave covers 16 rows x 64 bytes (the matrix-core lane layout), a wave owns 12
 * such chunks of a row tile, a workgroup of four waves half a row, and a workgroup walks over `tiles_per_group`
 * 16-row tiles, one tile in flight ahead -- interleaved with the other workgroups of its 4608-row block
 * (interleave != 0, as the kernel does) or contiguous.  groups_per_cu (0..8; 0 = no limit) caps how many workgroups
 * share a compute unit, by giving each that share of the LDS: the cached-step kernel, with its basis operands in
 * registers, runs one workgroup per compute unit.  rows must be a multiple of 4608. */
int32_t svdc_probe_tile_copy(void* dst, const void* src, int32_t rows, int32_t tiles_per_group, int32_t interleave,
                             int32_t groups_per_cu, void* stream);

/* Copy of the same matrix with the skeleton of the full-step kernel: one persistent workgroup per compute unit
 * loads a whole tile of `tile_rows` (16, 32 or 48) rows x 6144 bytes into registers in one burst, stores it, and only
 * then requests its next tile. */
int32_t svdc_probe_burst_copy(void* dst, const void* src, int32_t rows, int32_t tile_rows, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SVDCACHE_PROBES_H */
