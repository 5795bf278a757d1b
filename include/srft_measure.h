/*
 * srft_measure.h -- measurement aids, NOT part of the method and not part of libsrft_kv.so: plain streaming
 * kernels (libsrft_measure.so) used to calibrate the profiler's HBM byte counters and to measure what the
 * memory system offers a kernel that has the traffic shape of the write path or of the read path.
 * Status codes are srft_status (srft_kv.h).  Device pointers, caller-owned; calls enqueue on hip_stream
 * (a hipStream_t passed as void*, NULL = the default stream) and return without synchronising.
 */
#ifndef SRFT_MEASURE_H
#define SRFT_MEASURE_H

#include <stdint.h>

#include "srft_kv.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * A plain streaming copy of n_bytes (a multiple of 16, both pointers 16-byte aligned), persistent grid of
 * 8 workgroups per compute unit.  n_bytes == 0 is a no-op.
 */
int srft_stream_copy(void* dst_dev, const void* src_dev, int64_t n_bytes, void* hip_stream);

/*
 * A streaming kernel with a chosen traffic shape.  For each of n_tiles tiles it reads read_bytes_per_tile
 * contiguous bytes from src_dev (tile t at t * read_bytes_per_tile) and writes write_bytes_per_tile contiguous
 * bytes to dst_dev, with coalesced 16-byte accesses and no arithmetic.  With 8192 : 2560 it has the write path's
 * byte mix at d = 128 (32 vectors per tile), with 2560 : 8192 the read path's.
 * Byte counts must be multiples of 16, at most 32 KiB read per tile, and not both zero (one of them zero gives
 * the read-only or the write-only stream); workgroups = 0 picks 3 per compute unit.  `access` is a bit set:
 * 1 = non-temporal loads and stores; 2 = every lane reads 64 contiguous bytes with four 16-byte loads (the
 * shape a per-lane de-interleave of 32 consecutive inputs needs; read_bytes_per_tile must then be a multiple of
 * 16 KiB) instead of loads that cover 1 KiB per wavefront contiguously; 4 = every accelerator die (workgroup index
 * mod 8) walks one contiguous eighth of the tiles instead of every eighth tile (grids that are a multiple of 8).
 */
int srft_stream_mix(const void* src_dev, void* dst_dev, int64_t n_tiles, int read_bytes_per_tile,
                    int write_bytes_per_tile, int workgroups, int access, void* hip_stream);

int srft_measure_last_hip_error(void);    /* the hipError_t of the most recent SRFT_ERR_HIP of this library */

#ifdef __cplusplus
}
#endif
#endif /* SRFT_MEASURE_H */
