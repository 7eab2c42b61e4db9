/*
 * stream_probe.h -- C ABI of the benchmark's measurement aid (libmgwfbp_bench_aid.so).
 *
 * Not part of the MG-WFBP library and not part of the method: bench.py loads it to learn what the bare
 * read/write mix of a kernel reaches on the machine at hand, and to empty the GPU's memory-side cache
 * between timed steps.  Every function returns 0 on success, -1 for an invalid argument, -3 if the
 * launch failed; all of them enqueue on `hip_stream` (a hipStream_t passed as void*; NULL is the default
 * stream) and return without waiting.
 */
#ifndef MGWFBP_BENCH_AID_STREAM_PROBE_H
#define MGWFBP_BENCH_AID_STREAM_PROBE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Streams n_read read-only, n_write write-only and n_update updated-in-place binary32 device arrays of
 * `elems` elements each through the GPU with the access shape of the pipeline kernels (one workgroup of
 * 256 lanes per 2048-element tile, 16-byte non-temporal accesses, all loads of a tile before its first
 * store):
 *     write[i][e]  = read[i mod n_read][e]         (1.0f if n_read = 0)
 *     update[j][e] = update[j][e] + sum_i read[i][e]
 * read_ptrs / write_ptrs / update_ptrs are HOST arrays of device pointers (NULL allowed where the count
 * is 0); the arrays must not overlap.  Counts: n_read, n_write in {0, 1, 2, 4, 8, 16}, n_update in
 * {0, 1, 2}, not all zero; elems a positive multiple of 2048; 16-byte aligned arrays. */
int bench_aid_stream_probe(const float* const* read_ptrs, int32_t n_read, float* const* write_ptrs,
                           int32_t n_write, float* const* update_ptrs, int32_t n_update, uint64_t elems,
                           void* hip_stream);

/* The same arrays walked one array at a time (the order the library's kernels use): a workgroup of `block_lanes`
 * lanes owns vectors_per_step x block_lanes x 4 consecutive elements, loads its part of read array i, stores it to
 * write array i (i < n_write; write arrays beyond n_read get 1.0f), adds it to a running sum, goes on to array
 * i + 1, and finally adds the sum to the update arrays one after the other.  `lds_bytes` (<= 64 KiB) of unused
 * dynamic LDS per workgroup bounds how many workgroups share a compute unit (160 KiB each), i.e. how many bytes
 * of loads a compute unit has in flight.  (block_lanes, vectors_per_step) in {(64,1), (128,1), (128,2), (256,1),
 * (256,2), (256,4)}; elems a multiple of vectors_per_step x block_lanes x 4; any counts 0..16, not all zero. */
int bench_aid_paced_probe(const float* const* read_ptrs, int32_t n_read, float* const* write_ptrs,
                          int32_t n_write, float* const* update_ptrs, int32_t n_update, uint64_t elems,
                          int32_t block_lanes, int32_t vectors_per_step, uint32_t lds_bytes, void* hip_stream);

/* Displaces whatever the memory-side cache (256 MB on MI355X) holds: copies the first half of the device
 * buffer `buf` (`bytes` long, a multiple of 8192, 16-byte aligned) onto its second half with ordinary,
 * cacheable loads and stores, so bytes/2 are read and bytes/2 are written.  With bytes >= 1 GiB nothing that
 * an earlier kernel left in that cache survives. */
int bench_aid_cache_scrub(void* buf, uint64_t bytes, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif
