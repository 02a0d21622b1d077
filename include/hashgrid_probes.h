/*
 * hashgrid_probes.h - C ABI of libhashgrid_probes: small kernels that measure, on the GPU at hand, the
 * rates the encoding's passes are compared with.  Measurement tooling for the benchmark, kept out of
 * the encoding's own library (libhashgrid, hashgrid.h); nothing here is part of the method.
 *
 * Each call enqueues one kernel on `stream` (a hipStream_t passed as void*; NULL is the default
 * stream); the caller times it.  All pointers are device pointers owned by the caller.  Status codes
 * are hashgrid.h's.
 *   copy          dst[0..bytes) = src[0..bytes) with 16-byte accesses; bytes a multiple of 16,
 *                 both pointers 16-byte aligned.  Moves 2 * bytes.
 *   gather        n_gathers independent 4-byte loads at pseudo-random words of table
 *                 [table_words] (a power of two, at most 2^32), 16 per thread; the per-thread sums
 *                 go to sink [n_gathers / 16].  n_gathers must be a multiple of 4096.
 *   atomic_add    n_adds device-scope fp32 atomic adds of 1.0 at pseudo-random words of table
 *                 [table_words] (same constraints); the table is modified.
 *   gather_lines  the access shape of the encoding's forward pass on hashed levels: one thread per
 *                 "point" in workgroups of 1024; for each of n_levels "levels" a point reads two
 *                 adjacent 4-byte words in each of 4 pseudo-random 128-byte lines of that level's
 *                 slice (slice l mod n_slices of table [n_slices][slice_words], slice_words a power
 *                 of two >= 32), and the workgroup meets at a barrier before the next level.
 *                 n_points must be a multiple of 1024; the per-point sums go to sink [n_points].
 *                 Fetches n_points * n_levels * 4 lines.
 * HG_ERR_INVALID_ARG when a constraint above is not met; a size of 0 is HG_OK.
 */
#ifndef HASHGRID_PROBES_H
#define HASHGRID_PROBES_H

#include "hashgrid.h"

#ifdef __cplusplus
extern "C" {
#endif

hg_status hashgrid_probe_copy(const void* src, void* dst, uint64_t bytes, void* stream);
hg_status hashgrid_probe_gather(const uint32_t* table, uint64_t table_words, uint64_t n_gathers, uint32_t seed,
                                uint32_t* sink, void* stream);
hg_status hashgrid_probe_atomic_add(float* table, uint64_t table_words, uint64_t n_adds, uint32_t seed,
                                    void* stream);
hg_status hashgrid_probe_gather_lines(const uint32_t* table, uint64_t slice_words, uint32_t n_slices,
                                      uint64_t n_points, uint32_t n_levels, uint32_t seed, uint32_t* sink,
                                      void* stream);

#ifdef __cplusplus
}
#endif
#endif /* HASHGRID_PROBES_H */
