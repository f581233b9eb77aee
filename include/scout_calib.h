/*
 * scout_calib.h -- measurement aids (libscout_calib.so), not part of the method and not part of the
 * product library: a copy of known size for scaling HBM byte counters, and the two access patterns
 * of the path with nothing computed.  Every pointer is DEVICE memory owned by the caller; `stream` is
 * a hipStream_t; calls enqueue and return; return codes are those of scout.h.
 */
#ifndef SCOUT_CALIB_H
#define SCOUT_CALIB_H

#include "scout.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Measurement aid, not part of the method: copy `bytes` (a multiple of 16) of
 * device memory with one 16-byte load and store per element.  Profiling runs
 * read the HBM byte counters of this copy of known size to scale the counters
 * of the other kernels.
 */
int scout_calib_copy(const void* src, void* dst, size_t bytes, void* stream);

/*
 * Measurement aids, not part of the method: the two access patterns of the path
 * with nothing computed, so that a benchmark can state the rate this GPU
 * sustains for them next to the kernels' own.
 *   scout_calib_read    reads `bytes` (a multiple of 16) of device memory once,
 *                       as a stream (the digest pass's pattern);
 *   scout_calib_gather  reads the K and V tiles that sparse_decode_attn would
 *                       read for these lists (same arguments, same meaning), one
 *                       small workgroup per tile pair (the attention's pattern).
 * `sink` is a device word (or NULL) that the kernels practically never write;
 * it only keeps the loads alive.
 */
int scout_calib_read(const void* src, size_t bytes, void* sink, void* stream);
int scout_calib_gather(const scout_problem* p, const void* k_pool, const void* v_pool, int64_t n_slots,
                       const int32_t* slot_gpu, const int32_t* n_gpu, void* sink, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SCOUT_CALIB_H */
