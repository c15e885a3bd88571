/* linear_kv_diag.h -- tuning, introspection and measurement aids of the LineAR decode library.
 *
 * None of these calls is part of the method's boundary (include/linear_kv.h): they expose the
 * decode kernel's launch shape for sweeps and host-side tests, and the yardstick kernels the
 * benchmark measures the decode step against.  Conventions as in linear_kv.h.
 */
#ifndef LINEAR_KV_DIAG_H
#define LINEAR_KV_DIAG_H

#include "linear_kv.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Tuning of the decode kernel's launch shape (defaults are chosen per configuration).
 *   groups_per_wave : 1..16 row groups (one wave-wide 1 KiB load each) a wavefront should
 *                     take; fewer groups per wavefront = more wavefronts per pair; 0 = default;
 *   n_split         : workgroups the keys of one pair are split over, 1..64 (a split step
 *                     is two launches: partials, then merge); lowered for steps with too
 *                     few keys to give every workgroup one, raised for steps whose keys
 *                     would not fit; 0 = automatic. */
LINEAR_API int linear_set_tuning(linear_kv_t* kv, int32_t groups_per_wave, int32_t n_split);

/* Host-only introspection of the decode kernel's launch shape for a step that sees
 * `cached_keys` keys already in the cache (the appended one not counted), under the given
 * tuning (0 = default): shape[0] = workgroups per (sequence, head) pair, shape[1] = cached
 * keys per workgroup, shape[2] = wavefronts per workgroup, shape[3] = row groups a wavefront
 * holds, shape[4] = the wavefront of the last workgroup that takes the appended token,
 * shape[5] = keys per row group (one wave-wide 1 KiB load).  HOST pointers, no device work. */
LINEAR_API int linear_plan_shape(const linear_cfg_t* cfg, int32_t cached_keys, int32_t groups_per_wave,
                      int32_t n_split, int32_t* shape);

/* Measurement aids (no part of the method): what the decode step is measured against.
 * linear_probe_stream enqueues, for each of n_layers layers, one kernel that only reads rows
 * [0, rows) of every pair of that layer's K and V cache ([n_pairs, pitch_rows, row_bytes] bytes
 * each) -- the bytes a decode step over `rows` cached keys reads -- with no arithmetic and no
 * store: a plain streaming read launched exactly like the decode steps (one launch per layer,
 * back to back).  k_cache, v_cache: HOST arrays of n_layers DEVICE pointers.
 * linear_probe_empty enqueues `launches` kernels of `groups` workgroups of `threads` threads that
 * do nothing: the cost of a launch as such. */
LINEAR_API int linear_probe_stream(const void* const* k_cache, const void* const* v_cache, int32_t n_layers,
                        int32_t n_pairs, int32_t rows, int32_t pitch_rows, int32_t row_bytes, void* stream);
LINEAR_API int linear_probe_empty(int32_t launches, int32_t groups, int32_t threads, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* LINEAR_KV_DIAG_H */
