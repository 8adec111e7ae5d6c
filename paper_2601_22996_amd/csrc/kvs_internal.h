/*
 * kvs_internal.h -- calls between the library's own source files; not part of
 * the interface (kvsched.h) and not exported.
 */
#ifndef KVS_INTERNAL_H
#define KVS_INTERNAL_H

#include <stdint.h>

#include "kvsched.h"

/*
 * Algorithm 2 with dynamic refill at the points pts[0 .. n_pts) (tau0, sched, k; mode is not
 * looked at), results into the output rows rows[j].  The caller has checked the arguments.
 */
__attribute__((visibility("hidden"))) int32_t kvs_gbad_run(const kvs_jobs_t *jobs, const kvs_point_t *pts,
                                                           const int32_t *rows, int32_t n_pts, int64_t *peak,
                                                           uint8_t *feasible, int64_t *flow, int64_t *job_steps,
                                                           void *stream);

#endif /* KVS_INTERNAL_H */
