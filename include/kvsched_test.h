/*
 * kvsched_test.h -- TEST HOOKS of libkvsched.so.  Not part of the product
 * interface: no stability promise, nothing here is needed to use the library,
 * and the Python binding does not expose it.
 *
 * Each hook runs, on the host, the very integer helper the kernels use on the
 * device (the helpers are compiled for both), so that the tests can compare
 * them with plain arithmetic on machines without a GPU.
 */
#ifndef KVSCHED_TEST_H
#define KVSCHED_TEST_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Smallest p >= 0 with tau0 * 2^p >= x, for 1 <= x, tau0 <= 2^30. */
uint32_t kvs_host_class_index(uint32_t x, uint32_t tau0);

/* Number of slices of lad[0 .. n_lv) below x (n_lv when no slice covers x), 1 <= n_lv <= 64. */
uint32_t kvs_host_ladder_level(uint32_t x, const uint32_t *lad, uint32_t n_lv);

/* floor(x / d) through the multiply-high constant, for x < 2^31, d >= 1. */
uint32_t kvs_host_div(uint32_t x, uint32_t d);

/* Largest k with Peak(k, tau, s) <= M, 0 when none. */
uint64_t kvs_host_kstar(uint64_t tau, uint64_t s, uint64_t M);

/* sum_{i < n} floor(i * tau / k). */
uint64_t kvs_host_floor_sum(uint64_t n, uint64_t k, uint64_t tau);

/* Work units into which kvs_opt_perm cuts the orders of n jobs (0 for n outside 1..10). */
uint32_t kvs_host_perm_units(int32_t n);

/* Smallest flow time over the orders of work unit `unit`; -1 for bad arguments. */
int64_t kvs_host_best_of_unit(uint32_t unit, int32_t n, const int32_t *o, int64_t s, int64_t M);

#ifdef __cplusplus
}
#endif
#endif /* KVSCHED_TEST_H */
