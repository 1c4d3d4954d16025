/*
 * Test-only interface of the HOST TEST LIBRARY (libxattn_hosttest.so), which is built from the same
 * page-pool, beam-search and partition sources as libxattn.so but against a host-only stand-in for
 * the virtual-memory driver.  Nothing here is part of libxattn.so or of include/xattn.h.
 *
 * The stand-in hands out addresses from a counter with no memory behind them, counts live
 * reservations, pages and mappings, and fails on request, so that the pool's bookkeeping, its
 * roll-back paths and its background thread can be tested (and run under sanitizers) without a GPU.
 *
 * xtensor_test_fail_next(fail_op, fail_after): operation fail_op (1 reserve, 3 create, 5 map,
 *     6 unmap; -1 none) fails once after fail_after more successful calls of it.
 * xtensor_test_fake_counts: live reservations, physical pages and mappings of the stand-in.
 */
#ifndef XTENSOR_TEST_HOOKS_H_
#define XTENSOR_TEST_HOOKS_H_

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

int xtensor_test_fail_next(int fail_op, int fail_after);
int xtensor_test_fake_counts(size_t* reservations, size_t* handles, size_t* mappings);

#ifdef __cplusplus
}
#endif
#endif
