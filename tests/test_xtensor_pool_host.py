"""The xTensor page pool's bookkeeping (section 4.3: page triples, on-demand mapping, page reuse,
asynchronous pre-mapping, lazy release) and its failure handling, in the host test library: the pool's
source built against a host-only stand-in for the virtual-memory driver.  No GPU and no device memory
is involved; the GPU tests run the same pool source, in libxattn.so, on the HIP driver."""
import numpy as np
import pytest

import host_lib
import oracle
import paper_2510_14686_amd as xa
from paper_2510_14686_amd import binding as B

PAGE = xa.XTENSOR_CHUNK_BYTES
FREE, ALLOCATED, MAPPED, REUSABLE = 0, 1, 2, 3


@pytest.fixture(autouse=True)
def fake_driver():
    with host_lib.as_product_library():
        host_lib.fail_next(-1)
        base = host_lib.fake_counts()
        yield
        # every test must leave the stand-in as it found it: nothing reserved, created or mapped is leaked
        assert host_lib.fake_counts() == base
        host_lib.fail_next(-1)


def test_pool_starts_with_free_pages_and_ends_clean():
    pool = xa.xtensor_pool_create(0, 16, 1)
    assert xa.xtensor_pool_counts(pool) == (16, 0, 0, 0)
    assert host_lib.fake_counts()[1] == 16           # all physical pages exist up front
    for i in range(16):
        assert xa.xtensor_page_info(pool, i) == (FREE, 0)
    xa.xtensor_pool_destroy(pool)
    with pytest.raises(xa.XattnError):
        xa.xtensor_pool_destroy(pool)                        # not a live pool any more


def test_open_maps_only_the_used_prefix_in_scattered_order():
    pool = xa.xtensor_pool_create(0, 32, 2)
    base, rng, reused = xa.xtensor_open(pool, 7, 20 * PAGE, 3 * PAGE - 5)
    assert not reused and base % PAGE == 0
    assert xa.xtensor_pool_counts(pool) == (29, 0, 3, 0)
    ids = xa.xtensor_range_pages(rng)
    assert len(ids) == 3 and len(set(ids.tolist())) == 3
    for i in ids:
        assert xa.xtensor_page_info(pool, int(i)) == (MAPPED, 7)
    # virtual address -> page: the paper's identity, with the oracle's division
    for off in (0, PAGE - 1, PAGE, 2 * PAGE + 12345):
        idx, o = oracle.page_of(base + off, base, PAGE)
        assert idx == off // PAGE and o == off % PAGE and idx < len(ids)
    # another pool seed hands pages out in another order
    pool2 = xa.xtensor_pool_create(0, 32, 3)
    _, rng2, _ = xa.xtensor_open(pool2, 7, 20 * PAGE, 8 * PAGE)
    _, rng1b, _ = xa.xtensor_open(pool, 8, 20 * PAGE, 8 * PAGE)
    a, b = xa.xtensor_range_pages(rng2), xa.xtensor_range_pages(rng1b)
    assert not np.array_equal(np.sort(a), a) and not np.array_equal(a, b)     # scattered, seed-dependent
    for r in (rng, rng2, rng1b):
        xa.xtensor_close(r, False)
    xa.xtensor_pool_destroy(pool)
    xa.xtensor_pool_destroy(pool2)


def test_grow_maps_next_pages_on_demand():
    pool = xa.xtensor_pool_create(0, 8, 4)
    _, rng, _ = xa.xtensor_open(pool, 1, 6 * PAGE, 0)
    assert xa.xtensor_pool_counts(pool) == (8, 0, 0, 0)      # a reservation backs nothing
    assert xa.xtensor_grow(rng, 1) == 1                       # one byte needs one page
    assert xa.xtensor_grow(rng, PAGE) == 0
    before = xa.xtensor_range_pages(rng)
    assert xa.xtensor_grow(rng, 3 * PAGE + 1) == 3
    after = xa.xtensor_range_pages(rng)
    assert np.array_equal(after[:1], before) and len(after) == 4      # earlier pages stay where they were
    assert xa.xtensor_grow(rng, 2 * PAGE) == 0                # never shrinks
    with pytest.raises(xa.XattnError) as e:
        xa.xtensor_grow(rng, 7 * PAGE)                        # beyond the reservation
    assert e.value.status == B.XATTN_EINVAL
    assert xa.xtensor_pool_counts(pool) == (4, 0, 4, 0)
    xa.xtensor_close(rng, False)
    assert xa.xtensor_pool_counts(pool) == (8, 0, 0, 0)
    xa.xtensor_pool_destroy(pool)


def test_finished_request_leaves_a_reusable_set_that_a_matching_request_takes_over():
    pool = xa.xtensor_pool_create(0, 16, 5)
    base, rng, _ = xa.xtensor_open(pool, 10, 8 * PAGE, 5 * PAGE)
    pages = xa.xtensor_range_pages(rng)
    xa.xtensor_close(rng, True)
    assert xa.xtensor_pool_counts(pool) == (11, 0, 0, 5)
    for i in pages:
        assert xa.xtensor_page_info(pool, int(i))[0] == REUSABLE
    with pytest.raises(xa.XattnError):
        xa.xtensor_grow(rng, 6 * PAGE)                        # the old request's handle is closed
    maps_before = host_lib.fake_counts()[2]
    # a request of another size does not match: fresh range, fresh pages
    b2, r2, reused2 = xa.xtensor_open(pool, 11, 8 * PAGE, 4 * PAGE)
    assert not reused2 and b2 != base
    # a request of the same size takes the set over: same addresses, same pages, no map call
    maps_mid = host_lib.fake_counts()[2]
    b3, r3, reused3 = xa.xtensor_open(pool, 12, 8 * PAGE, 5 * PAGE - 100)
    assert reused3 and b3 == base
    assert np.array_equal(xa.xtensor_range_pages(r3), pages)
    assert host_lib.fake_counts()[2] == maps_mid == maps_before + 4
    for i in pages:
        assert xa.xtensor_page_info(pool, int(i)) == (MAPPED, 12)
    assert xa.xtensor_pool_counts(pool) == (7, 0, 9, 0)
    # a larger reservation than the reusable range offers is not a match
    xa.xtensor_close(r3, True)
    b4, r4, reused4 = xa.xtensor_open(pool, 13, 9 * PAGE, 5 * PAGE)
    assert not reused4
    for r in (r2, r4):
        xa.xtensor_close(r, False)
    xa.xtensor_pool_destroy(pool)                             # gives up the remaining reusable set itself


def test_reusable_sets_are_released_lazily_when_the_pool_runs_dry():
    pool = xa.xtensor_pool_create(0, 6, 6)
    _, a, _ = xa.xtensor_open(pool, 1, 4 * PAGE, 3 * PAGE)
    _, b, _ = xa.xtensor_open(pool, 2, 4 * PAGE, 2 * PAGE)
    xa.xtensor_close(a, True)
    xa.xtensor_close(b, True)
    assert xa.xtensor_pool_counts(pool) == (1, 0, 0, 5)
    _, c, reused = xa.xtensor_open(pool, 3, 6 * PAGE, 4 * PAGE)          # needs 4: 1 free + the oldest set (3)
    assert not reused
    assert xa.xtensor_pool_counts(pool) == (0, 0, 4, 2)
    with pytest.raises(xa.XattnError) as e:
        xa.xtensor_grow(c, 6 * PAGE + 1)                      # beyond the reservation: argument error
    assert e.value.status == B.XATTN_EINVAL
    assert xa.xtensor_grow(c, 6 * PAGE) == 2                  # takes the second set too
    assert xa.xtensor_pool_counts(pool) == (0, 0, 6, 0)
    _, d, _ = xa.xtensor_open(pool, 4, 2 * PAGE, 0)
    with pytest.raises(xa.XattnError) as e:
        xa.xtensor_grow(d, PAGE)                              # nothing free, nothing reusable
    assert e.value.status == B.XATTN_ENOMEM
    assert len(xa.xtensor_range_pages(d)) == 0 and len(xa.xtensor_range_pages(c)) == 6
    xa.xtensor_close(c, False)
    assert xa.xtensor_grow(d, PAGE) == 1
    xa.xtensor_close(d, False)
    xa.xtensor_pool_destroy(pool)


@pytest.mark.parametrize("fail_op,fail_after", [(5, 0), (5, 2), (1, 0)])
def test_failed_open_rolls_everything_back(fail_op, fail_after):
    pool = xa.xtensor_pool_create(0, 8, 7)
    host_lib.fail_next(fail_op, fail_after)    # map (5) or reserve (1) fails once
    with pytest.raises(xa.XattnError):
        xa.xtensor_open(pool, 1, 8 * PAGE, 4 * PAGE)
    assert xa.xtensor_pool_counts(pool) == (8, 0, 0, 0)       # no page stuck in Allocated or Mapped
    res, handles, maps = host_lib.fake_counts()
    assert maps == 0 and handles == 8
    _, r, _ = xa.xtensor_open(pool, 1, 8 * PAGE, 4 * PAGE)    # and the pool still works
    xa.xtensor_close(r, False)
    xa.xtensor_pool_destroy(pool)


def test_failed_grow_keeps_what_the_range_had():
    pool = xa.xtensor_pool_create(0, 8, 8)
    _, r, _ = xa.xtensor_open(pool, 1, 8 * PAGE, 2 * PAGE)
    host_lib.fail_next(5, 1)                   # second map of the grow fails
    with pytest.raises(xa.XattnError):
        xa.xtensor_grow(r, 6 * PAGE)
    assert len(xa.xtensor_range_pages(r)) == 3                # two it had, one it got before the failure
    assert xa.xtensor_pool_counts(pool) == (5, 0, 3, 0)
    assert xa.xtensor_grow(r, 6 * PAGE) == 3
    xa.xtensor_close(r, False)
    xa.xtensor_pool_destroy(pool)


def test_pool_creation_failure_releases_the_pages_already_created():
    host_lib.fail_next(3, 5)                   # sixth page creation fails
    with pytest.raises(xa.XattnError) as e:
        xa.xtensor_pool_create(0, 16, 9)
    assert e.value.status == B.XATTN_ENOMEM
    assert host_lib.fake_counts()[1] == 0


def test_asynchronous_premapping():
    pool = xa.xtensor_pool_create(0, 8, 10)
    _, r, _ = xa.xtensor_open(pool, 1, 8 * PAGE, 1 * PAGE)
    xa.xtensor_premap_async(r, 3 * PAGE)                      # "while the current token is decoded"
    xa.xtensor_premap_async(r, 5 * PAGE)
    xa.xtensor_premap_wait(r)
    assert len(xa.xtensor_range_pages(r)) == 5
    assert xa.xtensor_grow(r, 5 * PAGE) == 0                  # the step that needs the pages finds them mapped
    _, r2, _ = xa.xtensor_open(pool, 2, 8 * PAGE, 3 * PAGE)
    xa.xtensor_premap_async(r, 6 * PAGE)                      # pool has no page left for it
    with pytest.raises(xa.XattnError) as e:
        xa.xtensor_premap_wait(r)
    assert e.value.status == B.XATTN_ENOMEM
    xa.xtensor_premap_wait(r)                                 # the failure is reported once
    with pytest.raises(xa.XattnError):
        xa.xtensor_premap_async(r, 9 * PAGE)                  # beyond the reservation: refused at once
    xa.xtensor_premap_async(r2, 3 * PAGE)
    xa.xtensor_close(r2, False)                               # close waits for the pending request
    xa.xtensor_close(r, False)
    xa.xtensor_pool_destroy(pool)


def test_pool_refuses_to_die_with_open_ranges_and_rejects_bad_handles():
    pool = xa.xtensor_pool_create(0, 4, 11)
    _, r, _ = xa.xtensor_open(pool, 1, 2 * PAGE, PAGE)
    with pytest.raises(xa.XattnError) as e:
        xa.xtensor_pool_destroy(pool)
    assert e.value.status == B.XATTN_EINVAL
    for bad in (lambda: xa.xtensor_open(pool, 1, 0, 0), lambda: xa.xtensor_open(pool, 1, PAGE, 2 * PAGE),
                lambda: xa.xtensor_open(12345, 1, PAGE, 0), lambda: xa.xtensor_grow(12345, PAGE),
                lambda: xa.xtensor_close(0, False), lambda: xa.xtensor_page_info(pool, 4),
                lambda: xa.xtensor_pool_create(0, 0, 1), lambda: xa.xtensor_pool_create(3, 4, 1)):
        with pytest.raises(xa.XattnError):
            bad()
    xa.xtensor_close(r, False)
    with pytest.raises(xa.XattnError):
        xa.xtensor_close(r, False)                            # double close
    xa.xtensor_pool_destroy(pool)
