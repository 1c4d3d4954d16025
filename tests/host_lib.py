"""The host test library (libxattn_hosttest.so): the page pool, beam search and partition arithmetic of
the product, built with g++ against a host-only stand-in for the virtual-memory driver.  Test
infrastructure: the stand-in and its hooks exist only in this library, never in libxattn.so."""
import contextlib
import ctypes

import numpy as np

from paper_2510_14686_amd import binding
from paper_2510_14686_amd import build as xbuild

POOL_ENTRY_POINTS = ["xattn_last_error", "xtensor_pool_create", "xtensor_pool_destroy", "xtensor_pool_counts",
                     "xtensor_page_info", "xtensor_open", "xtensor_grow", "xtensor_premap_async",
                     "xtensor_premap_wait", "xtensor_close", "xtensor_range_pages", "xbeam_select"]
_lib = None


def load(path=None):
    global _lib
    if _lib is not None and path is None:
        return _lib
    lib = binding.bind(ctypes.CDLL(path or xbuild.build_hosttest()), required=POOL_ENTRY_POINTS)
    i32, sz, vp = ctypes.c_int, ctypes.c_size_t, ctypes.c_void_p
    lib.xtensor_test_fail_next.restype = i32
    lib.xtensor_test_fail_next.argtypes = [i32, i32]
    lib.xtensor_test_fake_counts.restype = i32
    lib.xtensor_test_fake_counts.argtypes = [ctypes.POINTER(sz)] * 3
    for name, args in (("xattn_test_plan", [vp, i32, i32, i32, i32, i32, vp]),
                       ("xattn_test_piece_bounds", [vp, i32, i32, i32, i32, i32, vp]),
                       ("xattn_test_piece_of", [vp, i32, i32, i32, i32, i32, i32]),
                       ("xattn_test_piece_segments", [vp, i32, i32, i32, i32, i32, i32, vp, i32]),
                       ("xattn_test_meta", [vp, i32, i32, i32, i32, i32, vp])):
        fn = getattr(lib, name)
        fn.restype = i32
        fn.argtypes = args
    if path is None:
        _lib = lib
    return lib


@contextlib.contextmanager
def as_product_library():
    """While active, the package's wrappers (xa.xtensor_open, xa.xbeam_select, ...) call the host test
    library instead of libxattn.so."""
    saved = binding._lib
    binding._lib = load()
    try:
        yield binding._lib
    finally:
        binding._lib = saved


def fail_next(fail_op=-1, fail_after=0):
    """Operation fail_op of the stand-in driver (1 reserve, 3 create, 5 map, 6 unmap) fails once after
    fail_after more successful calls."""
    assert load().xtensor_test_fail_next(fail_op, fail_after) == 0


def fake_counts():
    """(live reservations, live pages, live mappings) of the stand-in driver."""
    a, b, c = ctypes.c_size_t(), ctypes.c_size_t(), ctypes.c_size_t()
    assert load().xtensor_test_fake_counts(ctypes.byref(a), ctypes.byref(b), ctypes.byref(c)) == 0
    return int(a.value), int(b.value), int(c.value)


# ----------------------------------------------------------------------------- partition
def _lens(kv_lens):
    return np.ascontiguousarray(kv_lens, dtype=np.int32)


def plan(kv_lens, n_pieces, min_piece, seg_cost, skew=0):
    """(N, pieces in use); N = -1 and pieces = -1 beyond the 32-bit limit."""
    kv = _lens(kv_lens)
    total = ctypes.c_int32()
    n = load().xattn_test_plan(kv.ctypes.data, len(kv), n_pieces, min_piece, seg_cost, skew, ctypes.addressof(total))
    return int(total.value), n


def piece_bounds(kv_lens, n_pieces, min_piece, seg_cost, skew=0):
    kv = _lens(kv_lens)
    out = np.zeros(n_pieces + 2, np.int32)
    n = load().xattn_test_piece_bounds(kv.ctypes.data, len(kv), n_pieces, min_piece, seg_cost, skew, out.ctypes.data)
    assert n >= 1
    return out[:n + 1].copy()


def piece_of(kv_lens, n_pieces, min_piece, seg_cost, position, skew=0):
    kv = _lens(kv_lens)
    return load().xattn_test_piece_of(kv.ctypes.data, len(kv), n_pieces, min_piece, seg_cost, skew, position)


def piece_segments(kv_lens, n_pieces, min_piece, seg_cost, p, max_segs=8192, skew=0):
    """Rows (b, j0, j1, slot, whole) of piece p."""
    kv = _lens(kv_lens)
    out = np.zeros((max_segs, 5), np.int32)
    n = load().xattn_test_piece_segments(kv.ctypes.data, len(kv), n_pieces, min_piece, seg_cost, skew, p, out.ctypes.data, max_segs)
    assert 0 <= n <= max_segs
    return out[:n].copy()


def meta(kv_lens, n_pieces, min_piece, seg_cost, skew=0):
    """int32 [batch, 2]: (first partial slot, number of segments) per sequence."""
    kv = _lens(kv_lens)
    out = np.zeros((len(kv), 2), np.int32)
    assert load().xattn_test_meta(kv.ctypes.data, len(kv), n_pieces, min_piece, seg_cost, skew, out.ctypes.data) == 0
    return out
