"""MI355X-native decode attention over xTensor-style KV memory (libxattn.so + ctypes binding)."""
from .binding import (XATTN_CFG_MIN_PIECE_TOKENS, XATTN_CFG_MLA_LAYOUT, XATTN_CFG_PATH, XATTN_CFG_PIECES, XATTN_CFG_PV_MODE, XATTN_CFG_TIMING, XATTN_CFG_XCD_SKEW, XTENSOR_CHUNK_BYTES, XattnError,  # noqa: F401
                      load_library, xattn_configure, xattn_decode, xattn_decode_noalloc, xattn_last_error, xattn_set_workspace, xattn_timing_read,
                      xattn_workspace_bytes, xtensor_chunk_order, xtensor_download, xtensor_map,
                      xtensor_physical_view, xtensor_unmap, xtensor_upload)
from .binding import (XTENSOR_PAGE_ALLOCATED, XTENSOR_PAGE_FREE, XTENSOR_PAGE_MAPPED, XTENSOR_PAGE_REUSABLE,  # noqa: F401
                      xattn_mla_decode, xattn_mla_workspace_bytes, xattn_write_kvcache, xtensor_close, xtensor_grow, xtensor_open, xtensor_page_info,
                      xtensor_pool_counts, xtensor_pool_create, xtensor_pool_destroy, xtensor_premap_async,
                      xtensor_premap_wait, xtensor_range_pages)
from .binding import XBEAM_CHECK_INPUT, XBEAM_FULL_SORT, xbeam_select  # noqa: F401
from .kvstore import KVStore  # noqa: F401
