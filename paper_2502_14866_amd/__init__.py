"""MI355X-native unified block-sparse attention path of LServe (arxiv 2502.14866).

The product is the C-ABI library `liblserve.so` (include/lserve.h).  This package is a thin
ctypes binding with the same entry-point names; it only marshals arguments.  PyTorch supplies
device memory and streams.  There is no CPU fallback: if the library has not been built the
calls raise.
"""
from .binding import (  # noqa: F401
    LSERVE_CALL_BUILD_PAGE_STATS,
    LSERVE_CALL_SELECT_PAGES,
    LSERVE_CALL_SPARSE_DECODE,
    LSERVE_CALL_SPARSE_PREFILL,
    AttnDesc,
    LserveError,
    PagedKV,
    library_path,
    load_library,
    BlockMask,
    lserve_append_kv,
    lserve_masked_prefill_workspace_bytes,
    lserve_sparse_prefill_masked,
    lserve_paged_prefill_workspace_bytes,
    lserve_sparse_prefill_paged,
    lserve_sparse_prefill_chunk,
    lserve_build_page_stats,
    lserve_init,
    lserve_last_hip_error,
    lserve_probe_decode_read,
    lserve_select_pages,
    lserve_sparse_decode,
    lserve_sparse_decode_noalloc,
    lserve_sparse_prefill,
    lserve_strerror,
    lserve_workspace_bytes,
)
