"""CPU oracle (test infrastructure only).

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this
package.  It never imports the GPU package and the GPU package never imports it.
"""
from .reference import (  # noqa: F401
    build_oracle,
    widen,
    num_threads,
    append_kv,
    page_stats,
    page_scores,
    select_pages,
    sparse_decode,
    sparse_decode_values,
    quantize_q8,
    quantize_kv,
    dequantize_q8,
    sparse_prefill_rows,
    block_mask_prefill_rows,
    paged_prefill_rows,
    chunk_prefill_rows,
    count_nonempty_tiles,
    block_sparse_speedup,
)
