"""fp64 CPU oracle for attention over a paged KV cache (test infrastructure only).

Only the tests, the smoke check and the benchmark's cpu_baseline leg may import
this package.  It never imports the HIP library or its Python binding.
"""
from .ta_oracle import (  # noqa: F401
    Geometry,
    append_prefill,
    append_prefill_fp8,
    attend_rows,
    build,
    kv_append,
    kv_append_fp8,
    kv_page_evict,
    kv_page_restore,
    num_threads,
    paged_decode,
    paged_decode_fp8,
    quantise_e4m3,
    row_probs,
    widen_e4m3,
)
