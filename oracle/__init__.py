"""CPU oracle for the sparse-gradient encode + aggregate path (TEST INFRASTRUCTURE ONLY).

`zen_ref.c` is the plain single-threaded definition; this module compiles it with gcc and wraps it
with ctypes + numpy.  Nothing here imports or is imported by the HIP package.  Only the tests, the
smoke check and the benchmark's cpu_baseline leg may use it.
"""
from .zen_ref import (  # noqa: F401
    build,
    lib,
    use_library,
    hash32,
    hash_many,
    owner_table,
    nonzero,
    partition,
    gather,
    encode,
    bitmap_layout,
    bitmap_encode,
    bitmap_decode,
    aggregate,
    member_mask,
    densify,
    pull_apply,
    hash_slots,
    hierarchical_hash,
    overlap_ratio,
    union_sizes,
    skewness,
    time_balanced_parallelism,
    time_hierarchical_centralization,
    topk_threshold,
    threshold_apply,
    format_bytes,
    nonzero_blocks,
    imbalance,
)
