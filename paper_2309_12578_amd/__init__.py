"""MI355X (gfx950) implementation of SPION's layer-wise sparse attention hot path.

The product is the HIP library ``libspion.so`` (C ABI in ``include/spion.h``); this package is a
thin ctypes binding around it plus the FLOP / byte accounting used by the benchmark.  There is no
CPU fallback: every call fails loudly if the library is missing.
"""
from .binding import (  # noqa: F401
    SPION_BF16, SPION_F32, SPION_T_ABS, SPION_T_MEAN_KSTD, SPION_T_QUANTILE,
    SPION_PATTERN_NO_FILL, SPION_PATTERN_POOL_ONLY, SPION_PATTERN_FROM_POOL, SPION_ATTN_PAPER_DENOM, SPION_ATTN_BWD_QUERY_SIDE_ONLY,
    SPION_ATTN_BWD_KEY_SIDE_ONLY, SpionError, Pattern,
    lib_path, load, spion_version, spion_strerror,
    spion_pattern_workspace_bytes, spion_pattern, spion_pattern_static, spion_attn_workspace_bytes,
    spion_attn_fwd, spion_attn_bwd, generate_pattern, attn_fwd, attn_bwd,
    spion_score_mean, spion_frobenius_workspace_bytes, spion_frobenius_distance, score_mean,
    frobenius_distance, spion_index_check, index_is_well_formed, spion_copy_yardstick,
)
from .autograd import sparse_attention  # noqa: E402,F401
from .sublayer import SparseMHA  # noqa: E402,F401
