"""MI355X-native balanced block-sparse attention (the single-GPU hot path of db-SP, arXiv 2511.23113).

The product is libdbsp.so (HIP for gfx950 + a C++ host planner) behind the C ABI declared in
include/dbsp.h; this package is its thin Python binding.
"""

from .binding import (  # noqa: F401
    DBSP_EHIP,
    DBSP_EINVAL,
    DBSP_ENOMEM,
    DBSP_ESHAPE,
    DBSP_OK,
    DbspError,
    MODE_BALANCED,
    MODE_NAIVE,
    MODE_REWARD,
    MODE_ROUNDS,
    Plan,
    fit_cost_model,
    imbalance_ratio,
    load_library,
    mfma_probe,
    partition_blocks,
    partition_heads,
    plan_sparse_attn,
    plan_sparse_attn_reuse,
    ring_work,
    sparse_attn_fwd,
)
