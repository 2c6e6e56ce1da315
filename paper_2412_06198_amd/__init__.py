"""MI355X (gfx950) dynamic sparse prefill attention: Python binding of the C ABI in include/sa.h."""
from .binding import (  # noqa: F401
    SA_BLOCK_CLUSTER, SA_INTERVAL_SLASH, SA_PATTERN_AUTO, SA_TRIANGULAR,
    SaConfig, SaError, SaIndex, SaScores, Session, library, sa_build_index, sa_create,
    sa_default_budgets, sa_destroy, sa_estimate_and_index, sa_estimate_patterns, sa_index_bytes, sa_last_error,
    sa_scores_bytes, sa_search_patterns, sa_search_scratch_bytes, sa_set_workspace, sa_sparse_decode, sa_sparse_decode_static, sa_sparse_prefill,
    sa_sparse_prefill_counted, sa_version, sa_workspace_bytes,
)
