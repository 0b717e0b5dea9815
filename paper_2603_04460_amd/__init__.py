"""MI355X-native vertical-slash sparse prefill (VSPrefill inference hot path).

``binding`` wraps the C ABI of ``libvsprefill.so`` one-to-one (argument marshalling only).  The library is loaded on first use and a
missing build raises instead of falling back to anything else.
"""
from . import binding  # noqa: F401
from .binding import (  # noqa: F401
    VsError, IndexerWeights, Budget, rope_apply, index_score, index_score_workspace, select_budget,
    select_budget_workspace, sparse_prefill, sparse_prefill_static, sparse_prefill_workspace, sparse_prefill_tiles, sparse_prefill_counters, validate_lists, dense_prefill, aggregate, aggregate_workspace,
    index_train_step, index_train_workspace, version, exported_symbols, library_path,
)
