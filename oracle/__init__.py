"""fp64 CPU oracle for the vertical-slash sparse-prefill path (test infrastructure only).

Only the test-suite, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py``
may import this package.  It shares no code with the GPU library.
"""
from .vs_oracle import (  # noqa: F401
    build, rope_f64, rope_bf16, index_score, select, sparse_attention, dense_attention,
    vs_aggregate, f64_to_bf16, bf16_to_f64, index_train, TRAIN_EPS,
)
