"""CPU oracle for the APB-V host-share hot path.  TEST INFRASTRUCTURE ONLY.

Nothing in the product path (the HIP library, its Python binding) may import this package; it is
used by ``tests/``, by ``__graft_entry__.smoke()`` and by the ``cpu_baseline`` leg of ``bench.py``.
"""
from .apbv_oracle import (  # noqa: F401
    bf16_bits_to_f64,
    pooled_query,
    importance_scores,
    importance_scores_max,
    importance_scores_softmax_sum,
    logit_matrix,
    arg_top,
    compress_kv,
    make_passing_block,
    visibility_mask,
    host_attention,
    merge_lse,
)
