"""MI355X-native hot path of APB-V (arXiv 2601.21444): KV compression and fused host attention.

The compute lives in ``libapbv.so`` (hand-written gfx950 HIP kernels behind the C ABI declared in
``include/apbv.h``); this package only marshals arguments.  Importing the package does not load the
library; the first call does, and raises if it has not been built.
"""
from .binding import (  # noqa: F401
    ApbvError,
    ApbvAttentionItem,
    ApbvTensor,
    apbv_compress_kv,
    apbv_compress_kv_noalloc,
    NOALLOC_MAX_WORKSPACE_BYTES,
    apbv_compress_reduced_workspace_bytes,
    apbv_compress_workspace_bytes,
    apbv_host_attention,
    apbv_host_attention_group,
    apbv_merge_lse,
    apbv_query_attention,
    apbv_query_attention_workspace_bytes,
    apbv_version,
    load_library,
    status_string,
    tensor_view,
)
