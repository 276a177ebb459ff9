"""MI355X-native attention over a paged KV cache (arXiv 2506.07311, Algorithm 1 + Sec. III-B).

The product is the C-ABI library built from ``csrc/`` (see ``include/pagedattn.h``);
``binding`` marshals torch device tensors into it, ``workloads`` draws synthetic inputs.
Nothing here computes attention on the CPU: without the HIP library the calls raise.
"""
from .binding import (  # noqa: F401
    PagedAttnError,
    library_path,
    load_library,
    paged_attention_decode,
    paged_attention_decode_mod,
    paged_attention_prefill,
    paged_attention_prefill_mod,
    paged_attention_workspace_bytes,
    paged_kv_append,
    paged_kv_gather,
    prepare_decode,
    prepare_kv_append,
    prepare_prefill,
)
