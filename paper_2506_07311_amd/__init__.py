"""MI355X-native attention over a paged KV cache (arXiv 2506.07311, Algorithm 1 + Sec. III-B).

The product is the C-ABI library built from ``csrc/`` (see ``include/pagedattn.h``);
``binding`` marshals torch device tensors into it, ``workloads`` draws synthetic inputs.
Nothing here computes attention on the CPU: without the HIP library the calls raise.
"""
from .binding import (  # noqa: F401
    PA_GROW_EXACT,
    PA_GROW_POW2,
    PA_MOD_PREFIX_LM,
    PagedAttnError,
    library_path,
    load_library,
    pa_debug_check,
    pa_pool_create,
    pa_pool_destroy,
    pa_pool_get_row,
    pa_pool_make_writable,
    pa_pool_num_blocks,
    pa_pool_num_free,
    pa_pool_refcount,
    pa_pool_release,
    pa_pool_reserve,
    pa_pool_set_growth,
    pa_pool_share_prefix,
    pa_set_option,
    paged_attention_decode,
    paged_attention_decode_mod,
    paged_attention_decode_static,
    paged_attention_prefill,
    paged_attention_prefill_mod,
    paged_attention_workspace_bytes,
    paged_decode_step,
    paged_kv_append,
    paged_kv_gather,
    prepare_decode,
    prepare_decode_step,
    prepare_kv_append,
    prepare_prefill,
    prefix_lm_data,
)
