// Paged prefill on the matrix cores: support check, launch plan, dispatch over head_dim, and the head_dim 128
// kernels.
#include "prefill_mfma_impl.h"

namespace pa {

using namespace prefill;

template pa_status launch_prefill_mfma_dim<128>(const AttnArgs&, const PrefillPlan&, int64_t, int64_t, hipStream_t);
extern template pa_status launch_prefill_mfma_dim<64>(const AttnArgs&, const PrefillPlan&, int64_t, int64_t,
                                                      hipStream_t);
extern template pa_status launch_prefill_mfma_dim<256>(const AttnArgs&, const PrefillPlan&, int64_t, int64_t,
                                                       hipStream_t);

bool prefill_mfma_supported(const AttnArgs& a)
{
    if (a.dtype != PA_DTYPE_BF16 && a.dtype != PA_DTYPE_F16) return false;
    const int32_t d = a.cache.head_dim;
    if (d != 128 && d != 64 && !(d == 256 && a.cache.page_size >= 16)) return false;
    if (!(a.scale > 0.f)) return false;   // the kernel takes the max before scaling
    // the tile fetch keeps a row's byte offset inside its page (slot, KV head, piece) in 32 bits
    const int64_t in_page = (int64_t)(a.cache.page_size - 1) * a.cache.token_stride * 2 +
                            (int64_t)(a.cache.num_kv_heads - 1) * a.cache.head_stride * 2 + 512;
    if (in_page > 0xffffffffLL) return false;
    return true;
}

int32_t prefill_mfma_log2_pack(int32_t num_q_heads, int32_t num_kv_heads)
{
    // all heads of a group when the group size is a power of two (up to 16), else no packing
    const int32_t g = num_q_heads / num_kv_heads;
    int32_t lg = 0;
    while ((1 << (lg + 1)) <= g && lg < 4) ++lg;
    return (1 << lg) == g ? lg : 0;
}

pa_status launch_prefill_mfma(const AttnArgs& a, hipStream_t stream)
{
    PrefillPlan plan;
    plan.log2_pack = prefill_mfma_log2_pack(a.num_q_heads, a.cache.num_kv_heads);
    plan.chunk = a.plan.chunk;
    plan.nsplit = a.plan.nsplit;
    plan.skip_small = a.skip_small;
    plan.part_o = a.part_o;
    plan.part_lse = a.part_lse;
    plan.mods = a.mods;
    if (plan.nsplit > 1 && (plan.chunk % kBN != 0 || plan.chunk % a.cache.page_size != 0)) return PA_ERR_INVALID_ARG;
    const int64_t tiles = (((int64_t)a.max_q_len << plan.log2_pack) + kBM - 1) / kBM;
    if (tiles <= 0) return PA_OK;
    const int64_t blocks = tiles * plan.nsplit * (a.num_q_heads >> plan.log2_pack) * a.batch;
    if (blocks > 0x7fffffffLL) return PA_ERR_UNSUPPORTED;
    {
        ProfileScope prof("paged_prefill_mfma_kernel", stream);
        const pa_status st = a.cache.head_dim == 64    ? launch_prefill_mfma_dim<64>(a, plan, blocks, tiles, stream)
                             : a.cache.head_dim == 256 ? launch_prefill_mfma_dim<256>(a, plan, blocks, tiles, stream)
                                                       : launch_prefill_mfma_dim<128>(a, plan, blocks, tiles, stream);
        if (st != PA_OK || plan.nsplit == 1) return st;
    }
    return launch_merge(a, stream);
}

}  // namespace pa
