// Paged decode on the matrix cores: support check, dispatch over head_dim, and the head_dim 128 kernels.
#include <atomic>
#include <mutex>

#include "decode_mfma_impl.h"

// Arrival counters of the one-launch decode kernel when several workgroups share a (sequence, KV head): they live
// in the library's device image, so they are zero when the library is loaded and every kernel leaves them zero
// (the workgroup that arrives last resets its counter) -- no call ever has to clear them.  Each call takes the
// next window of the array, so that calls in flight on different streams count in different places; a window
// comes round again after kArriveSlots / kShortMaxUnits calls.  In host code this name is only a handle for
// hipGetSymbolAddress; kernels receive the address that call returns.
constexpr int32_t kArriveSlots = 65536;
static __device__ uint32_t arrive_counters[kArriveSlots];

namespace pa {

namespace {

std::mutex g_arrive_mutex;
uint32_t* g_arrive_ptr[64] = {};
std::atomic<uint32_t> g_arrive_cursor{0};

// `units` counters (all zero) for one launch on the current device.
pa_status arrival_window(int32_t units, uint32_t** out)
{
    if (units < 1 || units > kShortMaxUnits) return PA_ERR_INVALID_ARG;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return PA_ERR_HIP;
    uint32_t* base;
    {
        std::lock_guard<std::mutex> lock(g_arrive_mutex);
        if (!g_arrive_ptr[dev]) {
            void* p = nullptr;
            if (hipGetSymbolAddress(&p, HIP_SYMBOL(arrive_counters)) != hipSuccess || !p) return PA_ERR_HIP;
            g_arrive_ptr[dev] = static_cast<uint32_t*>(p);
        }
        base = g_arrive_ptr[dev];
    }
    const uint32_t window = g_arrive_cursor.fetch_add(1, std::memory_order_relaxed) % (kArriveSlots / kShortMaxUnits);
    *out = base + (size_t)window * kShortMaxUnits;
    return PA_OK;
}

}  // namespace

template void launch_decode_mfma_dim<128>(const AttnArgs&, hipStream_t);
extern template void launch_decode_mfma_dim<64>(const AttnArgs&, hipStream_t);
extern template void launch_decode_mfma_dim<256>(const AttnArgs&, hipStream_t);
template void launch_decode_short_dim<128>(const AttnArgs&, hipStream_t);
extern template void launch_decode_short_dim<64>(const AttnArgs&, hipStream_t);
extern template void launch_decode_short_dim<256>(const AttnArgs&, hipStream_t);

int32_t decode_mfma_heads_per_wg(int32_t num_kv_heads, int32_t head_dim)
{
    // head_dim 256 holds two tiles in about 250 registers: four waves per workgroup keep that inside the budget
    // of a 256-thread launch
    if (head_dim <= 128 && num_kv_heads % 8 == 0) return 8;
    return num_kv_heads % 4 == 0 ? 4 : num_kv_heads % 2 == 0 ? 2 : 1;
}

bool decode_mfma_supported(const AttnArgs& a)
{
    if (a.dtype != PA_DTYPE_BF16 && a.dtype != PA_DTYPE_F16) return false;
    const int32_t d = a.cache.head_dim;
    if (d != 64 && d != 128 && d != 256) return false;
    const int32_t G = a.num_q_heads / a.cache.num_kv_heads;
    if (G > 16 * 64) return false;                     // one grid slice per 16 heads of a group
    if (a.cache.num_kv_heads > 65535 * 8) return false;
    // per-lane byte offsets inside a 16-key block are kept in 32 bits
    if (a.cache.token_stride * 2 * 16 + a.cache.head_stride * 2 > 0x7fffffffLL) return false;
    // tile counts are kept in 32 bits (tiles hold 16 keys at head_dim 256, 32 otherwise)
    if ((int64_t)a.batch * ((a.max_seq_len + 15) / 16) > 0x7fffffffLL) return false;
    return true;
}

bool decode_short_supported(const AttnArgs& a)
{
    // one workgroup per (sequence, KV head, slice of 16 heads): the grid's y and z extents are 16-bit
    const int32_t G = a.num_q_heads / a.cache.num_kv_heads;
    return decode_mfma_supported(a) && !a.cu_q_lens && a.cache.num_kv_heads <= 65535 && (G + 15) / 16 <= 65535;
}

pa_status launch_decode_short(const AttnArgs& args, hipStream_t stream)
{
    AttnArgs a = args;
    a.short_arrive = nullptr;
    if (a.short_nsplit > 1) {
        const int32_t G = a.num_q_heads / a.cache.num_kv_heads;
        const int64_t units = (int64_t)a.batch * a.cache.num_kv_heads * ((G + 15) / 16);
        if (units > kShortMaxUnits || a.short_nsplit > kShortMaxSplit || !a.short_part) return PA_ERR_INVALID_ARG;
        const pa_status st = arrival_window((int32_t)units, &a.short_arrive);
        if (st != PA_OK) return st;
    }
    ProfileScope prof("paged_decode_short_kernel", stream);
    switch (a.cache.head_dim) {
        case 64: launch_decode_short_dim<64>(a, stream); break;
        case 128: launch_decode_short_dim<128>(a, stream); break;
        case 256: launch_decode_short_dim<256>(a, stream); break;
        default: return PA_ERR_UNSUPPORTED;
    }
    return launch_status();
}

pa_status launch_decode_mfma(const AttnArgs& a, hipStream_t stream)
{
    ProfileScope prof("paged_decode_mfma_kernel", stream);
    switch (a.cache.head_dim) {
        case 64: launch_decode_mfma_dim<64>(a, stream); break;
        case 128: launch_decode_mfma_dim<128>(a, stream); break;
        case 256: launch_decode_mfma_dim<256>(a, stream); break;
        default: return PA_ERR_UNSUPPORTED;
    }
    return launch_status();
}

}  // namespace pa
