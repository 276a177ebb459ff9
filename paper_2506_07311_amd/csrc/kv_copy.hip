// Algorithm 1's Assign (append) and Gather as pure 16-byte data movement on gfx950.
//
// Both kernels translate a logical token position t of sequence s exactly as Algorithm 1 states:
//   b = floor(t / P), o = t mod P, slot = block_table[s][b] * P + o,
// with the slot's element offset taken from the descriptor strides (64-bit arithmetic).  One thread moves
// one 16-byte piece of one (token, kv head) row, so consecutive lanes cover a row contiguously.
#include "common.h"

namespace pa {

namespace {

constexpr int kThreads = 256;

// vec_per_head = head_dim * elem_size / 16.
__global__ __launch_bounds__(kThreads) void paged_kv_append_kernel(
    uint4* __restrict__ k_cache, uint4* __restrict__ v_cache, const uint4* __restrict__ k_new,
    const uint4* __restrict__ v_new, const int32_t* __restrict__ seq_ids, const int32_t* __restrict__ positions,
    const int32_t* __restrict__ block_table, int64_t total_vec, int32_t vec_per_head, int32_t num_kv_heads,
    int32_t max_blocks, int32_t log2_page, int64_t page_stride_v, int64_t token_stride_v, int64_t head_stride_v)
{
    const int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (idx >= total_vec) return;
    const int32_t vec = (int32_t)(idx % vec_per_head);
    const int64_t th = idx / vec_per_head;
    const int32_t h = (int32_t)(th % num_kv_heads);
    const int64_t i = th / num_kv_heads;                 // appended token
    const int32_t s = seq_ids[i];
    const int32_t t = positions[i];
    const int32_t b = t >> log2_page;                    // floor(t / P)
    const int32_t o = t & ((1 << log2_page) - 1);        // t mod P
    const int64_t page = block_table[(int64_t)s * max_blocks + b];
    const int64_t dst = page * page_stride_v + (int64_t)o * token_stride_v + (int64_t)h * head_stride_v + vec;
    if (blockIdx.y == 0)
        k_cache[dst] = k_new[idx];
    else
        v_cache[dst] = v_new[idx];
}

// The append of a decode step: one new token per sequence, token s at position seq_lens[s] - 1 (Algorithm 1, Assign,
// with seq_ids = 0 .. batch-1 and positions = seq_lens - 1 implied); a sequence of length 0 receives nothing.
__global__ __launch_bounds__(kThreads) void paged_kv_append_last_kernel(
    uint4* __restrict__ k_cache, uint4* __restrict__ v_cache, const uint4* __restrict__ k_new,
    const uint4* __restrict__ v_new, const int32_t* __restrict__ seq_lens, const int32_t* __restrict__ block_table,
    int64_t total_vec, int32_t vec_per_head, int32_t num_kv_heads, int32_t max_blocks, int32_t log2_page,
    int64_t page_stride_v, int64_t token_stride_v, int64_t head_stride_v)
{
    const int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (idx >= total_vec) return;
    const int32_t vec = (int32_t)(idx % vec_per_head);
    const int64_t th = idx / vec_per_head;
    const int32_t h = (int32_t)(th % num_kv_heads);
    const int64_t s = th / num_kv_heads;
    const int32_t t = seq_lens[s] - 1;
    if (t < 0) return;
    const int32_t b = t >> log2_page;
    const int32_t o = t & ((1 << log2_page) - 1);
    const int64_t page = block_table[s * max_blocks + b];
    const int64_t dst = page * page_stride_v + (int64_t)o * token_stride_v + (int64_t)h * head_stride_v + vec;
    if (blockIdx.y == 0)
        k_cache[dst] = k_new[idx];
    else
        v_cache[dst] = v_new[idx];
}

__global__ __launch_bounds__(kThreads) void paged_kv_gather_kernel(
    const uint4* __restrict__ k_cache, const uint4* __restrict__ v_cache, uint4* __restrict__ out_k,
    uint4* __restrict__ out_v, const int32_t* __restrict__ block_table, const int32_t* __restrict__ seq_lens,
    const int32_t* __restrict__ cu_seq_lens, int32_t vec_per_head, int32_t num_kv_heads, int32_t max_blocks,
    int32_t log2_page, int64_t page_stride_v, int64_t token_stride_v, int64_t head_stride_v)
{
    const int32_t s = blockIdx.y;
    const int32_t len = seq_lens[s];
    const int64_t vec_per_token = (int64_t)vec_per_head * num_kv_heads;
    const int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x;   // over (t, h, vec) of this sequence
    if (idx >= (int64_t)len * vec_per_token) return;
    const int32_t vec = (int32_t)(idx % vec_per_head);
    const int64_t th = idx / vec_per_head;
    const int32_t h = (int32_t)(th % num_kv_heads);
    const int32_t t = (int32_t)(th / num_kv_heads);
    const int32_t b = t >> log2_page;
    const int32_t o = t & ((1 << log2_page) - 1);
    const int64_t page = block_table[(int64_t)s * max_blocks + b];
    const int64_t src = page * page_stride_v + (int64_t)o * token_stride_v + (int64_t)h * head_stride_v + vec;
    const int64_t dst = (int64_t)cu_seq_lens[s] * vec_per_token + idx;
    if (blockIdx.z == 0)
        out_k[dst] = k_cache[src];
    else
        out_v[dst] = v_cache[src];
}

// Copy of one physical page (K and V) onto another, for copy-on-write of a shared page.
__global__ __launch_bounds__(kThreads) void paged_kv_copy_page_kernel(
    uint4* __restrict__ k_cache, uint4* __restrict__ v_cache, int64_t src_page, int64_t dst_page, int32_t page_size,
    int32_t vec_per_head, int32_t num_kv_heads, int64_t page_stride_v, int64_t token_stride_v, int64_t head_stride_v)
{
    const int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x;   // over (slot, head, vec)
    if (idx >= (int64_t)page_size * num_kv_heads * vec_per_head) return;
    const int32_t vec = (int32_t)(idx % vec_per_head);
    const int64_t th = idx / vec_per_head;
    const int32_t h = (int32_t)(th % num_kv_heads);
    const int32_t o = (int32_t)(th / num_kv_heads);
    const int64_t in_page = (int64_t)o * token_stride_v + (int64_t)h * head_stride_v + vec;
    uint4* pool = blockIdx.y == 0 ? k_cache : v_cache;
    pool[dst_page * page_stride_v + in_page] = pool[src_page * page_stride_v + in_page];
}

// Precondition check of the device-side contents (debug utility).  counts: [0] dereferenced block-table entries
// outside [0, num_pages), [1] lengths outside [0, max_blocks * P], [2] appended tokens with a sequence id or a
// position out of range.
__global__ __launch_bounds__(kThreads) void paged_debug_check_kernel(
    const int32_t* __restrict__ block_table, const int32_t* __restrict__ seq_lens, int32_t batch, int32_t max_blocks,
    int32_t num_pages, int32_t log2_page, const int32_t* __restrict__ seq_ids, const int32_t* __restrict__ positions,
    int32_t T, unsigned long long* __restrict__ counts)
{
    const int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const int64_t table_entries = (int64_t)batch * max_blocks;
    const int64_t capacity = (int64_t)max_blocks << log2_page;
    if (idx < table_entries) {
        const int32_t s = (int32_t)(idx / max_blocks);
        const int32_t b = (int32_t)(idx % max_blocks);
        const int64_t len = seq_lens[s];
        if (b == 0 && (len < 0 || len > capacity)) atomicAdd(&counts[1], 1ULL);
        const int64_t used = (min(max(len, (int64_t)0), capacity) + (1 << log2_page) - 1) >> log2_page;
        if (b < used) {
            const int32_t page = block_table[idx];
            if (page < 0 || page >= num_pages) atomicAdd(&counts[0], 1ULL);
        }
    } else if (idx - table_entries < T) {
        const int64_t i = idx - table_entries;
        const int32_t s = seq_ids[i];
        const int32_t t = positions[i];
        if (s < 0 || s >= batch || t < 0 || t >= capacity) atomicAdd(&counts[2], 1ULL);
    }
}

__global__ void paged_debug_clear_kernel(unsigned long long* counts)
{
    if (threadIdx.x < 4) counts[threadIdx.x] = 0ULL;
}

// Plain contiguous read of two buffers, 16 bytes per lane, eight loads in flight per lane: what the memory system
// delivers to the simplest possible reader, as a yardstick for the decode kernels.  Each workgroup owns one
// contiguous range of either buffer; a wave instruction covers 1 KiB.  Nothing is written (the store is never taken).
constexpr int kReadThreads = 512;
constexpr int kReadDepth = 4;
constexpr int kReadWGs = 2048;

__global__ __launch_bounds__(kReadThreads) void pa_stream_read_kernel(const uint4* __restrict__ a,
                                                                      const uint4* __restrict__ b, int64_t vec_per_wg,
                                                                      uint4* __restrict__ sink)
{
    const uint4* pa = a + (int64_t)blockIdx.x * vec_per_wg;
    const uint4* pb = b + (int64_t)blockIdx.x * vec_per_wg;
    uint4 acc = {0u, 0u, 0u, 0u};
    for (int64_t off = threadIdx.x; off < vec_per_wg; off += kReadThreads * kReadDepth) {
        uint4 t[kReadDepth], u[kReadDepth];
#pragma unroll
        for (int i = 0; i < kReadDepth; ++i) t[i] = pa[off + i * kReadThreads];
#pragma unroll
        for (int i = 0; i < kReadDepth; ++i) u[i] = pb[off + i * kReadThreads];
#pragma unroll
        for (int i = 0; i < kReadDepth; ++i) {
            acc.x ^= t[i].x ^ u[i].y;
            acc.y ^= t[i].z ^ u[i].w;
            acc.z += t[i].y + u[i].x;
            acc.w += t[i].w + u[i].z;
        }
    }
    if (acc.x == 0x12345678u && acc.y == 0x9abcdef0u && acc.z == 0x0fedcba9u && acc.w == 0x87654321u) sink[0] = acc;
}

inline int elem_bytes(pa_dtype t) { return t == PA_DTYPE_F32 ? 4 : 2; }

}  // namespace

pa_status launch_stream_read(const void* a, const void* b, size_t bytes_each, void* sink, hipStream_t stream)
{
    const size_t unit = (size_t)kReadWGs * kReadThreads * kReadDepth * sizeof(uint4);   // 64 MiB
    if (bytes_each == 0 || bytes_each % unit != 0) return PA_ERR_INVALID_ARG;
    ProfileScope prof("pa_stream_read_kernel", stream);
    hipLaunchKernelGGL(pa_stream_read_kernel, dim3(kReadWGs), dim3(kReadThreads), 0, stream, (const uint4*)a,
                       (const uint4*)b, (int64_t)(bytes_each / sizeof(uint4) / kReadWGs), (uint4*)sink);
    return launch_status();
}

pa_status launch_kv_append(const pa_kv_cache_desc* c, const void* k_new, const void* v_new, const int32_t* seq_ids,
                           const int32_t* positions, int32_t T, const int32_t* block_table, int32_t max_blocks,
                           hipStream_t stream)
{
    const CacheView v = make_view(c);
    const int eb = elem_bytes(c->dtype);
    const int32_t epv = 16 / eb;                               // elements per 16-byte vector
    const int32_t vec_per_head = c->head_dim / epv;
    const int64_t total_vec = (int64_t)T * c->num_kv_heads * vec_per_head;
    const int64_t blocks = (total_vec + kThreads - 1) / kThreads;
    if (blocks > 0x7fffffffLL) return PA_ERR_UNSUPPORTED;
    ProfileScope prof("paged_kv_append_kernel", stream);
    hipLaunchKernelGGL(paged_kv_append_kernel, dim3((uint32_t)blocks, 2, 1), dim3(kThreads), 0, stream,
                       (uint4*)c->k_cache, (uint4*)c->v_cache, (const uint4*)k_new, (const uint4*)v_new, seq_ids,
                       positions, block_table, total_vec, vec_per_head, c->num_kv_heads, max_blocks, v.log2_page,
                       c->page_stride / epv, c->token_stride / epv, c->head_stride / epv);
    return launch_status();
}

pa_status launch_kv_append_last(const pa_kv_cache_desc* c, const void* k_new, const void* v_new,
                                const int32_t* seq_lens, const int32_t* block_table, int32_t batch, int32_t max_blocks,
                                hipStream_t stream)
{
    const CacheView v = make_view(c);
    const int eb = elem_bytes(c->dtype);
    const int32_t epv = 16 / eb;
    const int32_t vec_per_head = c->head_dim / epv;
    const int64_t total_vec = (int64_t)batch * c->num_kv_heads * vec_per_head;
    const int64_t blocks = (total_vec + kThreads - 1) / kThreads;
    if (blocks > 0x7fffffffLL) return PA_ERR_UNSUPPORTED;
    if (blocks == 0) return PA_OK;
    ProfileScope prof("paged_kv_append_last_kernel", stream);
    hipLaunchKernelGGL(paged_kv_append_last_kernel, dim3((uint32_t)blocks, 2, 1), dim3(kThreads), 0, stream,
                       (uint4*)c->k_cache, (uint4*)c->v_cache, (const uint4*)k_new, (const uint4*)v_new, seq_lens,
                       block_table, total_vec, vec_per_head, c->num_kv_heads, max_blocks, v.log2_page,
                       c->page_stride / epv, c->token_stride / epv, c->head_stride / epv);
    return launch_status();
}

pa_status launch_kv_gather(const pa_kv_cache_desc* c, void* out_k, void* out_v, const int32_t* block_table,
                           const int32_t* seq_lens, const int32_t* cu_seq_lens, int32_t batch, int32_t max_blocks,
                           int32_t max_seq_len, hipStream_t stream)
{
    const CacheView v = make_view(c);
    const int eb = elem_bytes(c->dtype);
    const int32_t epv = 16 / eb;
    const int32_t vec_per_head = c->head_dim / epv;
    const int64_t per_seq = (int64_t)max_seq_len * c->num_kv_heads * vec_per_head;
    const int64_t blocks = (per_seq + kThreads - 1) / kThreads;
    if (blocks > 0x7fffffffLL || batch > 65535) return PA_ERR_UNSUPPORTED;
    if (blocks == 0) return PA_OK;
    ProfileScope prof("paged_kv_gather_kernel", stream);
    hipLaunchKernelGGL(paged_kv_gather_kernel, dim3((uint32_t)blocks, (uint32_t)batch, 2), dim3(kThreads), 0, stream,
                       (const uint4*)c->k_cache, (const uint4*)c->v_cache, (uint4*)out_k, (uint4*)out_v, block_table,
                       seq_lens, cu_seq_lens, vec_per_head, c->num_kv_heads, max_blocks, v.log2_page,
                       c->page_stride / epv, c->token_stride / epv, c->head_stride / epv);
    return launch_status();
}

pa_status launch_debug_check(const pa_kv_cache_desc* c, const int32_t* block_table, const int32_t* seq_lens,
                             int32_t batch, int32_t max_blocks, const int32_t* seq_ids, const int32_t* positions,
                             int32_t T, void* scratch, hipStream_t stream)
{
    const CacheView v = make_view(c);
    const int64_t items = (int64_t)batch * max_blocks + T;
    const int64_t blocks = (items + kThreads - 1) / kThreads;
    if (blocks > 0x7fffffffLL) return PA_ERR_UNSUPPORTED;
    unsigned long long* counts = reinterpret_cast<unsigned long long*>(scratch);
    hipLaunchKernelGGL(paged_debug_clear_kernel, dim3(1), dim3(64), 0, stream, counts);
    if (blocks > 0)
        hipLaunchKernelGGL(paged_debug_check_kernel, dim3((uint32_t)blocks), dim3(kThreads), 0, stream, block_table,
                           seq_lens, batch, max_blocks, c->num_pages, v.log2_page, seq_ids, positions, T, counts);
    return launch_status();
}

pa_status launch_kv_copy_page(const pa_kv_cache_desc* c, int32_t src_page, int32_t dst_page, hipStream_t stream)
{
    const int eb = elem_bytes(c->dtype);
    const int32_t epv = 16 / eb;
    if (c->head_dim % epv || c->page_stride % epv || c->token_stride % epv || c->head_stride % epv)
        return PA_ERR_UNSUPPORTED;
    const int32_t vec_per_head = c->head_dim / epv;
    const int64_t total = (int64_t)c->page_size * c->num_kv_heads * vec_per_head;
    const int64_t blocks = (total + kThreads - 1) / kThreads;
    if (src_page < 0 || dst_page < 0 || src_page >= c->num_pages || dst_page >= c->num_pages) return PA_ERR_INVALID_ARG;
    ProfileScope prof("paged_kv_copy_page_kernel", stream);
    hipLaunchKernelGGL(paged_kv_copy_page_kernel, dim3((uint32_t)blocks, 2, 1), dim3(kThreads), 0, stream,
                       (uint4*)c->k_cache, (uint4*)c->v_cache, (int64_t)src_page, (int64_t)dst_page, c->page_size,
                       vec_per_head, c->num_kv_heads, c->page_stride / epv, c->token_stride / epv,
                       c->head_stride / epv);
    return launch_status();
}

}  // namespace pa
