// Shared host/device helpers of the gfx950 paged-attention library (internal header).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/pagedattn.h"
#include "../../include/pagedattn_mods.h"

namespace pa {

// ---------------------------------------------------------------------------------------------
// Device-side view of the pools and the block table (Algorithm 1's operands).
// ---------------------------------------------------------------------------------------------
struct CacheView {
    const void* k;
    const void* v;
    int64_t page_stride;   // elements
    int64_t token_stride;  // elements
    int64_t head_stride;   // elements
    int32_t page_size;     // P (power of two)
    int32_t log2_page;     // log2(P)
    int32_t num_kv_heads;
    int32_t head_dim;
};

inline CacheView make_view(const pa_kv_cache_desc* c)
{
    CacheView v;
    v.k = c->k_cache;
    v.v = c->v_cache;
    v.page_stride = c->page_stride;
    v.token_stride = c->token_stride;
    v.head_stride = c->head_stride;
    v.page_size = c->page_size;
    int l = 0;
    while ((1 << l) < c->page_size) ++l;
    v.log2_page = l;
    v.num_kv_heads = c->num_kv_heads;
    v.head_dim = c->head_dim;
    return v;
}

// Split-KV plan shared by the decode kernels and the merge kernel.  A sequence of length len is cut
// into ceil(len / chunk) chunks of `chunk` tokens; partial c of (row, head) lives at
// part_o[((row * Hq + head) * nsplit + c) * d .. + d) (fp32, normalised) and
// part_lse[(row * Hq + head) * nsplit + c] (natural-log LSE of the chunk's scaled scores).
struct SplitPlan {
    int32_t chunk;   // tokens per chunk; a multiple of max(P, 32)
    int32_t nsplit;  // grid extent = ceil(max_seq_len / chunk)
};

constexpr int32_t kMinChunk = 256;     // smallest chunk the planner will pick
constexpr int32_t kMaxSplits = 64;     // bound of nsplit used to size the workspace
constexpr int32_t kMaxDecodeWGs = 2048;  // bound of the tile-stream decode grid used to size the workspace

// ---------------------------------------------------------------------------------------------
// Launch bookkeeping: error capture and optional per-kernel event timing.
// ---------------------------------------------------------------------------------------------
void profile_begin(const char* kernel, hipStream_t stream);
void profile_end(hipStream_t stream);

struct ProfileScope {
    hipStream_t s;
    ProfileScope(const char* kernel, hipStream_t stream) : s(stream) { profile_begin(kernel, stream); }
    ~ProfileScope() { profile_end(s); }
};

// Host-checkable properties of a pool descriptor (pointers, dtype, sizes, strides, alignment), shared by every
// entry point that takes one.
pa_status check_cache(const pa_kv_cache_desc* c);

inline pa_status launch_status()
{
    return hipGetLastError() == hipSuccess ? PA_OK : PA_ERR_HIP;
}


// ---------------------------------------------------------------------------------------------
// Kernel launchers (each defined in its own .hip file).  All take validated arguments.
// ---------------------------------------------------------------------------------------------
pa_status launch_kv_append(const pa_kv_cache_desc* c, const void* k_new, const void* v_new, const int32_t* seq_ids,
                           const int32_t* positions, int32_t T, const int32_t* block_table, int32_t max_blocks,
                           hipStream_t stream);
pa_status launch_kv_append_last(const pa_kv_cache_desc* c, const void* k_new, const void* v_new,
                                const int32_t* seq_lens, const int32_t* block_table, int32_t batch, int32_t max_blocks,
                                hipStream_t stream);
pa_status launch_kv_gather(const pa_kv_cache_desc* c, void* out_k, void* out_v, const int32_t* block_table,
                           const int32_t* seq_lens, const int32_t* cu_seq_lens, int32_t batch, int32_t max_blocks,
                           int32_t max_seq_len, hipStream_t stream);

pa_status launch_debug_check(const pa_kv_cache_desc* c, const int32_t* block_table, const int32_t* seq_lens,
                             int32_t batch, int32_t max_blocks, const int32_t* seq_ids, const int32_t* positions,
                             int32_t T, void* scratch, hipStream_t stream);
pa_status launch_stream_read(const void* a, const void* b, size_t bytes_each, void* sink, hipStream_t stream);
pa_status launch_kv_copy_page(const pa_kv_cache_desc* c, int32_t src_page, int32_t dst_page, hipStream_t stream);

// Mask / score modifications of a call (pa_attn_mods with the "off" values normalised).  The kernels take a
// compile-time policy that says which hooks exist at all; NoMods compiles to the unmodified kernel.
struct ModArgs {
    int32_t window;              // 0 = off
    float softcap;               // 0 = off
    const float* alibi_slopes;   // null = off
    const int32_t* doc_ids;      // null = off
    int64_t doc_stride;
    int32_t user_mod;            // kId of a user modification (pagedattn_mods.h), 0 = off
    const void* user_data;
};

// U: a user modification struct of pagedattn_mods.h, or NoUser.  A user modification comes with every built-in hook
// compiled in (its instantiation is Mods<true, true, true, U>); a hook whose argument is absent does nothing.
struct NoUser {
    static constexpr int32_t kId = 0;
};
template <bool WINDOW, bool SCORE, bool DOC, typename U = NoUser>
struct Mods {
    static constexpr bool kWindow = WINDOW;   // sliding window
    static constexpr bool kScore = SCORE;     // soft cap and / or linear position bias
    static constexpr bool kDoc = DOC;         // document mask
    static constexpr bool kUser = U::kId != 0;
    static constexpr bool kAny = WINDOW || SCORE || DOC || kUser;
    typedef U User;
};
typedef Mods<false, false, false> NoMods;
typedef Mods<true, true, true> AllMods;

struct AttnArgs {
    CacheView cache;
    pa_dtype dtype;
    const void* q;           // [total_q, Hq, d]
    void* out;               // [total_q, Hq, d]
    float* lse;              // [total_q, Hq] or null
    const int32_t* cu_q_lens;  // [batch + 1] or null (decode: row == sequence)
    const int32_t* block_table;
    const int32_t* seq_lens;
    int32_t batch;
    int32_t total_q;
    int32_t max_q_len;
    int32_t num_q_heads;
    int32_t max_blocks;
    int32_t max_seq_len;
    float scale;
    int32_t causal;
    float* part_o;           // workspace: partial outputs
    float* part_lse;         // workspace: partial LSEs
    SplitPlan plan;          // chunked split (portable kernel)
    // tile-stream split (MFMA decode kernel): partial (w + s) of workgroup w and sequence s; the workgroups
    // holding a sequence's first / last tile are recorded in seg_first / seg_last (first = -1: no merge needed)
    int32_t stream_split;    // 1 when the tile-stream layout is in use
    int32_t num_wgs;
    int32_t* seg_first;
    int32_t* seg_last;
    int32_t skip_small;      // prefill kernel: leave sequences with q_len * G <= 16 to the decode kernel
    ModArgs mods;
    bool has_mods;
    // decode step with the append of one new token per sequence folded in (position seq_lens[s] - 1): [batch, Hkv, d]
    // rows of the cache dtype, or null
    const void* k_new;
    const void* v_new;
    // one-launch decode with several workgroups per (sequence, KV head, slice): their number, their partials (a
    // part of the workspace) and the arrival counters (zero on entry, zero again on exit)
    int32_t short_nsplit;
    float* short_part;
    uint32_t* short_arrive;
};

// Portable VALU kernel: any dtype / head_dim / page size / group size; decode and ragged prefill.
pa_status launch_attention_generic(const AttnArgs& a, hipStream_t stream);
// MFMA decode kernel: bf16, head_dim 128, group size <= 16.
bool decode_mfma_supported(const AttnArgs& a);
int32_t decode_mfma_heads_per_wg(int32_t num_kv_heads, int32_t head_dim);
pa_status launch_decode_mfma(const AttnArgs& a, hipStream_t stream);
// The same tiles in one launch for short contexts: a workgroup per (sequence, KV head), its waves split the context
// and merge through LDS; no workspace.
bool decode_short_supported(const AttnArgs& a);
pa_status launch_decode_short(const AttnArgs& a, hipStream_t stream);
// Floats of the partials of that kernel for `wgs` workgroups (several per sequence and KV head), and the most
// workgroups one call may split into.
inline size_t decode_short_part_floats(int64_t wgs, int32_t head_dim) { return (size_t)wgs * (16 * (size_t)head_dim + 32); }
constexpr int32_t kShortMaxSplit = 16;
constexpr int32_t kShortMaxUnits = 4096;   // (sequence, KV head, slice) units of a split call: one arrival counter each
// MFMA prefill kernel: bf16, head_dim 128.
bool prefill_mfma_supported(const AttnArgs& a);
int32_t prefill_mfma_log2_pack(int32_t num_q_heads, int32_t num_kv_heads);
pa_status launch_prefill_mfma(const AttnArgs& a, hipStream_t stream);
// LSE merge of the split partials into out / lse.
pa_status launch_merge(const AttnArgs& a, hipStream_t stream);

// ---------------------------------------------------------------------------------------------
// Small device helpers.
// ---------------------------------------------------------------------------------------------
#if defined(__HIPCC__)
__device__ __forceinline__ float bf16_bits_to_float(uint32_t bits16)
{
    return __uint_as_float(bits16 << 16);
}

__device__ __forceinline__ float f16_bits_to_float(uint32_t bits16)
{
    return (float)__builtin_bit_cast(_Float16, (uint16_t)bits16);
}

// Round-to-nearest-even fp32 -> fp16 bit pattern (v_cvt_f16_f32).
__device__ __forceinline__ uint32_t float_to_f16_bits(float f)
{
    return __builtin_bit_cast(uint16_t, (_Float16)f);
}

// Round-to-nearest-even fp32 -> bf16 bit pattern (NaN stays NaN).
__device__ __forceinline__ uint32_t float_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}

// Element traits of the 16-bit matrix-core kernels: packing with round-to-nearest-even, unpacking, and the two
// matrix instructions.  Operands travel as any 16-byte type (8 elements); the accumulators are fp32.
typedef __attribute__((ext_vector_type(4))) float mfma_f32x4;
typedef __attribute__((ext_vector_type(16))) float mfma_f32x16;

struct ElemBf16 {
    static constexpr pa_dtype kDtype = PA_DTYPE_BF16;
    typedef __attribute__((ext_vector_type(8))) __bf16 vec8;
    typedef __attribute__((ext_vector_type(2))) __bf16 vec2;
    __device__ static __forceinline__ uint32_t pack(float lo, float hi)
    {
        typedef __attribute__((ext_vector_type(2))) float f32x2;
        const f32x2 v = {lo, hi};
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, vec2));   // v_cvt_pk_bf16_f32
    }
    __device__ static __forceinline__ float lo_of(uint32_t w) { return __uint_as_float(w << 16); }
    __device__ static __forceinline__ float hi_of(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
    template <typename A, typename B>
    __device__ static __forceinline__ mfma_f32x4 mfma16(const A& a, const B& b, mfma_f32x4 c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(vec8, a), __builtin_bit_cast(vec8, b), c, 0, 0,
                                                       0);
    }
    template <typename A, typename B>
    __device__ static __forceinline__ mfma_f32x16 mfma32(const A& a, const B& b, mfma_f32x16 c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(vec8, a), __builtin_bit_cast(vec8, b), c, 0, 0,
                                                       0);
    }
};

struct ElemF16 {
    static constexpr pa_dtype kDtype = PA_DTYPE_F16;
    typedef __attribute__((ext_vector_type(8))) _Float16 vec8;
    typedef __attribute__((ext_vector_type(2))) _Float16 vec2;
    __device__ static __forceinline__ uint32_t pack(float lo, float hi)
    {
        typedef __attribute__((ext_vector_type(2))) float f32x2;
        const f32x2 v = {lo, hi};
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, vec2));
    }
    __device__ static __forceinline__ float lo_of(uint32_t w) { return (float)__builtin_bit_cast(vec2, w)[0]; }
    __device__ static __forceinline__ float hi_of(uint32_t w) { return (float)__builtin_bit_cast(vec2, w)[1]; }
    template <typename A, typename B>
    __device__ static __forceinline__ mfma_f32x4 mfma16(const A& a, const B& b, mfma_f32x4 c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(vec8, a), __builtin_bit_cast(vec8, b), c, 0, 0,
                                                      0);
    }
    template <typename A, typename B>
    __device__ static __forceinline__ mfma_f32x16 mfma32(const A& a, const B& b, mfma_f32x16 c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(vec8, a), __builtin_bit_cast(vec8, b), c, 0, 0,
                                                      0);
    }
};

// User hooks of a policy M on the score x (natural units) of key j; the key handed to the hooks is clamped to the
// context (tiles are padded with clamped keys whose scores the length mask removes anyway).
template <typename M, typename F>
__device__ __forceinline__ F user_score(const pa_mod_ctx& c, int32_t j, F x)
{
    if constexpr (M::kUser) {
        const int32_t jc = min(j, c.len - 1);
        return M::User::visible(c, jc) ? M::User::score(c, jc, x) : (F)-INFINITY;
    } else {
        return x;
    }
}

// Which sequence a packed query row belongs to and how many keys it may see.  cu_q_lens is the
// prefix-sum vector of Sec. III-B (null for decode, where row == sequence).  Query i of a sequence with
// q_len queries sits at position len - q_len + i; keys 0 .. n_keys-1 are allowed: n_keys = len under the
// length mask alone, min(len, position + 1) with the causal bound.
struct RowInfo {
    int32_t seq;
    int32_t n_keys;
    int32_t pos;      // the query's absolute position
    int32_t len;
};

__device__ __forceinline__ RowInfo locate_row(const int32_t* __restrict__ cu_q_lens,
                                              const int32_t* __restrict__ seq_lens, int32_t batch, int32_t row,
                                              int32_t causal)
{
    RowInfo r;
    int32_t q_len = 1, qi = 0;
    if (cu_q_lens == nullptr) {
        r.seq = row;
    } else {
        int32_t lo = 0, hi = batch;   // largest s with cu_q_lens[s] <= row
        while (hi - lo > 1) {
            const int32_t mid = (lo + hi) >> 1;
            if (cu_q_lens[mid] <= row) lo = mid; else hi = mid;
        }
        r.seq = lo;
        q_len = cu_q_lens[lo + 1] - cu_q_lens[lo];
        qi = row - cu_q_lens[lo];
    }
    const int32_t len = seq_lens[r.seq];
    int32_t n = len;
    if (causal) n = min(len, len - q_len + qi + 1);
    r.n_keys = max(n, 0);
    r.pos = len - q_len + qi;
    r.len = len;
    return r;
}

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
#endif

}  // namespace pa
