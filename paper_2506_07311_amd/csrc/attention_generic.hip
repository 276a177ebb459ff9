// Portable paged attention kernel (VALU, fp32 accumulation) for every shape the MFMA kernels do not
// cover: fp32 pools, head_dims other than 64 / 128 / 256, non-positive scales in prefill, head_dim 256 prefill
// with pages of fewer than 16 tokens; it also serves as an independent GPU cross-check.  One workgroup
// computes one (query row, query head, context chunk) by flash-style tiles of 1024 keys:
//   scores  s_j = scale * <q, K[j]>            one key per thread, 16-byte loads along head_dim
//   mask    keys >= n_keys are never touched   (length mask / causal bound, Sec. III-B)
//   online softmax over tiles (running max m, sum l, rescaled accumulator)
//   PV      16 lanes (bf16, d=128) share one V row, key groups are reduced through LDS at the end
// Page translation follows Algorithm 1 for every key: page = block_table[s][j >> log2 P], o = j & (P-1).
#include "common.h"

namespace pa {

namespace {

constexpr int kThreads = 256;
constexpr int kTile = 1024;
constexpr int kMaxD = 256;

template <typename T> struct Vec;
template <> struct Vec<float> {
    static constexpr int N = 4;
    typedef double dot_t;   // fp32 I/O is held to 1e-5: 128-term fp32 dot products alone would use most of that
    __device__ static void load(const void* p, float* f)
    {
        const float4 v = *reinterpret_cast<const float4*>(p);
        f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w;
    }
    __device__ static float load1(const void* base, int64_t i) { return reinterpret_cast<const float*>(base)[i]; }
    __device__ static void store1(void* base, int64_t i, float v) { reinterpret_cast<float*>(base)[i] = v; }
};
struct bf16_tag {};
template <> struct Vec<bf16_tag> {
    static constexpr int N = 8;
    typedef float dot_t;
    __device__ static void load(const void* p, float* f)
    {
        const uint4 v = *reinterpret_cast<const uint4*>(p);
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f[2 * i] = __uint_as_float(w[i] << 16);
            f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
    __device__ static float load1(const void* base, int64_t i)
    {
        return bf16_bits_to_float(reinterpret_cast<const uint16_t*>(base)[i]);
    }
    __device__ static void store1(void* base, int64_t i, float v)
    {
        reinterpret_cast<uint16_t*>(base)[i] = (uint16_t)float_to_bf16_bits(v);
    }
};

struct f16_tag {};
template <> struct Vec<f16_tag> {
    static constexpr int N = 8;
    typedef float dot_t;
    __device__ static void load(const void* p, float* f)
    {
        typedef __attribute__((ext_vector_type(8))) _Float16 half8;
        const half8 v = *reinterpret_cast<const half8*>(p);
#pragma unroll
        for (int i = 0; i < 8; ++i) f[i] = (float)v[i];
    }
    __device__ static float load1(const void* base, int64_t i)
    {
        return f16_bits_to_float(reinterpret_cast<const uint16_t*>(base)[i]);
    }
    __device__ static void store1(void* base, int64_t i, float v)
    {
        reinterpret_cast<uint16_t*>(base)[i] = (uint16_t)float_to_f16_bits(v);
    }
};

// Workgroup-wide max in the score type of the instantiation (double for fp32 I/O).
template <typename S>
__device__ __forceinline__ S block_max_t(S v, S* red)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const S u = __shfl_xor(v, o, 64);
        v = u > v ? u : v;
    }
    const int w = threadIdx.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[w] = v;
    __syncthreads();
    S a = red[0] > red[1] ? red[0] : red[1];
    S b = red[2] > red[3] ? red[2] : red[3];
    return a > b ? a : b;
}
__device__ __forceinline__ float tanh_t(float x) { return tanhf(x); }
__device__ __forceinline__ double tanh_t(double x) { return tanh(x); }

__device__ __forceinline__ float block_sum(float v, float* red)
{
    v = wave_sum(v);
    const int w = threadIdx.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[w] = v;
    __syncthreads();
    return (red[0] + red[1]) + (red[2] + red[3]);
}

// M: compile-time policy naming the mask / score hooks that exist in this instantiation (NoMods: none).
template <typename T, typename M>
__global__ __launch_bounds__(kThreads) void paged_attention_generic_kernel(
    CacheView cache, const void* __restrict__ q, void* __restrict__ out, float* __restrict__ lse,
    const int32_t* __restrict__ cu_q_lens, const int32_t* __restrict__ block_table,
    const int32_t* __restrict__ seq_lens, int32_t batch, int32_t num_q_heads, int32_t max_blocks, float scale,
    int32_t causal, float* __restrict__ part_o, float* __restrict__ part_lse, int32_t chunk, int32_t nsplit,
    ModArgs mods, const void* __restrict__ k_new, const void* __restrict__ v_new)
{
    using V = Vec<T>;
    constexpr int N = V::N;
    constexpr int EB = 16 / N;   // bytes per element
    __shared__ float q_s[kMaxD];
    typedef typename V::dot_t score_t;   // fp32 I/O keeps scores (and their distance to the max) in fp64
    __shared__ score_t sc[kTile];
    __shared__ float red[4];
    __shared__ score_t red_t[4];
    __shared__ float acc_s[kThreads * 8];

    const int tid = threadIdx.x;
    const int32_t d = cache.head_dim;
    const int32_t split = blockIdx.x % nsplit;
    const int64_t rh = blockIdx.x / nsplit;
    const int32_t h = (int32_t)(rh % num_q_heads);
    const int32_t row = (int32_t)(rh / num_q_heads);

    const RowInfo ri = locate_row(cu_q_lens, seq_lens, batch, row, causal);
    const int32_t s = ri.seq;
    const int32_t n_keys = ri.n_keys;
    int32_t c0 = split * chunk;
    int32_t c1 = min(n_keys, c0 + chunk);
    const int64_t o_idx = (int64_t)row * num_q_heads + h;
    if (M::kWindow && mods.window > 0) {   // keys outside the window are skipped, not masked
        c0 = max(c0, ri.pos - mods.window + 1);
        c1 = min(c1, ri.pos + mods.window);
    }

    if (c0 >= c1) {
        if (nsplit == 1) {   // empty context: out = 0, lse = -inf
            for (int e = tid; e < d; e += kThreads) V::store1(out, o_idx * d + e, 0.f);
            if (lse && tid == 0) lse[o_idx] = -INFINITY;
        } else if (M::kAny && split * chunk < n_keys) {
            // a chunk the merge will read, emptied by the window: an explicit empty partial
            for (int e = tid; e < d; e += kThreads) part_o[(o_idx * nsplit + split) * d + e] = 0.f;
            if (tid == 0) part_lse[o_idx * nsplit + split] = -INFINITY;
        }
        return;             // with nsplit > 1 the merge never reads chunks at or beyond n_keys
    }
    float slope = 0.f;
    const int32_t* doc = nullptr;
    int32_t my_doc = 0;
    if (M::kScore && mods.alibi_slopes) slope = mods.alibi_slopes[h];
    if (M::kDoc && mods.doc_ids) {
        doc = mods.doc_ids + (int64_t)s * mods.doc_stride;
        my_doc = doc[ri.pos];
    }

    const pa_mod_ctx uc = {mods.user_data, s, h, ri.pos, ri.len};   // what a user modification's hooks are told
    (void)uc;
    const int32_t G = num_q_heads / cache.num_kv_heads;
    const int32_t kvh = h / G;
    for (int e = tid; e < d; e += kThreads) q_s[e] = V::load1(q, o_idx * d + e);
    __syncthreads();

    const int32_t vpr = d / N;                 // 16-byte vectors per row
    const int32_t kgroups = kThreads / vpr;    // rows processed concurrently in PV
    const int32_t kg = tid / vpr;
    const int32_t vc = tid % vpr;
    const bool pv_active = kg < kgroups;
    const int32_t pmask = cache.page_size - 1;
    const int32_t* table = block_table + (int64_t)s * max_blocks;
    const char* kbase = reinterpret_cast<const char*>(cache.k) + (int64_t)kvh * cache.head_stride * EB;
    const char* vbase = reinterpret_cast<const char*>(cache.v) + (int64_t)kvh * cache.head_stride * EB;

    // Decode step with the append folded in (k_new != null; row == sequence): the new token sits at the last
    // position.  Its K / V rows are read from k_new / v_new wherever the loops below meet that key, and the workgroup
    // of the KV head's first query head whose chunk holds the key stores them into their slot (Algorithm 1, Assign).
    const int32_t new_pos = k_new ? ri.pos : -1;
    const char* knew_row = nullptr;
    const char* vnew_row = nullptr;
    if (k_new) {
        const int64_t new_off = ((int64_t)s * cache.num_kv_heads + kvh) * d * EB;
        knew_row = reinterpret_cast<const char*>(k_new) + new_off;
        vnew_row = reinterpret_cast<const char*>(v_new) + new_off;
        if (h % G == 0 && new_pos >= c0 && new_pos < c1 && tid < 2 * vpr) {
            const bool is_v = tid >= vpr;
            const int32_t piece = tid - (is_v ? vpr : 0);
            const int64_t page = table[new_pos >> cache.log2_page];
            const int64_t slot = (page * cache.page_stride + (int64_t)(new_pos & pmask) * cache.token_stride) * EB;
            char* dst = const_cast<char*>(is_v ? vbase : kbase) + slot + piece * 16;
            *reinterpret_cast<uint4*>(dst) =
                *reinterpret_cast<const uint4*>((is_v ? vnew_row : knew_row) + piece * 16);
        }
    }

    score_t m = -INFINITY;
    float l = 0.f;
    float acc[N];
#pragma unroll
    for (int e = 0; e < N; ++e) acc[e] = 0.f;

    for (int32_t t0 = c0; t0 < c1; t0 += kTile) {
        const int32_t tn = min(kTile, c1 - t0);
        // scores: one key per thread
        score_t lmax = -INFINITY;
        for (int32_t jj = tid; jj < tn; jj += kThreads) {
            const int32_t j = t0 + jj;
            const int64_t page = table[j >> cache.log2_page];
            const char* kr = kbase + (page * cache.page_stride + (int64_t)(j & pmask) * cache.token_stride) * EB;
            if (j == new_pos) kr = knew_row;
            typename V::dot_t dot = 0;
            for (int32_t c = 0; c < vpr; ++c) {
                float kv[N];
                V::load(kr + c * 16, kv);
#pragma unroll
                for (int e = 0; e < N; ++e) dot += (typename V::dot_t)q_s[c * N + e] * (typename V::dot_t)kv[e];
            }
            score_t sj = dot * (score_t)scale;
            if (M::kScore) {
                if (mods.softcap > 0.f) sj = (score_t)mods.softcap * tanh_t(sj / (score_t)mods.softcap);
                sj += (score_t)slope * (score_t)(j - ri.pos);
            }
            if (M::kDoc && doc && doc[j] != my_doc) sj = -INFINITY;
            if (M::kUser) sj = user_score<M>(uc, j, sj);   // in the score type: fp64 for fp32 pools
            sc[jj] = sj;
            lmax = sj > lmax ? sj : lmax;
        }
        const score_t m_new = block_max_t(m > lmax ? m : lmax, red_t);
        if (M::kDoc && m_new == -INFINITY) {       // no visible key so far (uniform over the workgroup)
            __syncthreads();
            continue;
        }
        const float alpha = expf((float)(m - m_new));   // m = -inf on the first tile gives 0
        float lsum = 0.f;
        for (int32_t jj = tid; jj < tn; jj += kThreads) {
            const float p = expf((float)(sc[jj] - m_new));
            sc[jj] = p;
            lsum += p;
        }
        l = l * alpha + block_sum(lsum, red);     // the barriers inside also publish sc[]
        m = m_new;
#pragma unroll
        for (int e = 0; e < N; ++e) acc[e] *= alpha;
        if (pv_active) {
            for (int32_t jj = kg; jj < tn; jj += kgroups) {
                const int32_t j = t0 + jj;
                const int64_t page = table[j >> cache.log2_page];
                const char* vr = vbase + (page * cache.page_stride + (int64_t)(j & pmask) * cache.token_stride) * EB;
                if (j == new_pos) vr = vnew_row;
                float vv[N];
                V::load(vr + vc * 16, vv);
                const float p = (float)sc[jj];
#pragma unroll
                for (int e = 0; e < N; ++e) acc[e] = fmaf(p, vv[e], acc[e]);
            }
        }
        __syncthreads();                           // sc[] is rewritten by the next tile
    }

    // reduce the key groups: acc_s[kg][d]
    if (pv_active) {
#pragma unroll
        for (int e = 0; e < N; ++e) acc_s[kg * d + vc * N + e] = acc[e];
    }
    __syncthreads();
    const float inv_l = (!M::kDoc || l > 0.f) ? 1.f / l : 0.f;
    for (int e = tid; e < d; e += kThreads) {
        float sum = 0.f;
        for (int g = 0; g < kgroups; ++g) sum += acc_s[g * d + e];
        const float o = sum * inv_l;
        if (nsplit == 1)
            V::store1(out, o_idx * d + e, o);
        else
            part_o[(o_idx * nsplit + split) * d + e] = o;
    }
    if (tid == 0) {
        const float r = (!M::kDoc || l > 0.f) ? (float)(m + (score_t)logf(l)) : -INFINITY;
        if (nsplit == 1) { if (lse) lse[o_idx] = r; }
        else part_lse[o_idx * nsplit + split] = r;
    }
}

}  // namespace

pa_status launch_attention_generic(const AttnArgs& a, hipStream_t stream)
{
    const int64_t blocks = (int64_t)a.total_q * a.num_q_heads * a.plan.nsplit;
    if (blocks > 0x7fffffffLL) return PA_ERR_UNSUPPORTED;
    ProfileScope prof("paged_attention_generic_kernel", stream);
    // hook combinations instantiated here: none; window and / or score; all (document masks)
    const int hooks = !a.has_mods ? 0 : a.mods.doc_ids ? 2 : 1;
    void (*kern)(CacheView, const void*, void*, float*, const int32_t*, const int32_t*, const int32_t*, int32_t,
                 int32_t, int32_t, float, int32_t, float*, float*, int32_t, int32_t, ModArgs, const void*,
                 const void*) = nullptr;
    typedef Mods<true, true, false> WindowScore;
    if (a.mods.user_mod) {                                // a user modification: one instantiation per listed struct
#define PA_USER_CASE(U)                                                                                 \
        if (a.mods.user_mod == U::kId) {                                                                \
            typedef Mods<true, true, true, U> UM;                                                       \
            kern = a.dtype == PA_DTYPE_F32    ? paged_attention_generic_kernel<float, UM>               \
                   : a.dtype == PA_DTYPE_BF16 ? paged_attention_generic_kernel<bf16_tag, UM>            \
                                              : paged_attention_generic_kernel<f16_tag, UM>;            \
        }
        PA_USER_MODS(PA_USER_CASE)
#undef PA_USER_CASE
        if (!kern) return PA_ERR_INVALID_ARG;
    } else if (a.dtype == PA_DTYPE_F32)
        kern = hooks == 0   ? paged_attention_generic_kernel<float, NoMods>
               : hooks == 1 ? paged_attention_generic_kernel<float, WindowScore>
                            : paged_attention_generic_kernel<float, AllMods>;
    else if (a.dtype == PA_DTYPE_BF16)
        kern = hooks == 0   ? paged_attention_generic_kernel<bf16_tag, NoMods>
               : hooks == 1 ? paged_attention_generic_kernel<bf16_tag, WindowScore>
                            : paged_attention_generic_kernel<bf16_tag, AllMods>;
    else
        kern = hooks == 0   ? paged_attention_generic_kernel<f16_tag, NoMods>
               : hooks == 1 ? paged_attention_generic_kernel<f16_tag, WindowScore>
                            : paged_attention_generic_kernel<f16_tag, AllMods>;
    hipLaunchKernelGGL(kern, dim3((uint32_t)blocks), dim3(kThreads), 0, stream, a.cache, a.q, a.out, a.lse,
                       a.cu_q_lens, a.block_table, a.seq_lens, a.batch, a.num_q_heads, a.max_blocks, a.scale, a.causal,
                       a.part_o, a.part_lse, a.plan.chunk, a.plan.nsplit, a.mods, a.cu_q_lens ? nullptr : a.k_new,
                       a.cu_q_lens ? nullptr : a.v_new);
    return launch_status();
}

}  // namespace pa
