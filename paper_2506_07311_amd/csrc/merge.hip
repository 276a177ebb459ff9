// Split-KV merge: combines the per-chunk softmax partials of one (query row, head) exactly.
// With partial c holding the normalised output o_c and lse_c = log sum_j exp(score_j) over its keys,
//   M = max_c lse_c,  w_c = exp(lse_c - M),  out = sum_c w_c o_c / sum_c w_c,  lse = M + log sum_c w_c.
// Only the ceil(n_keys / chunk) chunks that hold keys are read; a row without keys gets out = 0, lse = -inf.
#include "common.h"

namespace pa {

namespace {

// OUT: element type of `out` as a pa_dtype value.
template <int OUT>
__device__ __forceinline__ void store_out(void* out, int64_t i, float r)
{
    if (OUT == PA_DTYPE_BF16)
        reinterpret_cast<uint16_t*>(out)[i] = (uint16_t)float_to_bf16_bits(r);
    else if (OUT == PA_DTYPE_F16)
        reinterpret_cast<uint16_t*>(out)[i] = (uint16_t)float_to_f16_bits(r);
    else
        reinterpret_cast<float*>(out)[i] = r;
}

// Four consecutive output elements of one row.
template <int OUT>
__device__ __forceinline__ void store_out4(void* out, int64_t i, float4 r)
{
    if (OUT == PA_DTYPE_F32) {
        *reinterpret_cast<float4*>(reinterpret_cast<float*>(out) + i) = r;
    } else {
        uint2 w;
        if (OUT == PA_DTYPE_BF16) {
            w.x = float_to_bf16_bits(r.x) | (float_to_bf16_bits(r.y) << 16);
            w.y = float_to_bf16_bits(r.z) | (float_to_bf16_bits(r.w) << 16);
        } else {
            w.x = float_to_f16_bits(r.x) | (float_to_f16_bits(r.y) << 16);
            w.y = float_to_f16_bits(r.z) | (float_to_f16_bits(r.w) << 16);
        }
        *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(out) + i) = w;
    }
}

// A workgroup of 256 threads merges kMergePairs (query row, head) pairs: 32 lanes per pair, four consecutive output
// columns per lane and pass (head_dim is a multiple of 4 for every supported element type), 16-byte loads of the
// partial rows.  (One small workgroup per pair, as this kernel once was, is bound by the rate at which workgroups are
// dispatched: 65536 of them for a 2048-token prompt with 32 heads.)
constexpr int kMergePairs = 8;

template <int OUT>
__global__ __launch_bounds__(256) void paged_attention_merge_kernel(
    const float* __restrict__ part_o, const float* __restrict__ part_lse, void* __restrict__ out,
    float* __restrict__ lse, const int32_t* __restrict__ cu_q_lens, const int32_t* __restrict__ seq_lens,
    int32_t batch, int32_t num_q_heads, int32_t d, int32_t causal, int32_t chunk, int32_t nsplit, int64_t pairs)
{
    const int64_t o_idx = (int64_t)blockIdx.x * kMergePairs + (threadIdx.x >> 5);
    if (o_idx >= pairs) return;
    const int lane = threadIdx.x & 31;
    const int32_t row = (int32_t)(o_idx / num_q_heads);
    const RowInfo ri = locate_row(cu_q_lens, seq_lens, batch, row, causal);
    const int32_t n = (ri.n_keys + chunk - 1) / chunk;   // chunks that hold keys
    const float* pl = part_lse + o_idx * nsplit;
    const float* po = part_o + o_idx * nsplit * d;

    float M = -INFINITY;
    for (int32_t c = 0; c < n; ++c) M = fmaxf(M, pl[c]);
    const bool none = M == -INFINITY;            // no chunk holds a visible key (masks can empty every chunk)
    float wsum = 0.f;
    for (int32_t c = 0; c < n && !none; ++c) wsum += expf(pl[c] - M);
    for (int e = 4 * lane; e < d; e += 128) {
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int32_t c = 0; c < n && !none; ++c) {
            const float w = expf(pl[c] - M);
            const float4 v = *reinterpret_cast<const float4*>(po + (int64_t)c * d + e);
            acc.x = fmaf(w, v.x, acc.x);
            acc.y = fmaf(w, v.y, acc.y);
            acc.z = fmaf(w, v.z, acc.z);
            acc.w = fmaf(w, v.w, acc.w);
        }
        const float4 r = none ? make_float4(0.f, 0.f, 0.f, 0.f)
                              : make_float4(acc.x / wsum, acc.y / wsum, acc.z / wsum, acc.w / wsum);
        store_out4<OUT>(out, o_idx * d + e, r);
    }
    if (lse && lane == 0) lse[o_idx] = !none ? M + logf(wsum) : -INFINITY;
}

// Tile-stream layout: sequence s was cut by the workgroups seg_first[s] .. seg_last[s]; workgroup w left its
// partial at index (w + s).  seg_first[s] < 0 means one workgroup held the whole sequence and wrote the final
// result itself.  One workgroup merges one (sequence, head): the partial LSEs are fetched by as many threads at
// once and reduced through LDS, then every thread owns one output column and sums the weighted partial rows
// with independent loads (eight in flight), so the kernel costs a few memory latencies, not one per partial.
constexpr int kMergeThreads = 128;

// RAGGED (the few-query sequences of a prefill call): one workgroup per (sequence, KV head, column); column
// c of the 16 is query c / G, head c % G of the group; partials are 16 rows per KV head; sequences that did not
// take that path (q_len * G > 16) are skipped.
template <int OUT, bool RAGGED>
__global__ __launch_bounds__(kMergeThreads) void paged_attention_merge_stream_kernel(
    const float* __restrict__ part_o, const float* __restrict__ part_lse, void* __restrict__ out,
    float* __restrict__ lse, const int32_t* __restrict__ seq_lens, const int32_t* __restrict__ seg_first,
    const int32_t* __restrict__ seg_last, int32_t num_q_heads, int32_t d, const int32_t* __restrict__ cu_q_lens,
    int32_t num_kv_heads)
{
    __shared__ float w_s[kMaxDecodeWGs + 1];
    __shared__ float red[4];
    const int32_t rows = RAGGED ? num_kv_heads * 16 : num_q_heads;   // partial rows per (workgroup, sequence)
    const int32_t s = blockIdx.x / rows;
    const int32_t h = blockIdx.x % rows;
    int64_t o_idx = blockIdx.x;
    if (RAGGED) {
        const int32_t G = num_q_heads / num_kv_heads;
        const int32_t q_len = cu_q_lens[s + 1] - cu_q_lens[s];
        const int32_t col = h & 15;
        if (q_len < 1 || q_len * G > 16 || col >= q_len * G) return;
        o_idx = (int64_t)(cu_q_lens[s] + col / G) * num_q_heads + (h >> 4) * G + col % G;
    }
    const int tid = threadIdx.x;
    const int32_t len = seq_lens[s];
    const int32_t first = seg_first[s];
    const int32_t last = seg_last[s];
    if (len > 0 && first < 0) return;                  // already final
    const int32_t n = len > 0 ? last - first + 1 : 0;
    const int64_t p0 = (int64_t)(first + s) * rows + h;            // partial c sits `rows` rows further each

    // weights exp(lse_c - M) into LDS
    float mx = -INFINITY;
    for (int32_t c = tid; c < n; c += kMergeThreads) {
        const float v = part_lse[p0 + (int64_t)c * rows];
        w_s[c] = v;
        mx = fmaxf(mx, v);
    }
    mx = wave_max(mx);
    if ((tid & 63) == 0) red[tid >> 6] = mx;
    __syncthreads();
    float M = fmaxf(red[0], red[1]);
    const bool no_keys = M == -INFINITY;               // RAGGED: a row whose causal bound excludes every key
    if (no_keys) M = 0.f;
    float ws = 0.f;
    for (int32_t c = tid; c < n; c += kMergeThreads) {
        const float wgt = expf(w_s[c] - M);
        w_s[c] = wgt;
        ws += wgt;
    }
    ws = wave_sum(ws);
    if ((tid & 63) == 0) red[2 + (tid >> 6)] = ws;
    __syncthreads();
    const float wsum = red[2] + red[3];

    for (int e = tid; e < d; e += kMergeThreads) {
        const float* po = part_o + p0 * d + e;
        const int64_t step = (int64_t)rows * d;
        float acc = 0.f;
        int32_t c = 0;
        for (; c + 8 <= n; c += 8) {
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = po[(int64_t)(c + u) * step];
#pragma unroll
            for (int u = 0; u < 8; ++u) acc = fmaf(w_s[c + u], v[u], acc);
        }
        for (; c < n; ++c) acc = fmaf(w_s[c], po[(int64_t)c * step], acc);
        const float r = (n > 0 && !no_keys) ? acc / wsum : 0.f;
        store_out<OUT>(out, o_idx * d + e, r);
    }
    if (lse && tid == 0) lse[o_idx] = (n > 0 && !no_keys) ? M + logf(wsum) : -INFINITY;
}

}  // namespace

pa_status launch_merge(const AttnArgs& a, hipStream_t stream)
{
    const int64_t blocks = (int64_t)a.total_q * a.num_q_heads;
    if (blocks > 0x7fffffffLL) return PA_ERR_UNSUPPORTED;
    ProfileScope prof("paged_attention_merge_kernel", stream);
    if (a.stream_split) {
        // tile-stream partials of the MFMA decode kernel (16-bit pools only); with cu_q_lens: the few-query
        // sequences of a prefill call
        const bool ragged = a.cu_q_lens != nullptr;
        const int64_t sblocks = ragged ? (int64_t)a.batch * a.cache.num_kv_heads * 16 : blocks;
        if (sblocks > 0x7fffffffLL || a.dtype == PA_DTYPE_F32) return PA_ERR_UNSUPPORTED;
        auto kern = a.dtype == PA_DTYPE_BF16
                        ? (ragged ? paged_attention_merge_stream_kernel<PA_DTYPE_BF16, true>
                                  : paged_attention_merge_stream_kernel<PA_DTYPE_BF16, false>)
                        : (ragged ? paged_attention_merge_stream_kernel<PA_DTYPE_F16, true>
                                  : paged_attention_merge_stream_kernel<PA_DTYPE_F16, false>);
        hipLaunchKernelGGL(kern, dim3((uint32_t)sblocks), dim3(kMergeThreads), 0, stream, a.part_o, a.part_lse, a.out,
                           a.lse, a.seq_lens, a.seg_first, a.seg_last, a.num_q_heads, a.cache.head_dim, a.cu_q_lens,
                           a.cache.num_kv_heads);
        return launch_status();
    }
    auto kern = a.dtype == PA_DTYPE_BF16  ? paged_attention_merge_kernel<PA_DTYPE_BF16>
                : a.dtype == PA_DTYPE_F16 ? paged_attention_merge_kernel<PA_DTYPE_F16>
                                          : paged_attention_merge_kernel<PA_DTYPE_F32>;
    if (a.cache.head_dim % 4 != 0) return PA_ERR_UNSUPPORTED;   // (16-byte rows: every supported element type has it)
    hipLaunchKernelGGL(kern, dim3((uint32_t)((blocks + kMergePairs - 1) / kMergePairs)), dim3(256), 0, stream, a.part_o,
                       a.part_lse, a.out, a.lse, a.cu_q_lens, a.seq_lens, a.batch, a.num_q_heads, a.cache.head_dim,
                       a.causal, a.plan.chunk, a.plan.nsplit, blocks);
    return launch_status();
}

}  // namespace pa
