// Paged prefill (ragged packed queries, optional causal bound) for bf16 pools with head_dim 128 on gfx950.
//
// Prefill is a dense contraction (about 590 flop per byte at 2048 tokens), so it runs on the matrix cores
// with v_mfma_f32_32x32x16_bf16 in the flash-attention arrangement: one workgroup of 4 waves owns 128
// consecutive queries of one (sequence, query head); wave w owns 32 of them.  The context is walked in
// tiles of 64 keys.  A tile's K and V rows are fetched page by page through the block table (Algorithm 1:
// page = block_table[s][j >> log2 P], slot = j & (P-1)) with coalesced 16-byte loads into registers one
// tile ahead, then staged in LDS:
//   K   row-major [64 keys][128] (+16 B row padding: conflict-free 16-byte MFMA operand reads)
//   V^T [128 columns][64 keys]   (in-lane 4x8 transpose with byte permutes before the LDS write, keys stored
//                                 in the order the P operand needs them so that one 16-byte read is an operand)
// Both products are computed transposed so that every per-query quantity is lane-local (lane%32 = query):
//   S^T[key, q]  = K[key, :] . Q[q, :]^T        A = K from LDS, B = Q held in registers for the whole kernel
//   O^T[col, q] += V^T[col, key] . P^T[key, q]  A = V^T from LDS, B = P straight from the S^T accumulators
// The accumulator layout of S^T (lane holds keys 8a + 4h + b of its query) is, after packing to bf16, already
// the B-operand layout of the second product for a permuted key order; V^T is stored in that same order.
// Online softmax runs in the log2 domain; masking (length, causal, ragged rows) is by selection.
#include "common.h"

namespace pa {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(2))) float f32x2;

constexpr int kD = 128;
constexpr int kBM = 128;              // queries per workgroup
constexpr int kBN = 64;               // keys per tile
constexpr int kThreads = 256;
constexpr int kPreciseKeys = 512;      // contexts up to this length use two-term bf16 weights
constexpr int kKRow = 256 + 16;       // bytes per K row in LDS
constexpr int kVRow = 128 + 16;       // bytes per V^T row in LDS
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi)
{
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

__device__ __forceinline__ uint32_t word(const uint4 v, int w)
{
    return w == 0 ? v.x : w == 1 ? v.y : w == 2 ? v.z : v.w;
}

struct Stage {
    uint4 k0, k1, k2, k3;   // K rows (tid/16) + 16*i, 16-byte piece tid%16
    uint4 v0, v1, v2, v3;   // V rows 4*(tid/16) + i, 16-byte piece tid%16
};

// One 16-byte piece of the row of `key` (clamped to a live slot) of a pool: Algorithm 1's translation.
__device__ __forceinline__ uint4 load_row_piece(const char* base, const CacheView& cache, const int32_t* table,
                                                int32_t key, int32_t last_key)
{
    key = min(key, last_key);
    const int64_t page = table[key >> cache.log2_page];
    const int32_t slot = key & (cache.page_size - 1);
    return *reinterpret_cast<const uint4*>(base + (page * cache.page_stride + (int64_t)slot * cache.token_stride) * 2);
}

__device__ __forceinline__ void load_stage(Stage& st, const CacheView& cache, const int32_t* table, int32_t kvh,
                                           int32_t t0, int32_t last_key, int tid)
{
    const int c = tid & 15, g = tid >> 4;
    const int64_t head_off = (int64_t)kvh * cache.head_stride * 2 + c * 16;
    const char* kb = reinterpret_cast<const char*>(cache.k) + head_off;
    const char* vb = reinterpret_cast<const char*>(cache.v) + head_off;
    st.k0 = load_row_piece(kb, cache, table, t0 + g, last_key);
    st.k1 = load_row_piece(kb, cache, table, t0 + g + 16, last_key);
    st.k2 = load_row_piece(kb, cache, table, t0 + g + 32, last_key);
    st.k3 = load_row_piece(kb, cache, table, t0 + g + 48, last_key);
    st.v0 = load_row_piece(vb, cache, table, t0 + 4 * g + 0, last_key);
    st.v1 = load_row_piece(vb, cache, table, t0 + 4 * g + 1, last_key);
    st.v2 = load_row_piece(vb, cache, table, t0 + 4 * g + 2, last_key);
    st.v3 = load_row_piece(vb, cache, table, t0 + 4 * g + 3, last_key);
}

__device__ __forceinline__ void store_stage(const Stage& st, char* k_s, char* v_s, int tid)
{
    const int c = tid & 15, g = tid >> 4;
    *reinterpret_cast<uint4*>(k_s + (g + 0) * kKRow + c * 16) = st.k0;
    *reinterpret_cast<uint4*>(k_s + (g + 16) * kKRow + c * 16) = st.k1;
    *reinterpret_cast<uint4*>(k_s + (g + 32) * kKRow + c * 16) = st.k2;
    *reinterpret_cast<uint4*>(k_s + (g + 48) * kKRow + c * 16) = st.k3;
    // keys 4g .. 4g+3 of the tile: 16-key group ks = g/4, u = g%4; the second product reads, per 16-key group,
    // lane half h, element e <-> key 8*(e/4) + 4*h + e%4, so key 4u + b sits at slot 8*(u%2) + 4*(u/2) + b
    const int ks = g >> 2, u = g & 3;
    const int col_byte = (16 * ks + 8 * (u & 1) + 4 * (u >> 1)) * 2;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const uint32_t sel = (j & 1) ? 0x07060302u : 0x05040100u;
        uint2 w;
        w.x = __builtin_amdgcn_perm(word(st.v1, j / 2), word(st.v0, j / 2), sel);
        w.y = __builtin_amdgcn_perm(word(st.v3, j / 2), word(st.v2, j / 2), sel);
        *reinterpret_cast<uint2*>(v_s + (8 * c + j) * kVRow + col_byte) = w;
    }
}

__global__ __launch_bounds__(kThreads, 2) void paged_prefill_mfma_kernel(
    CacheView cache, const uint16_t* __restrict__ q, uint16_t* __restrict__ out, float* __restrict__ lse,
    const int32_t* __restrict__ cu_q_lens, const int32_t* __restrict__ block_table,
    const int32_t* __restrict__ seq_lens, int32_t num_q_heads, int32_t max_blocks, float scale, int32_t causal)
{
    __shared__ __attribute__((aligned(16))) char k_s[kBN * kKRow];
    __shared__ __attribute__((aligned(16))) char v_s[kD * kVRow];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int ql = lane & 31, hh = lane >> 5;
    const int32_t s = blockIdx.z;
    const int32_t h = blockIdx.y;
    const int32_t q_begin = cu_q_lens[s];
    const int32_t q_len = cu_q_lens[s + 1] - q_begin;
    const int32_t tile = gridDim.x - 1 - blockIdx.x;        // heaviest (latest) query tiles are dispatched first
    const int32_t m0 = tile * kBM;
    if (m0 >= q_len) return;
    const int32_t len = seq_lens[s];
    const int32_t G = num_q_heads / cache.num_kv_heads;
    const int32_t kvh = h / G;
    const int32_t* table = block_table + (int64_t)s * max_blocks;

    // this lane's query, its position and key bound
    const int32_t qi = m0 + 32 * wave + ql;
    const bool q_valid = qi < q_len;
    const int32_t qi_c = min(qi, q_len - 1);
    int32_t nk = len;                                        // keys 0 .. nk-1 are allowed
    if (causal) nk = min(len, len - q_len + qi_c + 1);
    nk = max(nk, 0);
    // workgroup-wide key range
    const int32_t q_last = min(m0 + kBM, q_len) - 1;
    int32_t nk_wg = len;
    if (causal) nk_wg = min(len, len - q_len + q_last + 1);
    nk_wg = max(nk_wg, 0);
    // per wave: the largest bound of its 32 queries decides which tiles it can skip
    int32_t nk_wave = len;
    if (causal) nk_wave = min(len, len - q_len + min(m0 + 32 * wave + 31, q_len - 1) + 1);
    nk_wave = max(nk_wave, 0);
    int32_t nk_wave_min = len;                               // smallest bound: tiles below it need no mask
    if (causal) nk_wave_min = max(0, min(len, len - q_len + min(m0 + 32 * wave, q_len - 1) + 1));

    const int64_t row = (int64_t)(q_begin + qi_c) * num_q_heads + h;
    // Q as B operand: lane%32 = query, step ks covers head_dim elements 16*ks + 8*hh .. +7
    bf16x8 qf[8];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
        qf[ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(q + row * kD + 16 * ks + 8 * hh));

    f32x16 o[4];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[t][r] = 0.f;
    float m = -INFINITY, l = 0.f;
    const float sc = scale * kLog2e;
    // Short contexts carry the softmax weights as two bf16 terms: with few keys the individual weights are
    // large and their 2^-9 rounding would show in the output; over long contexts it averages out.
    const bool precise = nk_wg <= kPreciseKeys;              // workgroup-uniform

    Stage st;
    if (nk_wg > 0) load_stage(st, cache, table, kvh, 0, len - 1, tid);
    for (int32_t t0 = 0; t0 < nk_wg; t0 += kBN) {
        __syncthreads();                                     // previous tile's LDS reads are done
        store_stage(st, k_s, v_s, tid);
        __syncthreads();
        if (t0 + kBN < nk_wg) load_stage(st, cache, table, kvh, t0 + kBN, len - 1, tid);
        if (t0 >= nk_wave) continue;                         // wave-uniform: nothing for this wave here

        // S^T tiles: keys 32*mt .. +31 of the tile against this wave's 32 queries
        f32x16 sacc[2];
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
#pragma unroll
            for (int r = 0; r < 16; ++r) sacc[mt][r] = 0.f;
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                const bf16x8 a = __builtin_bit_cast(
                    bf16x8, *reinterpret_cast<const uint4*>(k_s + (32 * mt + ql) * kKRow + 32 * ks + 16 * hh));
                sacc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[ks], sacc[mt], 0, 0, 0);
            }
        }
        // sacc[mt][r]: key t0 + 32*mt + 8*(r/4) + 4*hh + r%4, query lane%32
        const bool need_mask = t0 + kBN > nk_wave_min;       // wave-uniform
        float tmax = -INFINITY;
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                float x = sacc[mt][r] * sc;
                if (need_mask && t0 + 32 * mt + 8 * (r / 4) + 4 * hh + (r % 4) >= nk) x = -INFINITY;
                sacc[mt][r] = x;
                tmax = fmaxf(tmax, x);
            }
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
        const float m_new = fmaxf(m, tmax);
        const float m_use = m_new == -INFINITY ? 0.f : m_new;   // a query with no allowed key so far
        const float alpha = __builtin_amdgcn_exp2f(m - m_use);
        float psum = 0.f;
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float p = __builtin_amdgcn_exp2f(sacc[mt][r] - m_use);
                sacc[mt][r] = p;
                psum += p;
            }
        m = m_new;
        l = l * alpha + psum;
        if (__any(alpha != 1.f)) {
#pragma unroll
            for (int t = 0; t < 4; ++t) o[t] *= alpha;
        }
        // P^T as B operand of step ks (16 keys): elements e = 0..7 <-> accumulator registers 8*(ks%2) + e of tile ks/2
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const int mt = ks >> 1, r0 = 8 * (ks & 1);
            uint4 w, wl;
            w.x = pack_bf16(sacc[mt][r0 + 0], sacc[mt][r0 + 1]);
            w.y = pack_bf16(sacc[mt][r0 + 2], sacc[mt][r0 + 3]);
            w.z = pack_bf16(sacc[mt][r0 + 4], sacc[mt][r0 + 5]);
            w.w = pack_bf16(sacc[mt][r0 + 6], sacc[mt][r0 + 7]);
            const bf16x8 pf = __builtin_bit_cast(bf16x8, w);
            if (precise) {   // second bf16 term of the weights: p = hi + lo, lo = bf16(p - hi)
                wl.x = pack_bf16(sacc[mt][r0 + 0] - __uint_as_float(w.x << 16),
                                 sacc[mt][r0 + 1] - __uint_as_float(w.x & 0xffff0000u));
                wl.y = pack_bf16(sacc[mt][r0 + 2] - __uint_as_float(w.y << 16),
                                 sacc[mt][r0 + 3] - __uint_as_float(w.y & 0xffff0000u));
                wl.z = pack_bf16(sacc[mt][r0 + 4] - __uint_as_float(w.z << 16),
                                 sacc[mt][r0 + 5] - __uint_as_float(w.z & 0xffff0000u));
                wl.w = pack_bf16(sacc[mt][r0 + 6] - __uint_as_float(w.w << 16),
                                 sacc[mt][r0 + 7] - __uint_as_float(w.w & 0xffff0000u));
            }
            const bf16x8 pl = __builtin_bit_cast(bf16x8, wl);
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const bf16x8 a = __builtin_bit_cast(
                    bf16x8, *reinterpret_cast<const uint4*>(v_s + (32 * t + ql) * kVRow + 32 * ks + 16 * hh));
                o[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf, o[t], 0, 0, 0);
                if (precise) o[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pl, o[t], 0, 0, 0);
            }
        }
    }

    l += __shfl_xor(l, 32, 64);
    if (!q_valid) return;
    const float inv = l > 0.f ? 1.f / l : 0.f;
    // o[t][r]: column 32*t + 8*(r/4) + 4*hh + r%4 of this lane's query
    uint16_t* orow = out + row * kD;
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            uint2 w;
            w.x = pack_bf16(o[t][4 * a + 0] * inv, o[t][4 * a + 1] * inv);
            w.y = pack_bf16(o[t][4 * a + 2] * inv, o[t][4 * a + 3] * inv);
            *reinterpret_cast<uint2*>(orow + 32 * t + 8 * a + 4 * hh) = w;
        }
    if (lse && hh == 0) lse[row] = l > 0.f ? (m + __builtin_amdgcn_logf(l)) * kLn2 : -INFINITY;
}

}  // namespace

bool prefill_mfma_supported(const AttnArgs& a)
{
    if (a.dtype != PA_DTYPE_BF16 || a.cache.head_dim != kD) return false;
    if (a.batch > 65535 || a.num_q_heads > 65535) return false;
    return true;
}

pa_status launch_prefill_mfma(const AttnArgs& a, hipStream_t stream)
{
    const int32_t tiles = (a.max_q_len + kBM - 1) / kBM;
    if (tiles <= 0) return PA_OK;
    const dim3 grid((uint32_t)tiles, (uint32_t)a.num_q_heads, (uint32_t)a.batch);
    ProfileScope prof("paged_prefill_mfma_kernel", stream);
    hipLaunchKernelGGL(paged_prefill_mfma_kernel, grid, dim3(kThreads), 0, stream, a.cache, (const uint16_t*)a.q,
                       (uint16_t*)a.out, a.lse, a.cu_q_lens, a.block_table, a.seq_lens, a.num_q_heads, a.max_blocks,
                       a.scale, a.causal);
    return launch_status();
}

}  // namespace pa
