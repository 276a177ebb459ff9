// Paged prefill (ragged packed queries, optional causal bound) for bf16 / fp16 pools with head_dim D = 128 or 64 on
// gfx950 (and D = 256 for page sizes of 16 and more).  Internal header: the kernel templates; one translation unit
// per head_dim instantiates them.  The text below describes D = 128.  D = 64 is the same kernel with half the steps: LDS rows keep their 256-byte stride and
// swizzle, only the positions of the 8 existing 16-byte pieces are read (the fetch fills the other 8 positions
// with repeats), the score product takes 4 steps instead of 8 and the value product covers 2 column blocks, not 4.  D = 256 doubles the
// steps and the column blocks: LDS rows are 512 bytes (two swizzled 256-byte halves), the two tile buffers fill 128 KiB
// and the 128 accumulator registers of O leave room for one workgroup per compute unit only.
//
// Prefill is a dense contraction (about 590 flop per byte at 2048 tokens), so it runs on the matrix cores
// with v_mfma_f32_32x32x16_bf16 in the flash-attention arrangement: one workgroup of 4 waves owns 128
// consecutive ROWS of one (sequence, KV head); wave w owns 32 of them.  A row is a (query, query head) pair:
// the G query heads that share the KV head are packed next to each other (row = query * G + head; G a power of
// two up to 16, else one head per workgroup), so K and V are streamed once per KV head whatever G is and a
// call with few queries per sequence (decode rows, speculative tokens, short chunks) still fills the tile G
// times better.  "Query" below means such a row.  The context is walked in tiles of 64 keys; the launch may
// cut it into chunks (one workgroup per chunk, partials merged by the split-KV merge kernel) when the call has
// too few rows to fill the machine.  A tile's K and V rows are fetched page by page through the block table (Algorithm 1:
// page = block_table[s][j >> log2 P], slot = j & (P-1)) and written STRAIGHT INTO LDS by the load unit
// (global_load_lds_dwordx4: 16 bytes per lane, a wave fills 4 consecutive 256-byte rows per instruction), one
// tile ahead of the one being computed, into the other of two 32 KiB buffers -- no staging registers, no LDS
// store instructions, one barrier per tile.  Rows are unpadded (256 B = all 64 LDS banks); the 16-byte piece L
// of row r sits at piece L ^ swz(r), swz(r) = 4*(r%4) + (r/4)%4 (each lane simply fetches the piece that belongs
// at its LDS position), which makes both kinds of operand read conflict-free:
//   K rows are read as 16-byte MFMA operands (16 consecutive lanes = 16 consecutive rows, same logical piece:
//     swz takes 16 distinct values),
//   V rows are read TRANSPOSED with ds_read_b64_tr_b16, the LDS transpose load of gfx950 -- the contraction
//     index of P.V is the key while memory is contiguous along head_dim (32 lanes read 64 bytes of each of 4
//     consecutive rows: swz moves them to 4 different quarters of the banks).
// Both products are computed transposed so that every per-query quantity is lane-local (lane%32 = query):
//   S^T[key, q]  = K[key, :] . Q[q, :]^T        A = K from LDS, B = Q held in registers for the whole kernel
//   O^T[col, q] += V^T[col, key] . P^T[key, q]  A = V^T from LDS, B = P straight from the S^T accumulators
// The accumulator layout of S^T (lane holds keys 8a + 4h + b of its query) is, after packing to bf16, already
// the B-operand layout of the second product for a permuted key order, and the transpose loads fetch V in that
// same order.  Online softmax runs in the log2 domain; masking (length, causal, ragged rows) is by selection.
//
// Softmax weights enter the matrix cores as bf16.  With few keys the individual weights are large and their
// 2^-9 rounding shows in the output, so query tiles that see few keys -- at most kPreciseKeys, or fewer than
// kPreciseShare of the harmonic mean of the key counts of all the call's rows (precise_key_bound) -- carry the
// weights as two bf16 terms (p = hi + lo); over long contexts the rounding averages out.
#pragma once

#include "prefill_tiles.h"

namespace pa {

namespace {

using namespace prefill;

// LDS row stride of a K or V row: 256 bytes up to head_dim 128, 512 bytes at head_dim 256.  The swizzle always
// permutes the 16 pieces of a 256-byte half row among themselves (every row starts at bank 0 either way).
template <int D>
struct RowGeo {
    static constexpr int kRowB = D > 128 ? 512 : 256;
    static constexpr int kTileB = kBN * kRowB;        // K part of a tile buffer; the V part follows
    static constexpr int kBufB = 2 * kTileB;
};
// byte offset inside its row of logical 16-byte piece L of LDS row r
__device__ __forceinline__ int piece_pos(int L, int r) { return 16 * ((L & 16) | ((L & 15) ^ swz(r))); }

// Tile fetch for 512-byte rows: one load-to-LDS instruction of a wave fills 2 consecutive rows (lane l: position
// l%32 of row l/32); wave w issues, for i < 8, the K and V instructions of rows 8*i + 2*w, +1.  dst = buffer +
// 2*w*512; row = 2*w + lane/32; lane_off[i & 1] = kv-head offset + this lane's logical piece, which depends on the
// parity of i through the swizzle of row 8*i + row.
template <bool UNIFORM>
__device__ __forceinline__ void fetch_tile512(uint32_t lds, const PageIds& p, const CacheView& cache, int32_t t0, int32_t row,
                                              int32_t last_key, const uint32_t (&lane_off)[2])
{
    constexpr int TB = RowGeo<256>::kTileB;
    const int32_t pg[4] = {p.p0, p.p1, p.p2, p.p3};
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int32_t key = t0 + 8 * i + row;
        const int32_t slot = min(key, last_key) & (cache.page_size - 1);
        int64_t off;
        if (UNIFORM)
            off = (int64_t)pg[i >> 1] * cache.page_stride * 2 +
                  ((uint32_t)slot * (uint32_t)(cache.token_stride * 2) + lane_off[i & 1]);
        else
            off = ((int64_t)pg[i >> 1] * cache.page_stride + (int64_t)slot * cache.token_stride) * 2 + lane_off[i & 1];
        load_to_lds16(lds, i * (8 * 512), reinterpret_cast<const char*>(cache.k) + off);
        load_to_lds16(lds, i * (8 * 512) + TB, reinterpret_cast<const char*>(cache.v) + off);
    }
}

__device__ __forceinline__ uint4 lds_frag(const char* p)
{
    return *reinterpret_cast<const uint4*>(p);
}

// V^T operand of the second product for 32 head_dim columns and one 16-key step, from row-major V.
// ds_read_b64_tr_b16 works on blocks of 16 lanes: lane i of a block receives element i%4 of the 8 bytes
// addressed by lanes i/4, i/4+4, i/4+8, i/4+12 of its block.  Lane x = q + 4*j of a block therefore points at
// key j of the step, columns 4q..4q+3 of the block's 16 columns, and lane i ends up with column i of 4 keys.
// The two loads fetch the keys of contraction slots 0-3 and 4-7 (8 rows apart; their swizzles differ).
struct tr_pair {
    s16x4 lo, hi;
};
__device__ __forceinline__ uint4 lds_frag_tr(const char* lo, const char* hi)
{
    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
    tr_pair r;
    r.lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(lo));
    r.hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(hi));
    return __builtin_bit_cast(uint4, r);
}

// Which rows need two-term weights.  A row that sees n keys carries a weight-rounding error of about
// 2^-9 * sqrt(sum p^2) ~ 1 / sqrt(n) in absolute terms, and the outputs of a call are judged against the RMS of the
// whole output tensor, which behaves as 1 / sqrt(H) with H the harmonic mean of n over all rows of the call.  A row
// whose n is well below H is therefore large compared with the scale it is measured on, whatever its own length:
// a short sequence batched beside long ones, or the first rows of a long causal prompt.  Every workgroup derives H
// from the lengths (one lane per sequence; sum over the rows of a causal sequence of 1/n = ln((hi+1/2)/(lo-1/2))
// for n = lo..hi, capped at the window) -- a few dozen instructions next to loads it needs anyway -- and tiles whose first row
// sees fewer than kPreciseShare * H keys take the two-term path.  Wave-uniform result.
constexpr float kPreciseShare = 0.9f;

__device__ __forceinline__ int32_t precise_key_bound(const int32_t* __restrict__ cu_q_lens,
                                                     const int32_t* __restrict__ seq_lens, int32_t batch,
                                                     int32_t causal, int32_t window, int lane)
{
    float rows = 0.f, inv = 0.f;
    for (int32_t i = lane; i < batch; i += 64) {
        const int32_t q_len = cu_q_lens[i + 1] - cu_q_lens[i];
        const int32_t len = seq_lens[i];
        if (q_len <= 0 || len <= 0) continue;
        const int32_t hi = len;                                       // keys of the last row
        const int32_t lo = causal ? max(len - q_len + 1, 1) : len;    // keys of the first row that sees any
        const int32_t cap = window > 0 ? (causal ? window : 2 * window - 1) : 0x7fffffff;
        const int32_t n_rows = causal ? hi - lo + 1 : q_len;
        rows += (float)n_rows;
        if (!causal) {
            inv += (float)q_len / (float)min(len, cap);
            continue;
        }
        const int32_t b = min(hi, cap);
        if (b >= lo) inv += __builtin_amdgcn_logf(((float)b + 0.5f) / ((float)lo - 0.5f)) * kLn2;
        const int32_t above = hi - max(lo, cap + 1) + 1;              // rows that see the whole window
        if (above > 0) inv += (float)above / (float)cap;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        rows += __shfl_xor(rows, o, 64);
        inv += __shfl_xor(inv, o, 64);
    }
    const float h = inv > 0.f ? rows / inv : 0.f;
    return max(kPreciseKeys, (int32_t)fminf(kPreciseShare * h, 1.0e9f));
}

// Online-softmax update with the 32 keys of one half tile.  s holds raw scores on entry; the weights are
// returned in p.  The running statistic is a REFERENCE exponent m_ref (log2 domain) that may trail the true
// running max: weights are exp2(score - m_ref), and as long as a lane's 16 weights sum to at most kWeightSumMax
// every one of them is a number that fp32 sums and 16-bit operands carry without loss, and out = O / l does not
// depend on the reference.  So the common path takes no maximum at all: the weights are computed with the
// reference as it stands, and only when some lane's sum exceeds the bound (or is not a number: a fresh reference
// is -inf) -- always on a query's first keys, rarely later -- is the true maximum taken, the reference raised, O
// and l rescaled and the half's weights recomputed: a wave-uniform slow path that keeps the common path free of
// branches between the score and the value products.
// What the mask / score hooks need per row (this lane's).  Unused without their hook.
struct RowMods {
    int32_t lo;         // window: first visible key of this row
    int32_t lo_until;   // window: tiles that start before this key need the lower mask (wave-uniform)
    int32_t pos;        // score: the row's absolute position
    float slope2;       // score: bias slope * log2(e)
    float cap_in;       // score: scale / softcap, 0 without a cap
    float cap_out;      // score: softcap * log2(e)
    int32_t doc;        // document mask: the row's own document id
    pa_mod_ctx uc;      // user modification: what its hooks are told about the row
};

// M: compile-time policy of the hooks.  With score hooks the scores are first rewritten in place as
// log2(e) * (cap(scale * s) + slope * (key - pos)) and the rest runs with a unit scale.
template <bool MASK, bool FIRST, typename M, int T>
__device__ __forceinline__ void half_softmax(f32x16& p, f32x16& s, f32x16 (&o)[T], float& m_ref, float& l, float sc,
                                             int32_t key0, int32_t nk, const RowMods& rm, const int32_t* docs)
{
    // document mask: ids of this lane's 16 keys (4 groups of 4 consecutive keys, 8 apart) from the tile's ids in LDS
    int4 ids[4];
    if (M::kDoc) {
#pragma unroll
        for (int a = 0; a < 4; ++a) ids[a] = *reinterpret_cast<const int4*>(docs + 8 * a);
    }
    if (M::kScore) {
        const float b0 = rm.slope2 * (float)(key0 - rm.pos);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            float x;
            if (rm.cap_in > 0.f) {   // c * tanh(y / c) with tanh(z) = 1 - 2 / (1 + e^(2z))
                const float e2z = __builtin_amdgcn_exp2f(s[r] * rm.cap_in * (2.f * kLog2e));
                x = rm.cap_out * (1.f - 2.f * __builtin_amdgcn_rcpf(1.f + e2z));
            } else {
                x = s[r] * sc;
            }
            s[r] = x + __builtin_fmaf(rm.slope2, (float)(8 * (r / 4) + (r % 4)), b0);
        }
        sc = 1.f;
    }
    if (M::kUser) {   // (a user modification is compiled with the score hooks: the scores are in the log2 domain here)
#pragma unroll
        for (int r = 0; r < 16; ++r)
            s[r] = user_score<M>(rm.uc, key0 + 8 * (r / 4) + (r % 4), s[r] * kLn2) * kLog2e;
    }
    const bool below = M::kWindow && key0 < rm.lo_until;      // wave-uniform up to the lane's 4-key offset
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        if (MASK && key0 + 8 * (r / 4) + (r % 4) >= nk) s[r] = -INFINITY;   // mask by selection
        if (below && key0 + 8 * (r / 4) + (r % 4) < rm.lo) s[r] = -INFINITY;
        if (M::kDoc) {
            const int4 g = ids[r / 4];
            const int32_t id = (r % 4) == 0 ? g.x : (r % 4) == 1 ? g.y : (r % 4) == 2 ? g.z : g.w;
            if (id != rm.doc) s[r] = -INFINITY;
        }
    }
    float psum = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        p[r] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[r], sc, -m_ref));
        psum += p[r];
    }
    // keep the speculative weights ahead of the branch below (they are dead on its slow path, and the
    // optimiser would otherwise sink them behind the test, back onto the critical path)
    asm volatile("" ::"v"(p[0]), "v"(p[1]), "v"(p[2]), "v"(p[3]), "v"(p[4]), "v"(p[5]), "v"(p[6]), "v"(p[7]), "v"(p[8]),
                 "v"(p[9]), "v"(p[10]), "v"(p[11]), "v"(p[12]), "v"(p[13]), "v"(p[14]), "v"(p[15]));
    if (FIRST) {
        // instruction order for the region that holds both score products and this half's softmax: the second
        // half's 8 matrix instructions are issued with the vector work of the first half's softmax in between
        constexpr int KS = 2 * T;                             // matrix instructions per score product
        __builtin_amdgcn_sched_group_barrier(0x100, KS / 2, 0);
#pragma unroll
        for (int i = 0; i < KS; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        // (up to head_dim 128 the region also holds the 4 * T transpose loads of the half's V fragments)
#pragma unroll
        for (int i = 0; i < KS; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            if (i < KS / 2) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            if (T <= 4) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
            __builtin_amdgcn_sched_group_barrier(0x002, 72 / KS, 0);
        }
    }
    const bool jump = !(psum <= kWeightSumMax);               // also true for the NaN / inf of a fresh reference
    if (__any(jump)) {
        float tmax = -INFINITY;
#pragma unroll
        for (int r = 0; r < 16; ++r) tmax = fmaxf(tmax, s[r]);
        const float top = pair_max(tmax) * sc;                // sc > 0: scaling commutes with the max
        const float m_new = fmaxf(m_ref, top);
        const float m_use = m_new == -INFINITY ? 0.f : m_new; // a query with no allowed key so far
        const float alpha = __builtin_amdgcn_exp2f(m_ref - m_use);
#pragma unroll
        for (int t = 0; t < T; ++t) o[t] *= alpha;
        l *= alpha;
        m_ref = m_new;
        psum = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            p[r] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[r], sc, -m_use));
            psum += p[r];
        }
    }
    l += psum;
}

// V^T operand fragments of half tile `half` (two 16-key steps x T column blocks), read ahead of their use: the
// transpose loads do not depend on the weights, so they are issued a phase early (under the score products and the
// softmax) and their latency never stands in front of the value product.
// vx[2t], vx[2t+1] = this lane's swizzled transpose-load offsets (slots 0-3 / 4-7) for the 32 columns t.
template <int T>
__device__ __forceinline__ void load_v_frags(uint4 (&va)[T], uint4 (&vb)[T], const char* vbuf, int half,
                                             const uint32_t (&vx)[2 * T])
{
    constexpr int RB = 256;
    const char* v0 = vbuf + (32 * half) * RB;
#pragma unroll
    for (int t = 0; t < T; ++t) va[t] = lds_frag_tr(v0 + vx[2 * t], v0 + vx[2 * t + 1]);
#pragma unroll
    for (int t = 0; t < T; ++t) vb[t] = lds_frag_tr(v0 + 16 * RB + vx[2 * t], v0 + 16 * RB + vx[2 * t + 1]);
}

// The weights of 8 keys as a B operand (and their second 16-bit term: p = hi + lo, lo = round(p - hi)).
template <bool PRECISE, typename E>
__device__ __forceinline__ void pack_weights(uint4& w, uint4& wl, const f32x16& s, int r0)
{
    w.x = E::pack(s[r0 + 0], s[r0 + 1]);
    w.y = E::pack(s[r0 + 2], s[r0 + 3]);
    w.z = E::pack(s[r0 + 4], s[r0 + 5]);
    w.w = E::pack(s[r0 + 6], s[r0 + 7]);
    if (PRECISE) {
        wl.x = E::pack(s[r0 + 0] - E::lo_of(w.x), s[r0 + 1] - E::hi_of(w.x));
        wl.y = E::pack(s[r0 + 2] - E::lo_of(w.y), s[r0 + 3] - E::hi_of(w.y));
        wl.z = E::pack(s[r0 + 4] - E::lo_of(w.z), s[r0 + 5] - E::hi_of(w.z));
        wl.w = E::pack(s[r0 + 6] - E::lo_of(w.w), s[r0 + 7] - E::hi_of(w.w));
    } else {
        wl = w;
    }
}

// O^T += V^T P^T for the 32 keys of a half tile whose fragments load_v_frags brought.  P^T as B operand of a step:
// elements e = 0..7 <-> weights 8*step + e.
template <bool PRECISE, typename E, int T>
__device__ __forceinline__ void half_pv_frags(f32x16 (&o)[T], const f32x16& s, const uint4 (&va)[T], const uint4 (&vb)[T])
{
#pragma unroll
    for (int st = 0; st < 2; ++st) {
        uint4 w, wl;
        pack_weights<PRECISE, E>(w, wl, s, 8 * st);
        const uint4 (&cur)[T] = st ? vb : va;
#pragma unroll
        for (int t = 0; t < T; ++t) {
            o[t] = E::mfma32(cur[t], w, o[t]);
            if (PRECISE) o[t] = E::mfma32(cur[t], wl, o[t]);
        }
    }
}

// O^T += V^T P^T for the 32 keys of half tile `half` (two 16-key steps), head_dim 256: the second step's fragments
// take the place of the first step's as those are consumed (the 8 column blocks leave no room to hold both).
// vbuf = V part of the tile buffer.
template <bool PRECISE, typename E, int T>
__device__ __forceinline__ void half_pv(f32x16 (&o)[T], const f32x16& s, const char* vbuf, int half,
                                        const uint32_t (&vx)[2 * T])
{
    constexpr int RB = 512;
    uint4 va[T];
    const char* v0 = vbuf + (32 * half) * RB;
#pragma unroll
    for (int t = 0; t < T; ++t) va[t] = lds_frag_tr(v0 + vx[2 * t], v0 + vx[2 * t + 1]);
#pragma unroll
    for (int st = 0; st < 2; ++st) {
        uint4 w, wl;
        pack_weights<PRECISE, E>(w, wl, s, 8 * st);
#pragma unroll
        for (int t = 0; t < T; ++t) {
            o[t] = E::mfma32(va[t], w, o[t]);
            if (PRECISE) o[t] = E::mfma32(va[t], wl, o[t]);
            if (st == 0) va[t] = lds_frag_tr(v0 + 16 * RB + vx[2 * t], v0 + 16 * RB + vx[2 * t + 1]);
        }
    }
}

// S^T of half tile `half` (32 keys) against the wave's 32 queries: 8 chained matrix instructions, the K operand
// reads kept four ahead.  kx[ks] = this lane's swizzled operand offset for head_dim step ks.
template <typename E, int KS>
__device__ __forceinline__ void half_scores(f32x16& s, const char* kbuf, int half, const uint32_t (&kx)[KS],
                                            const uint4 (&qf)[KS])
{
    constexpr int RB = KS > 8 ? 512 : 256;
    s = (f32x16)(0.f);   // folded into the first matrix instruction's accumulator operand
    const char* kh = kbuf + (32 * half) * RB;
    uint4 ka[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) ka[i] = lds_frag(kh + kx[i]);
#pragma unroll
    for (int i = 0; i < KS; ++i) {
        s = E::mfma32(ka[i & 3], qf[i], s);
        if (i + 4 < KS) ka[i & 3] = lds_frag(kh + kx[i + 4]);
    }
}

// One 64-key tile for one wave, processed as two half tiles of 32 keys so that, within the wave, the softmax of
// one half (vector ALU) runs under the matrix instructions of the other half:
//     matrix cores:  S(h0)   S(h1)          PV(h0)          PV(h1)
//     vector ALU:            softmax(h0)    softmax(h1)
// buf = tile buffer (K rows, then V rows); key0 = first key of the tile + 4 * (lane/32); nk = keys this lane's
// query may see (MASK only); sc = scale * log2(e) > 0.
template <bool PRECISE, bool MASK, typename E, typename M, int T>
__device__ __forceinline__ void attend_tile(const char* buf, const uint32_t (&kx)[2 * T], const uint32_t (&vx)[2 * T],
                                            const uint4 (&qf)[2 * T], f32x16 (&o)[T], float& m, float& l, float sc,
                                            int32_t key0, int32_t nk, const RowMods& rm, const int32_t* docs)
{
    f32x16 s0, s1, p;
    constexpr int TB = kBN * (T > 4 ? 512 : 256);
    if constexpr (T <= 4) {
        uint4 va[T], vb[T];
        half_scores<E, 2 * T>(s0, buf, 0, kx, qf);
        half_scores<E, 2 * T>(s1, buf, 1, kx, qf);
        load_v_frags<T>(va, vb, buf + TB, 0, vx);
        half_softmax<MASK, true, M, T>(p, s0, o, m, l, sc, key0, nk, rm, docs);
        half_pv_frags<PRECISE, E, T>(o, p, va, vb);
        load_v_frags<T>(va, vb, buf + TB, 1, vx);
        half_softmax<MASK, false, M, T>(p, s1, o, m, l, sc, key0 + 32, nk, rm, docs + 32);
        half_pv_frags<PRECISE, E, T>(o, p, va, vb);
    } else {
        half_scores<E, 2 * T>(s0, buf, 0, kx, qf);
        half_scores<E, 2 * T>(s1, buf, 1, kx, qf);
        half_softmax<MASK, true, M, T>(p, s0, o, m, l, sc, key0, nk, rm, docs);
        half_pv<PRECISE, E, T>(o, p, buf + TB, 0, vx);
        half_softmax<MASK, false, M, T>(p, s1, o, m, l, sc, key0 + 32, nk, rm, docs + 32);
        half_pv<PRECISE, E, T>(o, p, buf + TB, 1, vx);
    }
}

// Query range and context length of the sequence a workgroup works on.
struct OwnLengths {
    int32_t q_begin, q_end, len;
};

template <bool PRECISE, bool UNIFORM, typename E, typename M, int D>
__device__ __forceinline__ void prefill_body(
    char* buf0, char* buf1, int32_t* docs0, int32_t* docs1, const CacheView& cache, const uint16_t* __restrict__ q, uint16_t* __restrict__ out, float* __restrict__ lse,
    const int32_t* __restrict__ cu_q_lens, const int32_t* __restrict__ block_table,
    const int32_t* __restrict__ seq_lens, int32_t batch, int32_t num_tiles, int32_t num_q_heads, int32_t max_blocks,
    float scale, int32_t causal, const PrefillPlan& plan, int32_t precise_keys, const OwnLengths& own)
{
    constexpr int KS = D / 16, T = D / 32;               // steps of a score product, 32-column blocks of O
    constexpr int RB = RowGeo<D>::kRowB;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int ql = lane & 31, hh = lane >> 5;
    // Rows of a workgroup's 128-row tile are (query, head) pairs: the 2^log2_pack query heads packed into a tile
    // share one KV head, row r of a sequence is query r >> log2_pack, packed head r & (pack - 1).
    const int32_t lg = plan.log2_pack;
    const int32_t heads = num_q_heads >> lg;                 // head groups along the grid
    // Workgroups are dispatched in blockIdx.x order: the row-tile index is the slowest-varying part and runs
    // backwards, so the whole grid is handed out heaviest (latest causal tiles) first; the context chunks of a
    // tile follow each other.
    const int32_t hb = heads * batch;
    const int32_t slow = (int32_t)(blockIdx.x / hb);
    const int32_t tile = num_tiles - 1 - slow / plan.nsplit;
    const int32_t split = slow % plan.nsplit;
    const int32_t rest = blockIdx.x % hb;
    const int32_t s = rest / heads;
    const int32_t hg = rest % heads;
    const int32_t q_begin = own.q_begin;                     // (this sequence's lengths: fetched by the kernel ahead of
    const int32_t q_len = own.q_end - own.q_begin;           //  everything else, see there)
    const int32_t n_rows = q_len << lg;
    const int32_t m0 = tile * kBM;
    if (m0 >= n_rows) return;
    if (plan.skip_small && q_len * (num_q_heads / cache.num_kv_heads) <= 16) return;
    const int32_t len = own.len;
    // workgroup-wide key range; it also selects which instantiation handles this tile
    const int32_t q_last = (min(m0 + kBM, n_rows) - 1) >> lg;
    int32_t nk_wg = len;
    if (causal) nk_wg = min(len, len - q_len + q_last + 1);
    nk_wg = max(nk_wg, 0);
    // sliding window: |key - pos| < window.  The workgroup starts at the 64-aligned key before the window of its
    // first row and, without a causal bound, ends with the window of its last row.
    const int32_t window = (M::kWindow && plan.mods.window > 0) ? plan.mods.window : 0;
    int32_t k_lo = 0;
    if (window > 0) {
        k_lo = max(len - q_len + (m0 >> lg) - window + 1, 0) & ~(kBN - 1);
        if (!causal) nk_wg = max(min(nk_wg, len - q_len + q_last + window), 0);
    }
    // Few effective keys mean few, large weights whose 16-bit rounding shows: rows that see far fewer keys than the
    // call's rows do on (harmonic) average (precise_keys, see precise_key_bound), short contexts and windows, and any
    // position bias (a steep slope concentrates the weight on a handful of keys however long the context is).
    // (a document mask can leave a row a handful of keys out of any context)
    int32_t n_first = len;                                   // keys the tile's first row sees
    if (causal) n_first = min(len, len - q_len + (m0 >> lg) + 1);
    if (window > 0) n_first = min(n_first, causal ? window : 2 * window - 1);
    const bool few_keys = n_first <= precise_keys ||
                          (M::kScore && plan.mods.alibi_slopes != nullptr) || (M::kDoc && plan.mods.doc_ids != nullptr) ||
                          M::kUser;
    if (few_keys != PRECISE) return;                        // the other instantiation handles this tile
    // this workgroup's chunk of the context; with a split, chunks without keys leave nothing behind (the merge
    // reads only the chunks that hold keys of a row)
    // (without a causal bound a window also cuts the END of a row's range, which the merge does not know: those
    // chunks must leave explicit empty partials, so the workgroup goes on with zero tiles)
    if (plan.nsplit > 1 && split * plan.chunk >= nk_wg && !(window > 0 && !causal)) return;
    const int32_t k_begin = max(split * plan.chunk, k_lo);
    const int32_t k_end = min(nk_wg, split * plan.chunk + plan.chunk);

    const int32_t G = num_q_heads / cache.num_kv_heads;
    const int32_t* table = block_table + (int64_t)s * max_blocks;

    // this lane's row: query, head, and key bound
    const int32_t r_lane = m0 + 32 * wave + ql;
    const bool q_valid = r_lane < n_rows;
    const int32_t r_c = min(r_lane, n_rows - 1);
    const int32_t qi_c = r_c >> lg;
    const int32_t h = (hg << lg) + (r_c & ((1 << lg) - 1));
    const int32_t kvh = (hg << lg) / G;
    const int32_t pos = len - q_len + qi_c;                  // the row's absolute position
    int32_t nk = len;                                        // keys 0 .. nk-1 are allowed
    if (causal) nk = min(len, pos + 1);
    else if (window > 0) nk = min(len, pos + window);
    nk = max(nk, 0);
    // per wave: the largest bound of its 32 rows decides which tiles it can skip, the smallest which
    // tiles need no mask
    const int32_t pos_first = len - q_len + (min(m0 + 32 * wave, n_rows - 1) >> lg);
    const int32_t pos_last = len - q_len + (min(m0 + 32 * wave + 31, n_rows - 1) >> lg);
    int32_t nk_wave = len, nk_wave_min = len;
    if (causal) {
        nk_wave = min(len, pos_last + 1);
        nk_wave_min = min(len, pos_first + 1);
    } else if (window > 0) {
        nk_wave = min(len, pos_last + window);
        nk_wave_min = min(len, pos_first + window);
    }
    nk_wave = max(nk_wave, 0);
    nk_wave_min = max(nk_wave_min, 0);
    RowMods rm;
    rm.lo = 0;
    rm.lo_until = 0;
    rm.pos = pos;
    rm.slope2 = 0.f;
    rm.cap_in = 0.f;
    rm.cap_out = 0.f;
    rm.doc = 0;
    const int32_t* doc_row = nullptr;
    if (M::kDoc && plan.mods.doc_ids) {
        doc_row = plan.mods.doc_ids + (int64_t)s * plan.mods.doc_stride;
        rm.doc = doc_row[max(pos, 0)];
    }
    rm.uc = pa_mod_ctx{plan.mods.user_data, s, h, pos, len};
    int32_t lo_wave = 0;                                     // tiles that end at or before it hold nothing for the wave
    if (window > 0) {
        rm.lo = pos - window + 1;
        rm.lo_until = pos_last - window + 1;
        lo_wave = pos_first - window + 1;
    }
    if (M::kScore) {
        if (plan.mods.alibi_slopes) rm.slope2 = plan.mods.alibi_slopes[h] * kLog2e;
        if (plan.mods.softcap > 0.f) {
            rm.cap_in = scale / plan.mods.softcap;
            rm.cap_out = plan.mods.softcap * kLog2e;
        }
    }

    const int64_t row = (int64_t)(q_begin + qi_c) * num_q_heads + h;
    // Q as B operand: lane%32 = query, step ks covers head_dim elements 16*ks + 8*hh .. +7
    uint4 qf[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qf[ks] = *reinterpret_cast<const uint4*>(q + row * D + 16 * ks + 8 * hh);

    f32x16 o[T];
#pragma unroll
    for (int t = 0; t < T; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[t][r] = 0.f;
    float m = -INFINITY, l = 0.f;
    const float sc = scale * kLog2e;

    // swizzled LDS offsets of this lane's operands (see the header): K piece (2*ks + hh) of row ql,
    // V pieces of the 32 columns t for the lane's transpose-load row
    uint32_t kx[KS], vx[2 * T];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) kx[ks] = ql * RB + piece_pos(2 * ks + hh, ql);
    {
        // transpose-load rows of this lane: key 4*hh + j (+8 for slots 4-7) of a 16-key step, columns 4*qq..+3 of
        // the 16-column block dblk of the 32 columns t
        const int j = (lane & 15) >> 2, qq = lane & 3, dblk = (lane >> 4) & 1;
#pragma unroll
        for (int t = 0; t < T; ++t) {
            const int piece = 4 * t + 2 * dblk + (qq >> 1);
            vx[2 * t] = (4 * hh + j) * RB + piece_pos(piece, 4 * hh + j) + 8 * (qq & 1);
            vx[2 * t + 1] = (4 * hh + j + 8) * RB + piece_pos(piece, 4 * hh + j + 8) + 8 * (qq & 1);
        }
    }
    // fetch role of this lane.  256-byte rows: position lane%16 of rows 16*i + frow holds logical piece
    // (lane%16) ^ swz(frow) (a row of head_dim 64 has 8 pieces: the other 8 positions receive repeats that nobody
    // reads).  512-byte rows: position lane%32 of rows 8*i + frow; the swizzle of that row depends on the parity of i.
    const int frow = D > 128 ? 2 * wave + (lane >> 5) : 4 * wave + (lane >> 4);
    const uint32_t head_off = (uint32_t)(kvh * cache.head_stride * 2);
    const uint32_t lane_off = head_off + 16 * (((lane & 15) ^ swz(frow)) & (D / 8 - 1));
    uint32_t lane_off2[2];
#pragma unroll
    for (int par = 0; par < 2; ++par)
        lane_off2[par] = head_off + 16 * ((lane & 16) | ((lane & 15) ^ swz(8 * par + frow)));
    const int32_t wrow = __builtin_amdgcn_readfirstlane(D > 128 ? 2 * wave * 512 : 4 * wave * 256);
    const int32_t last_key = len - 1;
    const uint32_t lds0 = lds_address(buf0 + wrow), lds1 = lds_address(buf1 + wrow);
    auto fetch = [&](uint32_t lds, const PageIds& pg, int32_t t0) {
        if constexpr (D > 128) fetch_tile512<UNIFORM>(lds, pg, cache, t0, frow, last_key, lane_off2);
        else fetch_tile<UNIFORM>(lds, pg, cache, t0, frow, last_key, lane_off);
    };

    // Document masks: wave 0 brings the 64 ids of the next tile (one per lane) and stores them next to the tile
    // buffer before the barrier that publishes the tile, together with their minimum and maximum (slots 64, 65).
    // A wave skips a tile whose id range misses the id range of its rows: always right, and it pays when documents
    // are contiguous runs of positions, as in packed batches.  (The tile is still fetched: deciding that ahead of
    // the fetch costs a dependent global load per tile, which was measured to cost more than the fetches it saves.)
    const bool doc_lane = M::kDoc && wave == 0;
    int32_t doc_next = 0;
    int32_t row_doc_min = rm.doc, row_doc_max = rm.doc;
    // minimum and maximum over the wave with data-parallel-primitive moves: shifts by 1, 2, 4, 8 inside each row
    // of 16 lanes, then lane 15 of a row into the next row, lane 31 into the upper half; lane 63 holds the result
    auto wave_range = [&](int32_t v, int32_t& mn, int32_t& mx) {
        mn = v;
        mx = v;
#define PA_RANGE_STEP(CTRL, ROWS)                                                                   \
        mn = min(mn, __builtin_amdgcn_update_dpp(mn, mn, CTRL, ROWS, 0xF, false));                  \
        mx = max(mx, __builtin_amdgcn_update_dpp(mx, mx, CTRL, ROWS, 0xF, false));
        PA_RANGE_STEP(0x111, 0xF) PA_RANGE_STEP(0x112, 0xF) PA_RANGE_STEP(0x114, 0xF) PA_RANGE_STEP(0x118, 0xF)
        PA_RANGE_STEP(0x142, 0xA) PA_RANGE_STEP(0x143, 0xC)
#undef PA_RANGE_STEP
        mn = __builtin_amdgcn_readlane(mn, 63);
        mx = __builtin_amdgcn_readlane(mx, 63);
    };
    auto put_docs = [&](int32_t* dst, int32_t v) {           // wave 0: the tile's ids and their range
        int32_t mn, mx;
        wave_range(v, mn, mx);
        dst[lane] = v;
        if (lane < 2) dst[kBN + lane] = lane ? mx : mn;
    };
    auto docs_overlap = [&](const int32_t* d) -> bool {      // wave-uniform
        if (!M::kDoc) return true;
        const int32_t mn = __builtin_amdgcn_readfirstlane(d[kBN]);
        const int32_t mx = __builtin_amdgcn_readfirstlane(d[kBN + 1]);
        return mx >= row_doc_min && mn <= row_doc_max;
    };
    auto tile_ids = [&](int32_t t0) -> int32_t { return doc_row ? doc_row[min(t0 + lane, last_key)] : 0; };
    if (M::kDoc) wave_range(rm.doc, row_doc_min, row_doc_max);
    PageIds ids;
    const int32_t n_tiles = (max(k_end - k_begin, 0) + kBN - 1) / kBN;
    if (n_tiles > 0) {
        load_ids<UNIFORM>(ids, cache, table, k_begin, frow, last_key);
        fetch(lds0, ids, k_begin);
        if (doc_lane) put_docs(docs0, tile_ids(k_begin));
        if (n_tiles > 1) load_ids<UNIFORM>(ids, cache, table, k_begin + kBN, frow, last_key);
    }
    wait_tile_loads();                                       // (outside the test: the loop below must start from a
    __syncthreads();                                         //  state without pending loads on every path)
    // Two tiles per trip so that each buffer is a distinct LDS object for the compiler: while the matrix cores
    // read one, the load unit fills the other with the next tile; the page ids of the tile after that are requested
    // at the same time.  The barrier at the end of a tile waits for this wave's loads first.
    for (int32_t t = 0; t < n_tiles; t += 2) {
        const int32_t t0 = k_begin + t * kBN;
        if (t + 1 < n_tiles) {
            fetch(lds1, ids, t0 + kBN);
            if (doc_lane) doc_next = tile_ids(t0 + kBN);
            if (t + 2 < n_tiles) load_ids<UNIFORM>(ids, cache, table, t0 + 2 * kBN, frow, last_key);
        }
        if (t0 < nk_wave && t0 + kBN > lo_wave && docs_overlap(docs0)) {   // wave-uniform: else nothing for this wave here
            if (t0 + kBN > nk_wave_min)                      // wave-uniform: some score of this tile is masked
                attend_tile<PRECISE, true, E, M, T>(buf0, kx, vx, qf, o, m, l, sc, t0 + 4 * hh, nk, rm, docs0 + 4 * hh);
            else
                attend_tile<PRECISE, false, E, M, T>(buf0, kx, vx, qf, o, m, l, sc, t0 + 4 * hh, nk, rm, docs0 + 4 * hh);
        }
        if (doc_lane && t + 1 < n_tiles) put_docs(docs1, doc_next);
        wait_tile_loads();
        __syncthreads();
        if (t + 1 >= n_tiles) break;
        const int32_t t1 = t0 + kBN;
        if (t + 2 < n_tiles) {
            fetch(lds0, ids, t1 + kBN);
            if (doc_lane) doc_next = tile_ids(t1 + kBN);
            if (t + 3 < n_tiles) load_ids<UNIFORM>(ids, cache, table, t1 + 2 * kBN, frow, last_key);
        }
        if (t1 < nk_wave && t1 + kBN > lo_wave && docs_overlap(docs1)) {
            if (t1 + kBN > nk_wave_min)
                attend_tile<PRECISE, true, E, M, T>(buf1, kx, vx, qf, o, m, l, sc, t1 + 4 * hh, nk, rm, docs1 + 4 * hh);
            else
                attend_tile<PRECISE, false, E, M, T>(buf1, kx, vx, qf, o, m, l, sc, t1 + 4 * hh, nk, rm, docs1 + 4 * hh);
        }
        if (doc_lane && t + 2 < n_tiles) put_docs(docs0, doc_next);
        wait_tile_loads();
        __syncthreads();
    }

    l += __shfl_xor(l, 32, 64);
    if (!q_valid) return;
    const float inv = l > 0.f ? 1.f / l : 0.f;
    // o[t][r]: column 32*t + 8*(r/4) + 4*hh + r%4 of this lane's query
    if (plan.nsplit > 1) {
        // partial of this chunk: normalised output in fp32 and the natural-log LSE over the chunk's keys
        const int64_t pidx = row * plan.nsplit + split;
        float* prow = plan.part_o + pidx * D;
#pragma unroll
        for (int t = 0; t < T; ++t)
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                float4 w;
                w.x = o[t][4 * a + 0] * inv;
                w.y = o[t][4 * a + 1] * inv;
                w.z = o[t][4 * a + 2] * inv;
                w.w = o[t][4 * a + 3] * inv;
                *reinterpret_cast<float4*>(prow + 32 * t + 8 * a + 4 * hh) = w;
            }
        if (hh == 0) plan.part_lse[pidx] = l > 0.f ? (m + __builtin_amdgcn_logf(l)) * kLn2 : -INFINITY;
        return;
    }
    uint16_t* orow = out + row * D;
#pragma unroll
    for (int t = 0; t < T; ++t)
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            uint2 w;
            w.x = E::pack(o[t][4 * a + 0] * inv, o[t][4 * a + 1] * inv);
            w.y = E::pack(o[t][4 * a + 2] * inv, o[t][4 * a + 3] * inv);
            *reinterpret_cast<uint2*>(orow + 32 * t + 8 * a + 4 * hh) = w;
        }
    if (lse && hh == 0) lse[row] = l > 0.f ? (m + __builtin_amdgcn_logf(l)) * kLn2 : -INFINITY;
}

// Both instantiations live in one kernel as two separate code paths (each with its own tile loop); a
// workgroup runs exactly one of them, decided by its context length.
template <bool UNIFORM, typename E, typename M, int D>
__global__ __launch_bounds__(kThreads, D > 128 ? 1 : 2) void paged_prefill_mfma_kernel(
    CacheView cache, const uint16_t* __restrict__ q, uint16_t* __restrict__ out, float* __restrict__ lse,
    const int32_t* __restrict__ cu_q_lens, const int32_t* __restrict__ block_table,
    const int32_t* __restrict__ seq_lens, int32_t batch, int32_t num_tiles, int32_t num_q_heads, int32_t max_blocks,
    float scale, int32_t causal, PrefillPlan plan)
{
    __shared__ __attribute__((aligned(1024))) char buf0[RowGeo<D>::kBufB];
    __shared__ __attribute__((aligned(1024))) char buf1[RowGeo<D>::kBufB];
    __shared__ __attribute__((aligned(16))) int32_t docs0[kBN + 4];
    __shared__ __attribute__((aligned(16))) int32_t docs1[kBN + 4];
    // The workgroup's own lengths are requested first (scalar loads), the scan of every sequence's lengths for the
    // two-term rule right behind them (vector loads): one round trip to memory instead of three in a row in front
    // of the query and block-table loads that depend on them.
    OwnLengths own;
    {
        const int32_t heads = num_q_heads >> plan.log2_pack;
        const int32_t s = (int32_t)(blockIdx.x % (uint32_t)(heads * batch)) / heads;
        own.q_begin = cu_q_lens[s];
        own.q_end = cu_q_lens[s + 1];
        own.len = seq_lens[s];
    }
    const int32_t precise_keys = precise_key_bound(cu_q_lens, seq_lens, batch, causal,
                                                   (M::kWindow && plan.mods.window > 0) ? plan.mods.window : 0,
                                                   (int)(threadIdx.x & 63));
    prefill_body<false, UNIFORM, E, M, D>(buf0, buf1, docs0, docs1, cache, q, out, lse, cu_q_lens, block_table, seq_lens, batch, num_tiles,
                                 num_q_heads, max_blocks, scale, causal, plan, precise_keys, own);
    prefill_body<true, UNIFORM, E, M, D>(buf0, buf1, docs0, docs1, cache, q, out, lse, cu_q_lens, block_table, seq_lens, batch, num_tiles,
                                num_q_heads, max_blocks, scale, causal, plan, precise_keys, own);
}

}  // namespace

// Every kernel instantiation of one head_dim; defined in that head_dim's translation unit.
template <int D>
pa_status launch_prefill_mfma_dim(const AttnArgs& a, const PrefillPlan& plan, int64_t blocks, int64_t tiles,
                                  hipStream_t stream)
{
    const dim3 grid((uint32_t)blocks, 1, 1);
    // page sizes of 16 and more make the page of a 16-key group wave-uniform (scalar page translation)
    const bool uniform = a.cache.page_size >= 16;
    if (D > 128 && !uniform) return PA_ERR_UNSUPPORTED;   // 512-byte rows: two rows per load must share a page
    typedef Mods<true, true, false> WindowScore;
    auto kern = paged_prefill_mfma_kernel<true, ElemBf16, NoMods, D>;
    if (a.mods.user_mod) {                                // a user modification: one instantiation per listed struct
        bool found = false;
#define PA_USER_CASE(U)                                                                                     \
        if (a.mods.user_mod == U::kId) {                                                                    \
            typedef Mods<true, true, true, U> UM;                                                           \
            found = true;                                                                                   \
            if (a.dtype == PA_DTYPE_BF16)                                                                   \
                kern = uniform ? paged_prefill_mfma_kernel<true, ElemBf16, UM, D>                           \
                               : paged_prefill_mfma_kernel<false, ElemBf16, UM, D>;                         \
            else                                                                                            \
                kern = uniform ? paged_prefill_mfma_kernel<true, ElemF16, UM, D>                            \
                               : paged_prefill_mfma_kernel<false, ElemF16, UM, D>;                          \
        }
        PA_USER_MODS(PA_USER_CASE)
#undef PA_USER_CASE
        if (!found) return PA_ERR_INVALID_ARG;
    } else if (a.has_mods && a.mods.doc_ids) {
        if (a.dtype == PA_DTYPE_BF16)
            kern = uniform ? paged_prefill_mfma_kernel<true, ElemBf16, AllMods, D>
                           : paged_prefill_mfma_kernel<false, ElemBf16, AllMods, D>;
        else
            kern = uniform ? paged_prefill_mfma_kernel<true, ElemF16, AllMods, D>
                           : paged_prefill_mfma_kernel<false, ElemF16, AllMods, D>;
    } else if (a.dtype == PA_DTYPE_BF16) {
        if (a.has_mods) kern = uniform ? paged_prefill_mfma_kernel<true, ElemBf16, WindowScore, D>
                                       : paged_prefill_mfma_kernel<false, ElemBf16, WindowScore, D>;
        else if (!uniform) kern = paged_prefill_mfma_kernel<false, ElemBf16, NoMods, D>;
    } else {
        if (a.has_mods) kern = uniform ? paged_prefill_mfma_kernel<true, ElemF16, WindowScore, D>
                                       : paged_prefill_mfma_kernel<false, ElemF16, WindowScore, D>;
        else kern = uniform ? paged_prefill_mfma_kernel<true, ElemF16, NoMods, D>
                            : paged_prefill_mfma_kernel<false, ElemF16, NoMods, D>;
    }
    hipLaunchKernelGGL(kern, grid, dim3(kThreads), 0, stream, a.cache, (const uint16_t*)a.q, (uint16_t*)a.out, a.lse,
                       a.cu_q_lens, a.block_table, a.seq_lens, a.batch, (int32_t)tiles, a.num_q_heads, a.max_blocks,
                       a.scale, a.causal, plan);
    return launch_status();
}

}  // namespace pa
