// Split-KV paged decode for bf16 / fp16 pools with head_dim D = 64, 128 or 256 on gfx950 (CDNA4); 16 query heads
// of a KV head per wave (larger groups take ceil(G/16) workgroups per tile range, which re-read K/V through L2).
// Internal header: the kernel templates; one translation unit per head_dim instantiates them.
// (The description below is written for D = 128; what changes with D is listed at Geo.)
//
// Decode is bound by streaming every resident K/V byte once from HBM, so the design is about memory:
//   * one wave owns one KV head of one (sequence, context chunk); the NW waves of a workgroup own NW
//     adjacent KV heads and meet at a barrier before every tile load, so that together, and at the same time,
//     they read whole contiguous token rows of a page;
//   * each wave walks its chunk in tiles of 32 keys; every K/V byte is fetched by one 16-byte load per
//     lane straight into the registers the MFMA reads -- no LDS round trip -- and the next tile's 16
//     loads (16 KB per wave) are in flight while the current tile is computed;
//   * page translation (Algorithm 1: page = block_table[s][j >> log2 P], slot = j & (P-1)) is wave-uniform
//     for P >= 16, i.e. scalar: page base in SGPRs plus loop-invariant per-lane offsets.
// The G grouped query heads turn q.K^T and P.V into small dense contractions, which run on the matrix
// cores (v_mfma_f32_16x16x32_bf16, G padded to 16 columns):
//   S^T[key, head] = K[key, :] . Q[head, :]^T    A = K rows exactly as loaded (lane%16 = key)
//   O^T[dcol, head] += V^T[dcol, key] . P^T[key, head]
// For P.V the contraction index is the key, while memory is contiguous along head_dim.  Each lane loads
// 8 keys x 8 head_dim columns and transposes that 8x8 block of 16-bit values in its own registers with
// 32 byte-permutes; since any key order is valid for a sum, the 8 keys a lane holds are chosen to be the
// ones whose probabilities the S^T accumulator layout already left in the matching lanes.
// Softmax statistics are lane-local per head (lane%16 = head in both accumulators); the only cross-lane
// traffic is a 4-way max per tile and one 4-way sum at the end.
// Two kernels share the tile code: paged_decode_mfma_kernel (the batch's context as one stream of tiles cut evenly
// over the workgroups, partials merged by a second launch) and paged_decode_short_kernel (short contexts: one
// workgroup per sequence and KV head, its waves split the context and merge through LDS, one launch).  Both exist
// in a variant that also performs the decode step's append of one new token per sequence (FUSED).
#pragma once

#include "common.h"

namespace pa {

namespace {

typedef mfma_f32x4 f32x4;

// Tile geometry per head_dim.  A wave's tile is kBlocks blocks of 16 keys; a K row is read in KS steps of 32
// elements; a lane's V loads cover 4 keys of each of kVBlocks blocks and kPasses 16-byte column pieces (piece =
// lane%16 + 16*pass).
//   D = 64:  rows hold 8 pieces, so only 8 of every 16 lanes can differ in piece.  Lanes 8-15 therefore load the V rows
//            of a SECOND pair of blocks (a tile is 64 keys: blocks 0, 1 for lanes 0-7, blocks 2, 3 for lanes 8-15) --
//            every load brings bytes nobody else loads -- and the value product runs twice per column, once as loaded
//            with the weights of blocks 0, 1 and once with the two lane halves swapped (a DPP rotate by 8) with the
//            weights of blocks 2, 3; accumulator rows 8-15 gather products of mismatched halves and are never stored.
//   D = 256: two column passes; tiles of 16 keys keep two tiles in registers (the second block's contraction slots
//            carry zero weights and zero values).
template <int D>
struct Geo {
    static constexpr int kD = D;
    static constexpr int kKS = D / 32;
    static constexpr int kBlocks = D == 256 ? 1 : D == 64 ? 4 : 2;
    static constexpr int kVBlocks = D == 256 ? 1 : 2;
    static constexpr int kTileKeys = 16 * kBlocks;
    static constexpr int kPasses = D == 256 ? 2 : 1;
    static constexpr int kPieceMask = D == 64 ? 7 : 15;
};
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

__device__ __forceinline__ uint4 load16(const char* p) { return *reinterpret_cast<const uint4*>(p); }

__device__ __forceinline__ uint32_t word(const uint4& v, int w)
{
    return w == 0 ? v.x : w == 1 ? v.y : w == 2 ? v.z : v.w;
}

template <typename GE>
struct Tile {
    uint4 k[GE::kBlocks][GE::kKS];        // [16-key block][32-element step of head_dim]: lane%16 = key, lane/16 = 8-element piece
    uint4 v[GE::kPasses][4 * GE::kVBlocks];  // 4 keys per block x 8 head_dim columns per lane and pass
    int32_t doc[GE::kBlocks][4];             // document ids of the lane's 4 score keys per block (document masks only)
};

// Everything a wave needs to address its KV head's rows.
struct Addr {
    const char* kbase;          // pool base + kv head offset
    const char* vbase;
    const int32_t* table;       // block-table row of the sequence
    const int32_t* doc;         // document-id row of the sequence (document masks only)
    int64_t page_bytes;
    int64_t token_bytes;
    int32_t log2_page;
    int32_t pmask;
    uint32_t koff;              // UNIFORM: lane-invariant byte offset of the lane's K piece inside a 16-key block
    uint32_t voff[4];           // UNIFORM: same for the lane's 4 V rows of a 16-key block
    int32_t r16, quad;
    // FUSED (the step's new token is appended by the same kernel): the K / V rows of key new_pos are read from
    // the new token's rows (k_new / v_new of this sequence and KV head) instead of the pool
    const char* knew;
    const char* vnew;
    int32_t new_pos;
    // PRE (a wave that knows its whole key range up front): lane i holds block-table entry ids_base + i, so a
    // tile's page id is a lane read instead of a dependent load in front of the tile's row loads
    int32_t ids;
    int32_t ids_base;
};

// Issue the 16 loads of the tile that starts at key `t0`.  Keys at or beyond `c1` are clamped to the last
// valid key, so every address is a live slot; their scores are masked by the caller.
template <bool UNIFORM, typename M, typename GE, bool FUSED = false, bool PRE = false>
__device__ __forceinline__ void load_tile(Tile<GE>& t, const Addr& a, int32_t t0, int32_t c1)
{
    constexpr int kTileKeys = GE::kTileKeys;
    if (M::kDoc) {   // ids of the keys whose scores this lane will hold (clamped like the rows themselves)
#pragma unroll
        for (int mt = 0; mt < GE::kBlocks; ++mt)
#pragma unroll
            for (int i = 0; i < 4; ++i)
                t.doc[mt][i] = a.doc ? a.doc[min(t0 + 16 * mt + 4 * a.quad + i, c1 - 1)] : 0;   // no ids: one document
    }
    // which of the tile's blocks this lane's V loads belong to: block mt for lanes 0-7 of 16 and, at head_dim 64,
    // block mt + 2 for lanes 8-15
    const int32_t vshift = (GE::kD == 64) ? 2 * (a.r16 >> 3) : 0;
    if constexpr (UNIFORM) {
        if (t0 + kTileKeys <= c1) {   // full tile: 16-key blocks, each inside one page
            int64_t blk[GE::kBlocks];                          // byte offset of each block's first row in its pool
#pragma unroll
            for (int mt = 0; mt < GE::kBlocks; ++mt) {
                const int32_t kb = t0 + 16 * mt;
                int64_t page;
                const int32_t rel = (kb >> a.log2_page) - a.ids_base;    // wave-uniform
                if (PRE && rel < 64)
                    page = __builtin_amdgcn_readlane(a.ids, rel);
                else
                    page = __builtin_amdgcn_readfirstlane(a.table[kb >> a.log2_page]);
                blk[mt] = page * a.page_bytes + (int64_t)(kb & a.pmask) * a.token_bytes;
            }
#pragma unroll
            for (int mt = 0; mt < GE::kBlocks; ++mt) {
                const int32_t kb = t0 + 16 * mt;
                const char* kp = a.kbase + blk[mt];
                const char* kl = (FUSED && kb + a.r16 == a.new_pos) ? a.knew + a.quad * 16 : kp + a.koff;
#pragma unroll
                for (int ks = 0; ks < GE::kKS; ++ks) t.k[mt][ks] = load16(kl + 64 * ks);
            }
#pragma unroll
            for (int mt = 0; mt < GE::kVBlocks; ++mt) {
                const char* vp = a.vbase + blk[mt];
                if constexpr (GE::kD == 64) {
                    if (vshift) vp = a.vbase + blk[mt + 2];
                }
                const int32_t kb = t0 + 16 * (mt + vshift);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const char* vl = (FUSED && kb + 4 * a.quad + i == a.new_pos) ? a.vnew + (a.r16 & GE::kPieceMask) * 16
                                                                                 : vp + a.voff[i];
#pragma unroll
                    for (int c = 0; c < GE::kPasses; ++c) t.v[c][4 * mt + i] = load16(vl + 256 * c);
                }
            }
            return;
        }
    }
    // ragged tail (or page size below 16): per-lane translation of clamped keys
    const int32_t last = c1 - 1;
#pragma unroll
    for (int mt = 0; mt < GE::kBlocks; ++mt) {
        const int32_t key = min(t0 + 16 * mt + a.r16, last);
        const int64_t page = a.table[key >> a.log2_page];
        const char* kp = a.kbase + page * a.page_bytes + (int64_t)(key & a.pmask) * a.token_bytes + a.quad * 16;
        if (FUSED && key == a.new_pos) kp = a.knew + a.quad * 16;
#pragma unroll
        for (int ks = 0; ks < GE::kKS; ++ks) t.k[mt][ks] = load16(kp + 64 * ks);
    }
#pragma unroll
    for (int mt = 0; mt < GE::kVBlocks; ++mt) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int32_t vkey = min(t0 + 16 * (mt + vshift) + 4 * a.quad + i, last);
            const int64_t vpage = a.table[vkey >> a.log2_page];
            const char* vp = a.vbase + vpage * a.page_bytes + (int64_t)(vkey & a.pmask) * a.token_bytes +
                             (a.r16 & GE::kPieceMask) * 16;
            if (FUSED && vkey == a.new_pos) vp = a.vnew + (a.r16 & GE::kPieceMask) * 16;
#pragma unroll
            for (int c = 0; c < GE::kPasses; ++c) t.v[c][4 * mt + i] = load16(vp + 256 * c);
        }
    }
}

template <typename GE>
struct State {
    f32x4 o[GE::kPasses][8];   // O^T accumulator: o[c][j][r] = column 128*c + 32*quad + 8*r + j of head lane%16
    float m;       // running max of the log2-domain scores of head lane%16
    float l;       // this lane's share of the running sum
};

// What the hooks need per row (this lane's column).  Unused members cost nothing without their hook.
struct RowMods {
    int32_t lo;         // window: first visible key of this row
    int32_t lo_until;   // window: tiles that start before this key need the lower mask (wave-uniform)
    int32_t pos;        // score: the row's absolute position
    float slope2;       // score: bias slope * log2(e)
    float cap_in;       // score: scale / softcap, 0 without a cap
    float cap_out;      // score: softcap * log2(e)
    float scale;        // score: plain scale (the unmodified path folds log2(e) into it)
    int32_t doc;        // document mask: the row's own document id
    pa_mod_ctx uc;      // user modification: what its hooks are told about the row
};

// lim = first key this lane's row may not see (the segment end, or less under a per-row causal bound);
// mask_from <= every lane's lim, wave-uniform: tiles that end at or before it need no mask.
template <bool RAGGED, typename E, typename M, typename GE>
__device__ __forceinline__ void compute_tile(State<GE>& st, const Tile<GE>& t, const uint4 (&qf)[GE::kKS], float sc,
                                             int32_t t0, int32_t lim, int32_t mask_from, int32_t quad,
                                             const RowMods& rm)
{
    constexpr int kTileKeys = GE::kTileKeys;
    constexpr int kBlocks = GE::kBlocks;
    f32x4 s[kBlocks < 2 ? 2 : kBlocks];
    s[1] = f32x4{0.f, 0.f, 0.f, 0.f};                  // a block the tile does not have: zero weights
#pragma unroll
    for (int mt = 0; mt < kBlocks; ++mt) {
        s[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < GE::kKS; ++ks)
            s[mt] = E::mfma16(t.k[mt][ks], qf[ks], s[mt]);
    }
    // s[mt][i] is the score of key t0 + 16*mt + 4*quad + i for head lane%16
    const bool partial = t0 + kTileKeys > mask_from;    // wave-uniform
    const bool below = M::kWindow && t0 < rm.lo_until;  // wave-uniform: the tile holds keys before some window
    float tmax = -INFINITY;
#pragma unroll
    for (int mt = 0; mt < kBlocks; ++mt)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int32_t key = t0 + 16 * mt + 4 * quad + i;
            float x;
            if (M::kScore) {
                // soft cap: c * tanh(y / c) with tanh(z) = 1 - 2 / (1 + e^(2z)); then the linear position bias;
                // everything lands in the log2 domain
                if (rm.cap_in > 0.f) {
                    const float e2z = __builtin_amdgcn_exp2f(s[mt][i] * rm.cap_in * (2.f * kLog2e));
                    x = rm.cap_out * (1.f - 2.f * __builtin_amdgcn_rcpf(1.f + e2z));
                } else {
                    x = s[mt][i] * sc;
                }
                x = __builtin_fmaf(rm.slope2, (float)(key - rm.pos), x);
            } else {
                x = s[mt][i] * sc;
            }
            if (M::kUser) x = user_score<M>(rm.uc, key, x * kLn2) * kLog2e;   // hooks work in natural units
            if (partial && key >= lim) x = -INFINITY;   // mask by selection
            if (below && key < rm.lo) x = -INFINITY;
            if (M::kDoc && t.doc[mt][i] != rm.doc) x = -INFINITY;
            s[mt][i] = x;
            tmax = fmaxf(tmax, x);
        }
    tmax = fmaxf(tmax, __shfl_xor(tmax, 16, 64));
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
    // decode: finite, every tile holds at least one valid key; a row under a causal bound or a document mask may
    // have seen none yet
    const float m_new = fmaxf(st.m, tmax);
    const float m_use = ((RAGGED || M::kDoc) && m_new == -INFINITY) ? 0.f : m_new;
    const float alpha = __builtin_amdgcn_exp2f(st.m - m_use);
    float psum = 0.f;
#pragma unroll
    for (int mt = 0; mt < kBlocks; ++mt)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float p = __builtin_amdgcn_exp2f(s[mt][i] - m_use);
            s[mt][i] = p;
            psum += p;
        }
    st.m = m_new;
    st.l = st.l * alpha + psum;
    if (__any(alpha != 1.f)) {
#pragma unroll
        for (int c = 0; c < GE::kPasses; ++c)
#pragma unroll
            for (int j = 0; j < 8; ++j) st.o[c][j] *= alpha;
    }
    // Probabilities as the B operand: contraction slot 8*quad + e <-> key (e<4 ? 4*quad+e : 16+4*quad+e-4) of a pair
    // of blocks.  They are carried as TWO bf16 terms (p = hi + lo, lo = bf16(p - hi)): the matrix cores idle most of
    // the time in this HBM-bound kernel, so the second product is free and removes the 2^-9 weight rounding that
    // would otherwise dominate the error of short contexts.
    constexpr int kPairs = kBlocks < 2 ? 1 : kBlocks / 2;   // pairs of blocks: 2 at head_dim 64, else 1
    uint4 pb[kPairs], pl[kPairs];
#pragma unroll
    for (int pr = 0; pr < kPairs; ++pr) {
        const f32x4& s0 = s[2 * pr];
        const f32x4& s1 = s[2 * pr + 1];
        pb[pr].x = E::pack(s0[0], s0[1]);
        pb[pr].y = E::pack(s0[2], s0[3]);
        pb[pr].z = E::pack(s1[0], s1[1]);
        pb[pr].w = E::pack(s1[2], s1[3]);
        pl[pr].x = E::pack(s0[0] - E::lo_of(pb[pr].x), s0[1] - E::hi_of(pb[pr].x));
        pl[pr].y = E::pack(s0[2] - E::lo_of(pb[pr].y), s0[3] - E::hi_of(pb[pr].y));
        pl[pr].z = E::pack(s1[0] - E::lo_of(pb[pr].z), s1[1] - E::hi_of(pb[pr].z));
        pl[pr].w = E::pack(s1[2] - E::lo_of(pb[pr].w), s1[3] - E::hi_of(pb[pr].w));
    }
    // in-register 8x8 transpose of V, one head_dim column (j) at a time, feeding the A operand
#pragma unroll
    for (int c = 0; c < GE::kPasses; ++c)
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t sel = (j & 1) ? 0x07060302u : 0x05040100u;
            uint4 a;   // columns j of rows (0,1), (2,3), (4,5), (6,7): word j/2 of each row, low or high half
            a.x = __builtin_amdgcn_perm(word(t.v[c][1], j / 2), word(t.v[c][0], j / 2), sel);
            a.y = __builtin_amdgcn_perm(word(t.v[c][3], j / 2), word(t.v[c][2], j / 2), sel);
            if constexpr (GE::kVBlocks == 2) {
                a.z = __builtin_amdgcn_perm(word(t.v[c][5], j / 2), word(t.v[c][4], j / 2), sel);
                a.w = __builtin_amdgcn_perm(word(t.v[c][7], j / 2), word(t.v[c][6], j / 2), sel);
            } else {
                a.z = 0u;   // the absent block: zero values under zero weights
                a.w = 0u;
            }
            st.o[c][j] = E::mfma16(a, pb[0], st.o[c][j]);
            st.o[c][j] = E::mfma16(a, pl[0], st.o[c][j]);
            if constexpr (kPairs == 2) {
                // head_dim 64: lanes 8-15 of every 16 hold the V rows of blocks 2, 3; rotate the halves (DPP
                // row_ror:8) so that rows 0-7 of the operand carry them, and multiply by those blocks' weights
                uint4 b;
                b.x = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)a.x, 0x128, 0xF, 0xF, false);
                b.y = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)a.y, 0x128, 0xF, 0xF, false);
                b.z = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)a.z, 0x128, 0xF, 0xF, false);
                b.w = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)a.w, 0x128, 0xF, 0xF, false);
                st.o[c][j] = E::mfma16(b, pb[1], st.o[c][j]);
                st.o[c][j] = E::mfma16(b, pl[1], st.o[c][j]);
            }
        }
}

// ---------------------------------------------------------------------------------------------------
// Work distribution.  The context of the whole batch is one stream of 32-key tiles (sequence after sequence,
// ceil(len/32) tiles each); workgroup w of the nwg launched owns the contiguous tile range
// [w*T/nwg, (w+1)*T/nwg).  Every workgroup therefore streams the same number of bytes whatever the length
// mix is, and a sequence is cut only where a workgroup boundary falls inside it.  Each (workgroup, sequence)
// intersection is one softmax partial; partial id = w + s is unique because w and s only grow along the
// stream.  The workgroup that holds a sequence's first / last tile records itself in seg_first / seg_last for
// the merge kernel; a sequence that lies inside one workgroup is written to `out` directly (seg_first = -1).
// ---------------------------------------------------------------------------------------------------
template <int TK>
__device__ __forceinline__ int32_t tiles_of(int32_t len) { return (len + TK - 1) / TK; }

// Tiles of sequence i in the stream.  RAGGED (called from the prefill entry point): only sequences whose
// q_len * G rows fit the 16 columns of the matrix instruction take part; the others hold no tiles here and are
// left to the prefill kernel.
// A sliding window (window > 0) removes the tiles that lie wholly before the earliest window of the sequence's
// queries from the stream: the work of a sequence is ceil((len - first_key) / 32) tiles, first_key a multiple of 32.
template <int TK>
__device__ __forceinline__ int32_t first_key_of(int32_t len, int32_t q_len, int32_t window)
{
    if (window <= 0) return 0;
    return max(len - q_len - window + 1, 0) & ~(TK - 1);
}

template <bool RAGGED, int TK>
__device__ __forceinline__ int32_t seq_tiles(const int32_t* __restrict__ seq_lens, const int32_t* __restrict__ cu_q_lens,
                                             int32_t G, int32_t i, int32_t window)
{
    int32_t q_len = 1;
    if (RAGGED) {
        q_len = cu_q_lens[i + 1] - cu_q_lens[i];
        if (q_len < 1 || q_len * G > 16) return 0;
    }
    const int32_t len = seq_lens[i];
    return tiles_of<TK>(len - first_key_of<TK>(len, q_len, window));
}

// Sum of tiles over the batch; every lane returns the same value.
template <bool RAGGED, int TK>
__device__ __forceinline__ int32_t total_tiles(const int32_t* __restrict__ seq_lens, const int32_t* __restrict__ cu_q_lens,
                                               int32_t G, int32_t batch, int lane, int32_t window)
{
    int32_t n = 0;
    for (int32_t i = lane; i < batch; i += 64) n += seq_tiles<RAGGED, TK>(seq_lens, cu_q_lens, G, i, window);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) n += __shfl_xor(n, o, 64);
    return n;
}

// Sequence that holds global tile g (0 <= g < total) and the number of tiles before that sequence.
template <bool RAGGED, int TK>
__device__ __forceinline__ void locate_tile(const int32_t* __restrict__ seq_lens, const int32_t* __restrict__ cu_q_lens,
                                            int32_t G, int32_t batch, int32_t g, int lane, int32_t window,
                                            int32_t& seq, int32_t& tiles_before)
{
    int32_t base = 0;
    seq = batch;
    tiles_before = 0;
    for (int32_t blk = 0; blk < batch; blk += 64) {
        const int32_t idx = blk + lane;
        const int32_t n = idx < batch ? seq_tiles<RAGGED, TK>(seq_lens, cu_q_lens, G, idx, window) : 0;
        int32_t inc = n;                                   // inclusive scan over the 64 lanes
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int32_t t = __shfl_up(inc, o, 64);
            if (lane >= o) inc += t;
        }
        const int32_t blk_total = __shfl(inc, 63, 64);
        if (g < base + blk_total) {
            const uint64_t hit = __ballot(base + inc > g);
            const int first = __ffsll((unsigned long long)hit) - 1;
            seq = blk + first;
            tiles_before = base + __shfl(inc, first, 64) - __shfl(n, first, 64);
            return;
        }
        base += blk_total;
    }
}

// RAGGED: launched from the prefill entry point for the sequences with few queries (q_len * G <= 16): the 16
// columns are (query, head) pairs, column = query * G + head, each with its own causal bound; q / out / lse rows
// come from cu_q_lens; partials are 16 rows per KV head.
// E: element traits (bf16 / fp16).  M: compile-time policy of the mask / score hooks.
// FUSED (plain decode only): the step's append is folded in as in the one-launch kernel below -- the wave whose
// segment holds a sequence's last tile stores the new token's rows of its KV head and reads them from k_new / v_new.
template <int NW, bool UNIFORM, bool RAGGED, typename E, typename M, typename GE, bool FUSED = false>
__global__ __launch_bounds__(NW * 64) void paged_decode_mfma_kernel(
    CacheView cache, const uint16_t* __restrict__ q, uint16_t* __restrict__ out, float* __restrict__ lse,
    const int32_t* __restrict__ block_table, const int32_t* __restrict__ seq_lens, int32_t batch,
    int32_t num_q_heads, int32_t max_blocks, float scale, float* __restrict__ part_o, float* __restrict__ part_lse,
    int32_t* __restrict__ seg_first, int32_t* __restrict__ seg_last, const int32_t* __restrict__ cu_q_lens,
    int32_t causal, ModArgs mods, const uint16_t* __restrict__ k_new, const uint16_t* __restrict__ v_new)
{
    constexpr int kD = GE::kD;
    constexpr int kTileKeys = GE::kTileKeys;
    const int32_t window = M::kWindow ? mods.window : 0;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));   // wave-uniform: a scalar
    const int32_t w = blockIdx.x;
    const int32_t kvh = blockIdx.y * NW + wave;
    const int32_t G = num_q_heads / cache.num_kv_heads;
    const int32_t r16 = lane & 15, quad = lane >> 4;
    const float sc = scale * kLog2e;

    // Only min(nwg, total) workgroups take part, so that every participating one holds at least one tile
    // and the partials of a sequence belong to consecutive workgroups with none missing.
    int32_t total, g, g_end, s, before;
    if (batch <= 64) {
        // one read of the lengths serves both the total and the search for this workgroup's first sequence
        const int32_t n = lane < batch ? seq_tiles<RAGGED, kTileKeys>(seq_lens, cu_q_lens, G, lane, window) : 0;
        int32_t inc = n;                                   // inclusive scan over the 64 lanes
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int32_t t = __shfl_up(inc, o, 64);
            if (lane >= o) inc += t;
        }
        total = __shfl(inc, 63, 64);
        const int32_t nwg = min((int32_t)gridDim.x, total);
        if (w >= nwg) return;
        g = (int32_t)(((int64_t)w * total) / nwg);
        g_end = (int32_t)(((int64_t)(w + 1) * total) / nwg);
        const uint64_t hit = __ballot(inc > g);
        s = __ffsll((unsigned long long)hit) - 1;
        before = __shfl(inc, s, 64) - __shfl(n, s, 64);
    } else {
        total = total_tiles<RAGGED, kTileKeys>(seq_lens, cu_q_lens, G, batch, lane, window);
        const int32_t nwg = min((int32_t)gridDim.x, total);
        if (w >= nwg) return;
        g = (int32_t)(((int64_t)w * total) / nwg);
        g_end = (int32_t)(((int64_t)(w + 1) * total) / nwg);
        locate_tile<RAGGED, kTileKeys>(seq_lens, cu_q_lens, G, batch, g, lane, window, s, before);
    }
    s = __builtin_amdgcn_readfirstlane(s);
    before = __builtin_amdgcn_readfirstlane(before);

    Addr a;
    a.doc = nullptr;
    a.knew = nullptr;
    a.vnew = nullptr;
    a.new_pos = -1;
    a.ids = 0;
    a.ids_base = 0;
    a.kbase = reinterpret_cast<const char*>(cache.k) + (int64_t)kvh * cache.head_stride * 2;
    a.vbase = reinterpret_cast<const char*>(cache.v) + (int64_t)kvh * cache.head_stride * 2;
    a.page_bytes = cache.page_stride * 2;
    a.token_bytes = cache.token_stride * 2;
    a.log2_page = cache.log2_page;
    a.pmask = cache.page_size - 1;
    a.r16 = r16;
    a.quad = quad;
    a.koff = (uint32_t)(r16 * a.token_bytes + quad * 16);
#pragma unroll
    for (int i = 0; i < 4; ++i) a.voff[i] = (uint32_t)((4 * quad + i) * a.token_bytes + (r16 & GE::kPieceMask) * 16);

    while (g < g_end) {
        // segment: tiles [t_begin, t_end) of sequence s
        const int32_t len = seq_lens[s];
        const int32_t nt = seq_tiles<RAGGED, kTileKeys>(seq_lens, cu_q_lens, G, s, window);
        if (nt == 0) { ++s; continue; }                    // sequences without tiles in this stream
        const int32_t t_begin = g - before;
        const int32_t t_end = min(nt, g_end - before);
        // this lane's column: query qi of the sequence's q_len, head h (valid if r16 < rows)
        // (group sizes above 16: blockIdx.z picks 16 of the group's heads; these workgroups stream the same K/V)
        const int32_t h0 = RAGGED ? 0 : 16 * (int32_t)blockIdx.z;
        int32_t rows = min(G - h0, 16), qi = 0, q_row = s, q_len = 1;
        if (RAGGED) {
            const int32_t q_begin = cu_q_lens[s];
            q_len = cu_q_lens[s + 1] - q_begin;
            rows = q_len * G;
            qi = min(r16, rows - 1) / G;
            q_row = q_begin + qi;
        }
        const int32_t key0 = first_key_of<kTileKeys>(len, q_len, window);   // the stream's first key of this sequence
        const int32_t c0 = key0 + t_begin * kTileKeys;
        const int32_t c1 = min(len, key0 + t_end * kTileKeys);
        const int32_t pos = len - q_len + qi;              // this row's position
        int32_t lim = c1;
        if (RAGGED && causal) lim = min(c1, pos + 1);      // keys 0 .. pos
        RowMods rm;
        rm.lo = 0;
        rm.lo_until = 0;
        rm.pos = pos;
        rm.slope2 = 0.f;
        rm.cap_in = 0.f;
        rm.cap_out = 0.f;
        rm.scale = scale;
        rm.doc = 0;
        if (M::kDoc && mods.doc_ids) {
            a.doc = mods.doc_ids + (int64_t)s * mods.doc_stride;
            rm.doc = a.doc[max(pos, 0)];
        }
        if (M::kWindow && window > 0) {
            rm.lo = pos - window + 1;                      // |j - pos| < window, lower side
            rm.lo_until = len - window;                    // the last row's lower bound is the largest
            if (RAGGED && !causal) lim = min(lim, pos + window);
        }
        if (M::kScore) {
            if (mods.alibi_slopes && r16 < rows)
                rm.slope2 = mods.alibi_slopes[kvh * G + (RAGGED ? min(r16, rows - 1) - qi * G : h0 + r16)] * kLog2e;
            if (mods.softcap > 0.f) {
                rm.cap_in = scale / mods.softcap;
                rm.cap_out = mods.softcap * kLog2e;
            }
        }
        const int32_t mask_from = RAGGED ? c1 - 16 : c1;   // q_len <= 16: no bound lies further below the end
        const int32_t h = kvh * G + (RAGGED ? min(r16, rows - 1) - qi * G : h0 + min(r16, rows - 1));
        rm.uc = pa_mod_ctx{mods.user_data, s, h, pos, len};
        const int64_t o_idx = (int64_t)q_row * num_q_heads + h;
        a.table = block_table + (int64_t)s * max_blocks;
        if constexpr (FUSED) {
            a.new_pos = -1;
            if (t_end == nt) {                               // this segment ends the sequence: it holds the new token
                const int64_t new_row = ((int64_t)s * cache.num_kv_heads + kvh) * kD * 2;
                a.knew = reinterpret_cast<const char*>(k_new) + new_row;
                a.vnew = reinterpret_cast<const char*>(v_new) + new_row;
                a.new_pos = len - 1;
                constexpr int kPieces = kD / 8;
                if (blockIdx.z == 0 && lane < 2 * kPieces) {
                    const bool is_v = lane >= kPieces;
                    const int piece = lane - (is_v ? kPieces : 0);
                    const int64_t page = a.table[a.new_pos >> a.log2_page];
                    const int64_t slot = page * a.page_bytes + (int64_t)(a.new_pos & a.pmask) * a.token_bytes + piece * 16;
                    char* dst = const_cast<char*>(is_v ? a.vbase : a.kbase) + slot;
                    *reinterpret_cast<uint4*>(dst) = load16((is_v ? a.vnew : a.knew) + piece * 16);
                }
            }
        }

        // Q as the B operand of S^T = K Q^T: lane%16 = head, contraction slot 8*quad + e of step ks <-> element
        // 32*ks + 8*quad + e of head_dim -- the same element order the K loads use.
        uint4 qf[GE::kKS];
#pragma unroll
        for (int ks = 0; ks < GE::kKS; ++ks) {
            qf[ks] = uint4{0, 0, 0, 0};
            if (r16 < rows) qf[ks] = *reinterpret_cast<const uint4*>(q + o_idx * kD + 32 * ks + 8 * quad);
        }
        State<GE> st;
#pragma unroll
        for (int c = 0; c < GE::kPasses; ++c)
#pragma unroll
            for (int j = 0; j < 8; ++j) st.o[c][j] = f32x4{0.f, 0.f, 0.f, 0.f};
        st.m = -INFINITY;
        st.l = 0.f;

        // two tiles in registers: while one is computed the other's loads are in flight
        Tile<GE> ta, tb;
        load_tile<UNIFORM, M, GE, FUSED>(ta, a, c0, c1);
        for (int32_t t0 = c0; t0 < c1; t0 += 2 * kTileKeys) {
            const int32_t t1 = t0 + kTileKeys;
            // The waves of a workgroup (adjacent KV heads) meet before every tile load, so that together they request whole
            // token rows of the same pages at the same time: DRAM sees long contiguous runs instead of the 256-byte
            // head slices of waves that have drifted apart (measured: 76.2 % -> 78.6 % of HBM peak at head_dim 128).
            if (NW > 1) __builtin_amdgcn_s_barrier();
            if (t1 < c1) load_tile<UNIFORM, M, GE, FUSED>(tb, a, t1, c1);
            compute_tile<RAGGED, E, M, GE>(st, ta, qf, sc, t0, lim, mask_from, quad, rm);
            if (t1 >= c1) break;
            if (NW > 1) __builtin_amdgcn_s_barrier();
            if (t1 + kTileKeys < c1) load_tile<UNIFORM, M, GE, FUSED>(ta, a, t1 + kTileKeys, c1);
            compute_tile<RAGGED, E, M, GE>(st, tb, qf, sc, t1, lim, mask_from, quad, rm);
        }

        float l = st.l;
        l += __shfl_xor(l, 16, 64);
        l += __shfl_xor(l, 32, 64);
        const bool whole = t_begin == 0 && t_end == nt;    // the sequence's stream lies inside this workgroup
        // D = 64: accumulator rows 8-15 (lanes of quads 2 and 3) repeat rows 0-7 and are not stored
        if (r16 < rows && (kD != 64 || quad < 2)) {
            // l == 0: a row whose causal bound lies before this segment, or none of whose document's keys lie in it
            constexpr bool kMayBeEmpty = RAGGED || M::kDoc;
            const float inv = (!kMayBeEmpty || l > 0.f) ? 1.f / l : 0.f;
            const float lse_nat = (!kMayBeEmpty || l > 0.f) ? (st.m + __builtin_amdgcn_logf(l)) * kLn2 : -INFINITY;
            if (whole) {
#pragma unroll
                for (int c = 0; c < GE::kPasses; ++c)
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        uint4 wv;
                        wv.x = E::pack(st.o[c][0][r] * inv, st.o[c][1][r] * inv);
                        wv.y = E::pack(st.o[c][2][r] * inv, st.o[c][3][r] * inv);
                        wv.z = E::pack(st.o[c][4][r] * inv, st.o[c][5][r] * inv);
                        wv.w = E::pack(st.o[c][6][r] * inv, st.o[c][7][r] * inv);
                        *reinterpret_cast<uint4*>(out + o_idx * kD + 128 * c + 32 * quad + 8 * r) = wv;
                    }
                if (lse && quad == 0) lse[o_idx] = lse_nat;
            } else {
                const int64_t p_idx = RAGGED ? ((int64_t)(w + s) * cache.num_kv_heads + kvh) * 16 + r16
                                             : (int64_t)(w + s) * num_q_heads + h;
#pragma unroll
                for (int c = 0; c < GE::kPasses; ++c) {
                    float* po = part_o + p_idx * kD + 128 * c + 32 * quad;
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        *reinterpret_cast<float4*>(po + 8 * r) = float4{st.o[c][0][r] * inv, st.o[c][1][r] * inv,
                                                                        st.o[c][2][r] * inv, st.o[c][3][r] * inv};
                        *reinterpret_cast<float4*>(po + 8 * r + 4) = float4{st.o[c][4][r] * inv, st.o[c][5][r] * inv,
                                                                            st.o[c][6][r] * inv, st.o[c][7][r] * inv};
                    }
                }
                if (quad == 0) part_lse[p_idx] = lse_nat;
            }
        }
        if (wave == 0 && lane == 0 && blockIdx.y == 0 && blockIdx.z == 0) {
            if (t_begin == 0) seg_first[s] = whole ? -1 : w;
            if (t_end == nt) seg_last[s] = w;
        }
        g = before + t_end;
        before += nt;
        ++s;
    }
}

// ---------------------------------------------------------------------------------------------------
// Short contexts in one launch.  When a step holds little data its time is launches and dependent memory round
// trips, not bandwidth: the tile stream above needs a second launch to merge its partials.  Here one workgroup
// owns one (sequence, KV head[, slice of 16 heads]); its NW waves split the sequence's tiles into NW contiguous
// ranges, run the same tile loop, and merge their NW partials through LDS -- no workspace, no merge kernel.
// LDS: NW x 16 rows x (D + 4) floats of unnormalised accumulators (rows padded by 16 bytes so that the 16 rows of
// a quad land on distinct banks), NW x 16 maxima and NW x 16 sums: 66 KiB at head_dim 128 and 256.
// ---------------------------------------------------------------------------------------------------
// FUSED: the kernel also performs the step's append (Algorithm 1, Assign) of one new token per sequence at position
// len - 1: the wave that owns the sequence's last tile (always the last wave of the last workgroup) stores the
// token's K / V rows of this KV head into their slot, and reads those rows from k_new / v_new instead of the pool, so
// nothing waits for the store.  (Workgroups of other head slices of the same KV head read the new rows the same way
// and store nothing.)
// nsplit > 1 (contexts of a few thousand tokens with few sequences, where one workgroup per (sequence, KV head)
// would stream its context through a single compute unit): nsplit workgroups share a (sequence, KV head, slice), each
// takes a contiguous share of the tiles, leaves its merged partial (unnormalised accumulator rows, maxima, sums) in
// `part` and counts itself in on the unit's arrival counter; the workgroup that arrives last merges the nsplit
// partials in split order -- the result does not depend on who that is -- and sets the counter back to zero, so the
// counters are zero again when the kernel ends: still one launch, no merge kernel, nothing to clear beforehand.
// part: nsplit blocks of 16 * D + 32 floats per unit; arrive: one counter per unit, zero on entry.
template <int NW, bool UNIFORM, bool FUSED, typename E, typename M, typename GE>
__global__ __launch_bounds__(NW * 64) void paged_decode_short_kernel(
    CacheView cache, const uint16_t* __restrict__ q, uint16_t* __restrict__ out, float* __restrict__ lse,
    const int32_t* __restrict__ block_table, const int32_t* __restrict__ seq_lens, int32_t num_q_heads,
    int32_t max_blocks, float scale, ModArgs mods, const uint16_t* __restrict__ k_new,
    const uint16_t* __restrict__ v_new, int32_t nsplit, float* __restrict__ part, uint32_t* __restrict__ arrive)
{
    constexpr int kD = GE::kD;
    constexpr int kTileKeys = GE::kTileKeys;
    constexpr int kRow = kD + 4;
    __shared__ __attribute__((aligned(16))) float sm_o[NW * 16 * kRow];
    __shared__ float sm_m[NW * 16];
    __shared__ float sm_l[NW * 16];
    __shared__ uint32_t sm_last;

    const int32_t window = M::kWindow ? mods.window : 0;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));   // wave-uniform: a scalar
    const int32_t s = (int32_t)blockIdx.x / nsplit;
    const int32_t split = (int32_t)blockIdx.x - s * nsplit;
    const int32_t kvh = blockIdx.y;
    const int32_t G = num_q_heads / cache.num_kv_heads;
    const int32_t h0 = 16 * (int32_t)blockIdx.z;
    const int32_t rows = min(G - h0, 16);
    const int32_t r16 = lane & 15, quad = lane >> 4;
    const float sc = scale * kLog2e;

    const int32_t len = seq_lens[s];
    const int32_t key0 = first_key_of<kTileKeys>(len, 1, window);
    const int32_t nt = tiles_of<kTileKeys>(len - key0);
    const int32_t wt0 = (int32_t)(((int64_t)split * nt) / nsplit);               // this workgroup's share of the tiles
    const int32_t wtn = (int32_t)(((int64_t)(split + 1) * nt) / nsplit) - wt0;
    const int32_t t_begin = wt0 + (int32_t)(((int64_t)wave * wtn) / NW);
    const int32_t t_end = wt0 + (int32_t)(((int64_t)(wave + 1) * wtn) / NW);
    const int32_t c0 = key0 + t_begin * kTileKeys;
    const int32_t c1 = min(len, key0 + t_end * kTileKeys);
    const int32_t pos = len - 1;

    State<GE> st;
#pragma unroll
    for (int c = 0; c < GE::kPasses; ++c)
#pragma unroll
        for (int j = 0; j < 8; ++j) st.o[c][j] = f32x4{0.f, 0.f, 0.f, 0.f};
    st.m = -INFINITY;
    st.l = 0.f;

    if (t_begin < t_end) {                                   // wave-uniform: this wave holds tiles
        Addr a;
        a.doc = nullptr;
        a.kbase = reinterpret_cast<const char*>(cache.k) + (int64_t)kvh * cache.head_stride * 2;
        a.vbase = reinterpret_cast<const char*>(cache.v) + (int64_t)kvh * cache.head_stride * 2;
        a.page_bytes = cache.page_stride * 2;
        a.token_bytes = cache.token_stride * 2;
        a.log2_page = cache.log2_page;
        a.pmask = cache.page_size - 1;
        a.r16 = r16;
        a.quad = quad;
        a.koff = (uint32_t)(r16 * a.token_bytes + quad * 16);
#pragma unroll
        for (int i = 0; i < 4; ++i)
            a.voff[i] = (uint32_t)((4 * quad + i) * a.token_bytes + (r16 & GE::kPieceMask) * 16);
        a.table = block_table + (int64_t)s * max_blocks;
        // the block-table entries of this wave's key range, one per lane (ranges of more than 64 pages fall back
        // to loads for the part beyond)
        a.ids_base = c0 >> a.log2_page;
        a.ids = a.table[min(a.ids_base + lane, (c1 - 1) >> a.log2_page)];
        a.knew = nullptr;
        a.vnew = nullptr;
        a.new_pos = -1;
        if constexpr (FUSED) {
            const int64_t new_row = ((int64_t)s * cache.num_kv_heads + kvh) * kD * 2;
            a.knew = reinterpret_cast<const char*>(k_new) + new_row;
            a.vnew = reinterpret_cast<const char*>(v_new) + new_row;
            a.new_pos = pos;
            if (wave == NW - 1 && split == nsplit - 1 && blockIdx.z == 0) {
                constexpr int kPieces = kD / 8;              // 16-byte pieces of a row; K then V: at most 64 lanes
                if (lane < 2 * kPieces) {
                    const bool is_v = lane >= kPieces;
                    const int piece = lane - (is_v ? kPieces : 0);
                    const int64_t page = a.table[pos >> a.log2_page];
                    const int64_t slot = page * a.page_bytes + (int64_t)(pos & a.pmask) * a.token_bytes + piece * 16;
                    char* dst = const_cast<char*>(is_v ? a.vbase : a.kbase) + slot;
                    *reinterpret_cast<uint4*>(dst) = load16((is_v ? a.vnew : a.knew) + piece * 16);
                }
            }
        }

        RowMods rm;
        rm.lo = 0;
        rm.lo_until = 0;
        rm.pos = pos;
        rm.slope2 = 0.f;
        rm.cap_in = 0.f;
        rm.cap_out = 0.f;
        rm.scale = scale;
        rm.doc = 0;
        if (M::kDoc && mods.doc_ids) {
            a.doc = mods.doc_ids + (int64_t)s * mods.doc_stride;
            rm.doc = a.doc[pos];
        }
        rm.uc = pa_mod_ctx{mods.user_data, s, kvh * G + h0 + min(r16, rows - 1), pos, len};
        if (M::kWindow && window > 0) {
            rm.lo = pos - window + 1;
            rm.lo_until = len - window;
        }
        if (M::kScore) {
            if (mods.alibi_slopes && r16 < rows) rm.slope2 = mods.alibi_slopes[kvh * G + h0 + r16] * kLog2e;
            if (mods.softcap > 0.f) {
                rm.cap_in = scale / mods.softcap;
                rm.cap_out = mods.softcap * kLog2e;
            }
        }
        const int64_t q_idx = (int64_t)s * num_q_heads + kvh * G + h0 + min(r16, rows - 1);
        uint4 qf[GE::kKS];
#pragma unroll
        for (int ks = 0; ks < GE::kKS; ++ks) {
            qf[ks] = uint4{0, 0, 0, 0};
            if (r16 < rows) qf[ks] = *reinterpret_cast<const uint4*>(q + q_idx * kD + 32 * ks + 8 * quad);
        }
        Tile<GE> ta, tb;
        load_tile<UNIFORM, M, GE, FUSED, true>(ta, a, c0, c1);
        for (int32_t t0 = c0; t0 < c1; t0 += 2 * kTileKeys) {
            const int32_t t1 = t0 + kTileKeys;
            if (t1 < c1) load_tile<UNIFORM, M, GE, FUSED, true>(tb, a, t1, c1);
            compute_tile<false, E, M, GE>(st, ta, qf, sc, t0, c1, c1, quad, rm);
            if (t1 >= c1) break;
            if (t1 + kTileKeys < c1) load_tile<UNIFORM, M, GE, FUSED, true>(ta, a, t1 + kTileKeys, c1);
            compute_tile<false, E, M, GE>(st, tb, qf, sc, t1, c1, c1, quad, rm);
        }
    }

    // publish the wave's partial: unnormalised accumulator, running maximum (log2 domain), sum
    float l = st.l;
    l += __shfl_xor(l, 16, 64);
    l += __shfl_xor(l, 32, 64);
    if (kD != 64 || quad < 2) {                              // D = 64: quads 2 and 3 repeat quads 0 and 1
        float* po = sm_o + (wave * 16 + r16) * kRow + 32 * quad;
#pragma unroll
        for (int c = 0; c < GE::kPasses; ++c)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                *reinterpret_cast<float4*>(po + 128 * c + 8 * r) =
                    float4{st.o[c][0][r], st.o[c][1][r], st.o[c][2][r], st.o[c][3][r]};
                *reinterpret_cast<float4*>(po + 128 * c + 8 * r + 4) =
                    float4{st.o[c][4][r], st.o[c][5][r], st.o[c][6][r], st.o[c][7][r]};
            }
    }
    if (quad == 0) {
        sm_m[wave * 16 + r16] = st.m;
        sm_l[wave * 16 + r16] = l;
    }
    __syncthreads();                                         // every wave arrives exactly once, with or without tiles

    // merge: thread -> (row, 4 columns); weights 2^(m_p - M), a partial without any visible key weighs nothing
    const int64_t out_row0 = (int64_t)s * num_q_heads + kvh * G + h0;
    const int64_t unit = ((int64_t)s * gridDim.y + kvh) * gridDim.z + blockIdx.z;
    constexpr int kPartFloats = 16 * kD + 32;                // accumulator rows, then 16 maxima, then 16 sums
    float* const my_part = part + (unit * nsplit + split) * kPartFloats;
    for (int it = threadIdx.x; it < 16 * (kD / 4); it += NW * 64) {
        const int row = it / (kD / 4), c4 = it % (kD / 4);
        if (row >= rows) continue;
        float mx = -INFINITY;
#pragma unroll
        for (int p = 0; p < NW; ++p) mx = fmaxf(mx, sm_m[p * 16 + row]);
        float sum = 0.f;
        float4 acc = float4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int p = 0; p < NW; ++p) {
            const float mp = sm_m[p * 16 + row];
            const float wgt = mp == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(mp - mx);
            const float4 v = *reinterpret_cast<const float4*>(sm_o + (p * 16 + row) * kRow + 4 * c4);
            sum = __builtin_fmaf(wgt, sm_l[p * 16 + row], sum);
            acc.x = __builtin_fmaf(wgt, v.x, acc.x);
            acc.y = __builtin_fmaf(wgt, v.y, acc.y);
            acc.z = __builtin_fmaf(wgt, v.z, acc.z);
            acc.w = __builtin_fmaf(wgt, v.w, acc.w);
        }
        if (nsplit > 1) {                                    // this workgroup's partial, relative to its own maximum
            // component-major ([4][16 rows][D / 4]): consecutive lanes store consecutive words
            float* po = my_part + row * (kD / 4) + c4;
            __hip_atomic_store(po + 0 * 4 * kD, acc.x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(po + 1 * 4 * kD, acc.y, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(po + 2 * 4 * kD, acc.z, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(po + 3 * 4 * kD, acc.w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (c4 == 0) {
                __hip_atomic_store(my_part + 16 * kD + row, mx, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __hip_atomic_store(my_part + 16 * kD + 16 + row, sum, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            continue;
        }
        const float inv = sum > 0.f ? 1.f / sum : 0.f;       // sum == 0: an empty sequence (or no visible key)
        uint2 wv;
        wv.x = E::pack(acc.x * inv, acc.y * inv);
        wv.y = E::pack(acc.z * inv, acc.w * inv);
        *reinterpret_cast<uint2*>(out + (out_row0 + row) * kD + 4 * c4) = wv;
        if (lse && c4 == 0) lse[out_row0 + row] = sum > 0.f ? (mx + __builtin_amdgcn_logf(sum)) * kLn2 : -INFINITY;
    }
    if (nsplit == 1) return;

    // Arrival.  The partials are written and read with device-scope atomic accesses (write-through stores, loads
    // that bypass the caches that are not coherent across the chip), so publishing them needs no cache write-back
    // or invalidation -- a release fence per workgroup costs about as much here as the context split gains -- only
    // order: every wave waits until its stores have been acknowledged, the barrier collects the waves, then one thread
    // counts the workgroup in; the workgroup that finds nsplit - 1 earlier arrivals reads the partials after its
    // counting has returned.  It merges them in split order and hands the counter back as it found it.  (Every
    // workgroup of the unit gets here exactly once, with or without tiles.)
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    if (threadIdx.x == 0) {
        const uint32_t before = __hip_atomic_fetch_add(arrive + unit, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const uint32_t last = before == (uint32_t)(nsplit - 1) ? 1u : 0u;
        if (last) __hip_atomic_store(arrive + unit, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        sm_last = last;
    }
    __syncthreads();
    if (sm_last == 0u) return;
    const float* const unit_part = part + unit * nsplit * kPartFloats;
    for (int it = threadIdx.x; it < 16 * (kD / 4); it += NW * 64) {
        const int row = it / (kD / 4), c4 = it % (kD / 4);
        if (row >= rows) continue;
        float mx = -INFINITY;
        for (int p = 0; p < nsplit; ++p)
            mx = fmaxf(mx, __hip_atomic_load(unit_part + p * kPartFloats + 16 * kD + row, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
        float sum = 0.f;
        float4 acc = float4{0.f, 0.f, 0.f, 0.f};
        for (int p = 0; p < nsplit; ++p) {
            const float* pp = unit_part + p * kPartFloats;
            const float mp = __hip_atomic_load(pp + 16 * kD + row, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const float wgt = mp == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(mp - mx);
            float4 v;
            const float* pv = pp + row * (kD / 4) + c4;
            v.x = __hip_atomic_load(pv + 0 * 4 * kD, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            v.y = __hip_atomic_load(pv + 1 * 4 * kD, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            v.z = __hip_atomic_load(pv + 2 * 4 * kD, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            v.w = __hip_atomic_load(pv + 3 * 4 * kD, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            sum = __builtin_fmaf(wgt, __hip_atomic_load(pp + 16 * kD + 16 + row, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT), sum);
            acc.x = __builtin_fmaf(wgt, v.x, acc.x);
            acc.y = __builtin_fmaf(wgt, v.y, acc.y);
            acc.z = __builtin_fmaf(wgt, v.z, acc.z);
            acc.w = __builtin_fmaf(wgt, v.w, acc.w);
        }
        const float inv = sum > 0.f ? 1.f / sum : 0.f;
        uint2 wv;
        wv.x = E::pack(acc.x * inv, acc.y * inv);
        wv.y = E::pack(acc.z * inv, acc.w * inv);
        *reinterpret_cast<uint2*>(out + (out_row0 + row) * kD + 4 * c4) = wv;
        if (lse && c4 == 0) lse[out_row0 + row] = sum > 0.f ? (mx + __builtin_amdgcn_logf(sum)) * kLn2 : -INFINITY;
    }
}

template <int NW, typename E, typename M, typename GE>
void launch_short_nw(const AttnArgs& a, hipStream_t stream)
{
    const int32_t G = a.num_q_heads / a.cache.num_kv_heads;
    const int32_t nsplit = a.short_nsplit > 1 ? a.short_nsplit : 1;
    const dim3 grid((uint32_t)(a.batch * nsplit), (uint32_t)a.cache.num_kv_heads, (uint32_t)((G + 15) / 16));
    const bool uniform = a.cache.page_size >= 16;
    auto kern = a.k_new ? (uniform ? paged_decode_short_kernel<NW, true, true, E, M, GE>
                                   : paged_decode_short_kernel<NW, false, true, E, M, GE>)
                        : (uniform ? paged_decode_short_kernel<NW, true, false, E, M, GE>
                                   : paged_decode_short_kernel<NW, false, false, E, M, GE>);
    hipLaunchKernelGGL(kern, grid, dim3(NW * 64), 0, stream, a.cache, (const uint16_t*)a.q, (uint16_t*)a.out, a.lse,
                       a.block_table, a.seq_lens, a.num_q_heads, a.max_blocks, a.scale, a.mods,
                       (const uint16_t*)a.k_new, (const uint16_t*)a.v_new, nsplit, a.short_part, a.short_arrive);
}

template <int NW, typename E, typename M, typename GE>
void launch_nw(const AttnArgs& a, hipStream_t stream)
{
    const int32_t G = a.num_q_heads / a.cache.num_kv_heads;
    const dim3 grid((uint32_t)a.num_wgs, (uint32_t)(a.cache.num_kv_heads / NW), a.cu_q_lens ? 1u : (uint32_t)((G + 15) / 16));
    const bool uniform = a.cache.page_size >= 16;
    auto kern = a.cu_q_lens ? (uniform ? paged_decode_mfma_kernel<NW, true, true, E, M, GE>
                                       : paged_decode_mfma_kernel<NW, false, true, E, M, GE>)
                : a.k_new   ? (uniform ? paged_decode_mfma_kernel<NW, true, false, E, M, GE, true>
                                       : paged_decode_mfma_kernel<NW, false, false, E, M, GE, true>)
                            : (uniform ? paged_decode_mfma_kernel<NW, true, false, E, M, GE>
                                       : paged_decode_mfma_kernel<NW, false, false, E, M, GE>);
    hipLaunchKernelGGL(kern, grid, dim3(NW * 64), 0, stream, a.cache, (const uint16_t*)a.q, (uint16_t*)a.out, a.lse,
                       a.block_table, a.seq_lens, a.batch, a.num_q_heads, a.max_blocks, a.scale, a.part_o,
                       a.part_lse, a.seg_first, a.seg_last, a.cu_q_lens, a.causal, a.mods,
                       (const uint16_t*)(a.cu_q_lens ? nullptr : a.k_new), (const uint16_t*)(a.cu_q_lens ? nullptr : a.v_new));
}

template <typename E, typename M, typename GE>
void launch_em(const AttnArgs& a, hipStream_t stream)
{
    switch (decode_mfma_heads_per_wg(a.cache.num_kv_heads, GE::kD)) {
        case 8:
            if constexpr (GE::kD <= 128) launch_nw<8, E, M, GE>(a, stream);
            break;
        case 4: launch_nw<4, E, M, GE>(a, stream); break;
        case 2: launch_nw<2, E, M, GE>(a, stream); break;
        default: launch_nw<1, E, M, GE>(a, stream); break;
    }
}

}  // namespace

// Every kernel instantiation of one head_dim; defined in that head_dim's translation unit.
template <int D>
void launch_decode_short_dim(const AttnArgs& a, hipStream_t stream)
{
    typedef Mods<true, true, false> WindowScore;
    typedef Geo<D> GE;
    constexpr int NW = D > 128 ? 4 : 8;                 // head_dim 256: two tiles take about 250 registers
    const bool docs = a.has_mods && a.mods.doc_ids;
    if (a.mods.user_mod) {                              // a user modification: one instantiation per listed struct
#define PA_USER_CASE(U)                                                                        \
        if (a.mods.user_mod == U::kId) {                                                       \
            if (a.dtype == PA_DTYPE_BF16) launch_short_nw<NW, ElemBf16, Mods<true, true, true, U>, GE>(a, stream);  \
            else launch_short_nw<NW, ElemF16, Mods<true, true, true, U>, GE>(a, stream);       \
            return;                                                                            \
        }
        PA_USER_MODS(PA_USER_CASE)
#undef PA_USER_CASE
        return;
    }
    if (a.dtype == PA_DTYPE_BF16) {
        if (docs) launch_short_nw<NW, ElemBf16, AllMods, GE>(a, stream);
        else if (a.has_mods) launch_short_nw<NW, ElemBf16, WindowScore, GE>(a, stream);
        else launch_short_nw<NW, ElemBf16, NoMods, GE>(a, stream);
    } else {
        if (docs) launch_short_nw<NW, ElemF16, AllMods, GE>(a, stream);
        else if (a.has_mods) launch_short_nw<NW, ElemF16, WindowScore, GE>(a, stream);
        else launch_short_nw<NW, ElemF16, NoMods, GE>(a, stream);
    }
}

template <int D>
void launch_decode_mfma_dim(const AttnArgs& a, hipStream_t stream)
{
    typedef Mods<true, true, false> WindowScore;
    typedef Geo<D> GE;
    const bool docs = a.has_mods && a.mods.doc_ids;
    if (a.mods.user_mod) {
#define PA_USER_CASE(U)                                                                        \
        if (a.mods.user_mod == U::kId) {                                                       \
            if (a.dtype == PA_DTYPE_BF16) launch_em<ElemBf16, Mods<true, true, true, U>, GE>(a, stream);  \
            else launch_em<ElemF16, Mods<true, true, true, U>, GE>(a, stream);                 \
            return;                                                                            \
        }
        PA_USER_MODS(PA_USER_CASE)
#undef PA_USER_CASE
        return;
    }
    if (a.dtype == PA_DTYPE_BF16) {
        if (docs) launch_em<ElemBf16, AllMods, GE>(a, stream);
        else if (a.has_mods) launch_em<ElemBf16, WindowScore, GE>(a, stream);
        else launch_em<ElemBf16, NoMods, GE>(a, stream);
    } else {
        if (docs) launch_em<ElemF16, AllMods, GE>(a, stream);
        else if (a.has_mods) launch_em<ElemF16, WindowScore, GE>(a, stream);
        else launch_em<ElemF16, NoMods, GE>(a, stream);
    }
}

}  // namespace pa
