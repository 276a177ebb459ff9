/*
 * CPU oracle for attention over a paged KV cache -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, obviously-correct implementation of what the GPU library
 * computes, written from the paper's Algorithm 1 (Assign / Gather index
 * translation) and from the plain definition of softmax attention with the
 * length mask of Sec. III-B ("FlexAttention Kernel" paragraph).  It exists so
 * the tests, the smoke check and the benchmark's CPU-baseline leg have
 * something independent to compare the HIP kernels with.  It shares no code,
 * header, table or helper with the GPU path and must never be called from it.
 *
 * All pointers are HOST pointers.  Caches are addressed through element
 * strides, so both the literal token-major layout [NP, P, Hkv, d] of
 * Algorithm 1 (flat slot p = page * P + o) and a head-major one can be
 * described.  dtype: 0 = IEEE fp32, 1 = bfloat16 (upper 16 bits of an fp32),
 * 2 = IEEE binary16.
 *
 * Every function returns 0 on success and a negative code when an argument
 * or a device-side precondition (page id out of range, position beyond the
 * table) is violated; nothing is written in that case beyond what was
 * already processed.
 */
#ifndef PAGED_ORACLE_H
#define PAGED_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1, ORACLE_F16 = 2 };

enum {
    ORACLE_OK = 0,
    ORACLE_BAD_ARG = -1,      /* NULL pointer, non power-of-two page, ...      */
    ORACLE_BAD_PAGE = -2,     /* block-table entry outside [0, num_pages)      */
    ORACLE_BAD_POSITION = -3, /* position / length beyond max_blocks * P       */
    ORACLE_NO_MEMORY = -4
};

typedef struct {
    void *k_cache;        /* physical K pool                                   */
    void *v_cache;        /* physical V pool (a separate buffer, Sec. III-B)   */
    int64_t page_stride;  /* elements between consecutive physical pages       */
    int64_t token_stride; /* elements between consecutive slots of a page      */
    int64_t head_stride;  /* elements between consecutive KV heads of a slot   */
    int32_t num_pages;    /* NP                                                */
    int32_t page_size;    /* P, a power of two (Algorithm 1, Require)          */
    int32_t num_kv_heads; /* Hkv                                               */
    int32_t head_dim;     /* d, innermost and contiguous                       */
    int32_t dtype;        /* ORACLE_F32, ORACLE_BF16 or ORACLE_F16             */
} oracle_cache;

/* Algorithm 1, Assign.  For i = 0..T-1 in order: t = positions[i],
 * s = seq_ids[i], b = floor(t / P), o = t mod P,
 * p = block_table[s][b] * P + o, K[p] <- k_new[i], V[p] <- v_new[i].
 * k_new / v_new are [T, Hkv, d] contiguous in the cache dtype; the copy is
 * bytewise.  Later tokens overwrite earlier ones that map to the same slot. */
int oracle_kv_append(const oracle_cache *c, const void *k_new, const void *v_new,
                     const int32_t *seq_ids, const int32_t *positions, int32_t T,
                     const int32_t *block_table, int32_t batch, int32_t max_blocks);

/* Algorithm 1, Gather.  For each sequence s and t = 0..seq_lens[s]-1 the same
 * translation; the slot's Hkv*d elements are copied bytewise to
 * out_k / out_v row (cu_seq_lens[s] + t) of a packed [sum(len), Hkv, d] array. */
int oracle_kv_gather(const oracle_cache *c, void *out_k, void *out_v,
                     const int32_t *block_table, const int32_t *seq_lens,
                     const int32_t *cu_seq_lens, int32_t batch, int32_t max_blocks);

/* Attention by the direct definition, in fp64.
 *
 * q is [total_q, Hq, d] in the cache dtype, packed per sequence at
 * cu_q_lens[s] .. cu_q_lens[s+1] (decode: cu_q_lens = 0,1,..,batch).
 * Query i of sequence s (Tq = its query count, len = seq_lens[s]) sits at
 * absolute position pos = len - Tq + i.  Allowed keys:
 *     J = { j : 0 <= j < len  and  (causal == 0 or j <= pos) }
 * (the length mask of Sec. III-B read 0-based, as Gather's loop bounds fix it).
 * With kvh = floor(h / G), G = Hq / Hkv:
 *     x_j = scale * <q[i,h,:], K_s[j,kvh,:]>,  m = max_J x_j,
 *     w_j = exp(x_j - m),  Z = sum_J w_j,
 *     out[i,h,:] = sum_J (w_j / Z) V_s[j,kvh,:],   lse[i,h] = m + ln Z.
 * K_s, V_s are the sequence's keys/values produced by Gather and widened
 * exactly to fp64.  Empty J: out = 0, lse = -inf.
 *
 * out: double[total_q, Hq, d].  lse: double[total_q, Hq] or NULL.
 * weights: NULL, or double[total_q, Hq, weights_stride]; receives w_j / Z at
 * index j for j in J and 0 for every other j < weights_stride. */
int oracle_attention(const oracle_cache *c, const void *q, double *out, double *lse,
                     double *weights, int64_t weights_stride,
                     const int32_t *cu_q_lens, const int32_t *block_table,
                     const int32_t *seq_lens, int32_t batch, int32_t num_q_heads,
                     int32_t max_blocks, double scale, int32_t causal);

/* The same with user-defined mask and score modifications in the sense of
 * FlexAttention's mask_mod / score_mod (Sec. II-C, Sec. III-B), for the three
 * families this library builds in.  With pos the query's absolute position:
 *   mask:   key j is also required to satisfy
 *             |j - pos| < window                       if window > 0  (sliding window)
 *             doc_ids[s][j] == doc_ids[s][pos]         if doc_ids     (document mask;
 *                                   doc_ids is int32 [batch, doc_stride], logical positions)
 *   score:  x_j = scale * <q, k_j>
 *           x_j <- softcap * tanh(x_j / softcap)       if softcap > 0
 *           x_j <- x_j + alibi_slopes[h] * (j - pos)   if alibi_slopes (double[Hq])
 * and one user-defined pair (mask_mod / score_mod as a caller may write them, Sec. II-C), the prefix-LM family:
 *   mask:   j <= pos  or  j < prefix_lens[s]           if prefix_lens (int32[batch]): the first prefix_lens[s]
 *                                   tokens see each other in both directions, the rest is causal
 *   score:  x_j <- x_j + prefix_bias                   for the keys j < prefix_lens[s] (after the two above)
 * then softmax over the visible keys as above.  mods == NULL: no modification. */
typedef struct {
    int32_t window;
    double softcap;
    const double *alibi_slopes;
    const int32_t *doc_ids;
    int64_t doc_stride;
    const int32_t *prefix_lens;
    double prefix_bias;
} oracle_mods;

int oracle_attention_mod(const oracle_cache *c, const void *q, double *out, double *lse,
                         double *weights, int64_t weights_stride,
                         const int32_t *cu_q_lens, const int32_t *block_table,
                         const int32_t *seq_lens, int32_t batch, int32_t num_q_heads,
                         int32_t max_blocks, double scale, int32_t causal, const oracle_mods *mods);

/* Exact merge of softmax partials over disjoint key sets (the split-KV
 * identity): given n partials (o_c normalised, lse_c) returns the result over
 * the union:  M = max lse_c,  o = sum e^{lse_c - M} o_c / sum e^{lse_c - M},
 * lse = M + ln sum e^{lse_c - M}.  o_parts: double[n, d]; lse_parts: double[n].
 * Partials with lse = -inf (empty sets) contribute nothing. */
int oracle_merge_partials(const double *o_parts, const double *lse_parts, int32_t n,
                          int32_t d, double *out, double *lse);

/* The exact widening the attention applies to its inputs: n elements of `dtype` -> fp64. */
int oracle_widen(const void *src, int64_t n, int32_t dtype, double *dst);

/* Number of OpenMP threads the attention loop will use. */
int oracle_num_threads(void);

#ifdef __cplusplus
}
#endif
#endif /* PAGED_ORACLE_H */
