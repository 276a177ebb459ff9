/*
 * CPU oracle for attention over a paged KV cache -- TEST INFRASTRUCTURE ONLY.
 * See paged_oracle.h.  Plain C, fp64 arithmetic, no tiling, no online softmax,
 * no split: Algorithm 1's index translation written out, then the textbook
 * definition of masked softmax attention.  OpenMP only spreads independent
 * (query, head) pairs over cores.
 */
#include "paged_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static int elem_size(int dtype) { return dtype == ORACLE_F32 ? 4 : 2; }

static int cache_ok(const oracle_cache *c)
{
    if (!c || !c->k_cache || !c->v_cache) return 0;
    if (c->dtype != ORACLE_F32 && c->dtype != ORACLE_BF16 && c->dtype != ORACLE_F16) return 0;
    if (c->num_pages <= 0 || c->num_kv_heads <= 0 || c->head_dim <= 0) return 0;
    if (c->page_size <= 0 || (c->page_size & (c->page_size - 1)) != 0) return 0; /* Alg. 1: P is a power of two */
    return 1;
}

/* Algorithm 1 (Assign and Gather share it): logical token t of sequence s ->
 * element offset of its slot in the pool.  b = floor(t / P), o = t mod P,
 * slot = page_table[s][b] * P + o; in a strided pool the slot starts at
 * page * page_stride + o * token_stride.  Returns 0 or an error code. */
static int translate(const oracle_cache *c, const int32_t *block_table, int32_t max_blocks,
                     int32_t s, int64_t t, int64_t *elem_off)
{
    int64_t P = c->page_size;
    if (t < 0) return ORACLE_BAD_POSITION;
    int64_t b = t / P;
    int64_t o = t % P;
    if (b >= max_blocks) return ORACLE_BAD_POSITION;
    int64_t page = block_table[(int64_t)s * max_blocks + b];
    if (page < 0 || page >= c->num_pages) return ORACLE_BAD_PAGE;
    *elem_off = page * c->page_stride + o * c->token_stride;
    return ORACLE_OK;
}

int oracle_kv_append(const oracle_cache *c, const void *k_new, const void *v_new,
                     const int32_t *seq_ids, const int32_t *positions, int32_t T,
                     const int32_t *block_table, int32_t batch, int32_t max_blocks)
{
    if (!cache_ok(c) || T < 0 || batch < 0 || max_blocks < 0) return ORACLE_BAD_ARG;
    if (T == 0) return ORACLE_OK;
    if (!k_new || !v_new || !seq_ids || !positions || !block_table) return ORACLE_BAD_ARG;
    const int es = elem_size(c->dtype);
    const int64_t row = (int64_t)c->head_dim * es; /* bytes of one head of one token */
    for (int32_t i = 0; i < T; ++i) {
        int32_t s = seq_ids[i];
        if (s < 0 || s >= batch) return ORACLE_BAD_ARG;
        int64_t off;
        int rc = translate(c, block_table, max_blocks, s, positions[i], &off);
        if (rc) return rc;
        for (int32_t h = 0; h < c->num_kv_heads; ++h) {
            int64_t dst = (off + (int64_t)h * c->head_stride) * es;
            int64_t src = ((int64_t)i * c->num_kv_heads + h) * row;
            memcpy((char *)c->k_cache + dst, (const char *)k_new + src, (size_t)row);
            memcpy((char *)c->v_cache + dst, (const char *)v_new + src, (size_t)row);
        }
    }
    return ORACLE_OK;
}

/* Gather of one sequence into contiguous [len, Hkv, d] buffers (raw bytes). */
static int gather_one(const oracle_cache *c, const int32_t *block_table, int32_t max_blocks,
                      int32_t s, int32_t len, char *out_k, char *out_v)
{
    const int es = elem_size(c->dtype);
    const int64_t row = (int64_t)c->head_dim * es;
    for (int32_t t = 0; t < len; ++t) {
        int64_t off;
        int rc = translate(c, block_table, max_blocks, s, t, &off);
        if (rc) return rc;
        for (int32_t h = 0; h < c->num_kv_heads; ++h) {
            int64_t src = (off + (int64_t)h * c->head_stride) * es;
            int64_t dst = ((int64_t)t * c->num_kv_heads + h) * row;
            memcpy(out_k + dst, (const char *)c->k_cache + src, (size_t)row);
            memcpy(out_v + dst, (const char *)c->v_cache + src, (size_t)row);
        }
    }
    return ORACLE_OK;
}

int oracle_kv_gather(const oracle_cache *c, void *out_k, void *out_v,
                     const int32_t *block_table, const int32_t *seq_lens,
                     const int32_t *cu_seq_lens, int32_t batch, int32_t max_blocks)
{
    if (!cache_ok(c) || batch < 0 || max_blocks < 0) return ORACLE_BAD_ARG;
    if (batch == 0) return ORACLE_OK;
    if (!out_k || !out_v || !block_table || !seq_lens || !cu_seq_lens) return ORACLE_BAD_ARG;
    const int64_t tok = (int64_t)c->num_kv_heads * c->head_dim * elem_size(c->dtype);
    for (int32_t s = 0; s < batch; ++s) {
        if (seq_lens[s] < 0) return ORACLE_BAD_ARG;
        int rc = gather_one(c, block_table, max_blocks, s, seq_lens[s],
                            (char *)out_k + cu_seq_lens[s] * tok,
                            (char *)out_v + cu_seq_lens[s] * tok);
        if (rc) return rc;
    }
    return ORACLE_OK;
}

/* IEEE binary16 by its definition: sign, 5-bit exponent (bias 15), 10-bit fraction. */
static double half_value(uint16_t bits)
{
    const int sign = bits >> 15, e = (bits >> 10) & 31, f = bits & 1023;
    double v;
    if (e == 0) v = ldexp((double)f, -24);                   /* zero and subnormals: f * 2^-24 */
    else if (e == 31) v = f ? NAN : INFINITY;
    else v = ldexp(1.0 + (double)f / 1024.0, e - 15);
    return sign ? -v : v;
}

/* Exact widening: fp32 -> fp64 is exact; bf16 is the upper half of an fp32; binary16 by definition. */
static double widen(const void *base, int64_t idx, int dtype)
{
    if (dtype == ORACLE_F32) {
        float f;
        memcpy(&f, (const char *)base + idx * 4, 4);
        return (double)f;
    }
    uint16_t hbits;
    memcpy(&hbits, (const char *)base + idx * 2, 2);
    if (dtype == ORACLE_F16) return half_value(hbits);
    uint32_t bits = (uint32_t)hbits << 16;
    float f;
    memcpy(&f, &bits, 4);
    return (double)f;
}

int oracle_attention(const oracle_cache *c, const void *q, double *out, double *lse,
                     double *weights, int64_t weights_stride,
                     const int32_t *cu_q_lens, const int32_t *block_table,
                     const int32_t *seq_lens, int32_t batch, int32_t num_q_heads,
                     int32_t max_blocks, double scale, int32_t causal)
{
    return oracle_attention_mod(c, q, out, lse, weights, weights_stride, cu_q_lens, block_table, seq_lens, batch,
                                num_q_heads, max_blocks, scale, causal, NULL);
}

/* mask_mod: is key j visible to the query at position pos of sequence s? */
static int visible(const oracle_mods *mods, int32_t s, int64_t pos, int64_t j)
{
    if (!mods) return 1;
    if (mods->window > 0) {
        const int64_t dist = j > pos ? j - pos : pos - j;
        if (dist >= mods->window) return 0;
    }
    if (mods->doc_ids) {
        const int32_t *doc = mods->doc_ids + (int64_t)s * mods->doc_stride;
        if (doc[j] != doc[pos]) return 0;
    }
    if (mods->prefix_lens && !(j <= pos || j < mods->prefix_lens[s])) return 0;
    return 1;
}

/* score_mod: soft cap first, then the linear position bias. */
static double modded(const oracle_mods *mods, double x, int32_t s, int32_t h, int64_t pos, int64_t j)
{
    if (!mods) return x;
    if (mods->softcap > 0.0) x = mods->softcap * tanh(x / mods->softcap);
    if (mods->alibi_slopes) x += mods->alibi_slopes[h] * (double)(j - pos);
    if (mods->prefix_lens && j < mods->prefix_lens[s]) x += mods->prefix_bias;
    return x;
}

int oracle_attention_mod(const oracle_cache *c, const void *q, double *out, double *lse,
                         double *weights, int64_t weights_stride,
                         const int32_t *cu_q_lens, const int32_t *block_table,
                         const int32_t *seq_lens, int32_t batch, int32_t num_q_heads,
                         int32_t max_blocks, double scale, int32_t causal, const oracle_mods *mods)
{
    if (!cache_ok(c) || batch < 0 || max_blocks < 0) return ORACLE_BAD_ARG;
    if (mods && (mods->window < 0 || (mods->doc_ids && mods->doc_stride <= 0))) return ORACLE_BAD_ARG;
    if (batch == 0) return ORACLE_OK;
    if (!q || !out || !cu_q_lens || !block_table || !seq_lens) return ORACLE_BAD_ARG;
    const int32_t Hq = num_q_heads, Hkv = c->num_kv_heads, d = c->head_dim;
    if (Hq <= 0 || Hq % Hkv != 0) return ORACLE_BAD_ARG;
    const int32_t G = Hq / Hkv;
    const int es = elem_size(c->dtype);

    for (int32_t s = 0; s < batch; ++s) {
        const int32_t len = seq_lens[s];
        const int32_t q0 = cu_q_lens[s];
        const int32_t Tq = cu_q_lens[s + 1] - q0;
        if (len < 0 || Tq < 0) return ORACLE_BAD_ARG;
        if (Tq == 0) continue;

        /* Step 1: Gather (Algorithm 1) into contiguous K_s, V_s, then widen to fp64. */
        const int64_t n = (int64_t)len * Hkv * d;
        char *rk = (char *)malloc((size_t)(n * es) + 1);
        char *rv = (char *)malloc((size_t)(n * es) + 1);
        double *Ks = (double *)malloc((size_t)(n + 1) * sizeof(double));
        double *Vs = (double *)malloc((size_t)(n + 1) * sizeof(double));
        if (!rk || !rv || !Ks || !Vs) { free(rk); free(rv); free(Ks); free(Vs); return ORACLE_NO_MEMORY; }
        int rc = gather_one(c, block_table, max_blocks, s, len, rk, rv);
        if (rc) { free(rk); free(rv); free(Ks); free(Vs); return rc; }
        for (int64_t e = 0; e < n; ++e) { Ks[e] = widen(rk, e, c->dtype); Vs[e] = widen(rv, e, c->dtype); }
        free(rk); free(rv);

        /* Step 2: softmax(scale * q K^T + mask) V, one (query, head) at a time. */
        int failed = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
        for (int32_t i = 0; i < Tq; ++i) {
            for (int32_t h = 0; h < Hq; ++h) {
                const int32_t kvh = h / G;
                const int64_t pos = (int64_t)len - Tq + i;
                /* allowed keys are 0 .. nkeys-1 */
                int64_t nkeys = len;
                if (causal && pos + 1 < nkeys) nkeys = pos + 1;
                if (nkeys < 0) nkeys = 0;
                const int64_t row = (int64_t)(q0 + i) * Hq + h;
                double *o = out + row * d;
                for (int32_t e = 0; e < d; ++e) o[e] = 0.0;
                if (weights) for (int64_t j = 0; j < weights_stride; ++j) weights[row * weights_stride + j] = 0.0;
                if (nkeys == 0) { if (lse) lse[row] = -INFINITY; continue; }

                double *x = (double *)malloc((size_t)nkeys * sizeof(double));
                if (!x) { failed = 1; continue; }
                double m = -INFINITY;
                for (int64_t j = 0; j < nkeys; ++j) {
                    if (!visible(mods, s, pos, j)) { x[j] = -INFINITY; continue; }
                    const double *kr = Ks + (j * Hkv + kvh) * d;
                    double acc = 0.0;
                    for (int32_t e = 0; e < d; ++e) acc += widen(q, row * d + e, c->dtype) * kr[e];
                    x[j] = modded(mods, scale * acc, s, h, pos, j);
                    if (x[j] > m) m = x[j];
                }
                if (m == -INFINITY) { if (lse) lse[row] = -INFINITY; free(x); continue; }   /* nothing visible */
                double Z = 0.0;
                for (int64_t j = 0; j < nkeys; ++j) { x[j] = exp(x[j] - m); Z += x[j]; }
                for (int64_t j = 0; j < nkeys; ++j) {
                    const double w = x[j] / Z;
                    const double *vr = Vs + (j * Hkv + kvh) * d;
                    for (int32_t e = 0; e < d; ++e) o[e] += w * vr[e];
                    if (weights && j < weights_stride) weights[row * weights_stride + j] = w;
                }
                if (lse) lse[row] = m + log(Z);
                free(x);
            }
        }
        free(Ks); free(Vs);
        if (failed) return ORACLE_NO_MEMORY;
    }
    return ORACLE_OK;
}

int oracle_merge_partials(const double *o_parts, const double *lse_parts, int32_t n,
                          int32_t d, double *out, double *lse)
{
    if (n < 0 || d <= 0 || !out || (n > 0 && (!o_parts || !lse_parts))) return ORACLE_BAD_ARG;
    double M = -INFINITY;
    for (int32_t c = 0; c < n; ++c) if (lse_parts[c] > M) M = lse_parts[c];
    for (int32_t e = 0; e < d; ++e) out[e] = 0.0;
    if (M == -INFINITY) { if (lse) *lse = -INFINITY; return ORACLE_OK; }
    double Z = 0.0;
    for (int32_t c = 0; c < n; ++c) if (lse_parts[c] != -INFINITY) Z += exp(lse_parts[c] - M);
    for (int32_t c = 0; c < n; ++c) {
        if (lse_parts[c] == -INFINITY) continue;
        const double w = exp(lse_parts[c] - M) / Z;
        for (int32_t e = 0; e < d; ++e) out[e] += w * o_parts[(int64_t)c * d + e];
    }
    if (lse) *lse = M + log(Z);
    return ORACLE_OK;
}

int oracle_widen(const void *src, int64_t n, int32_t dtype, double *dst)
{
    if (!src || !dst || n < 0) return ORACLE_BAD_ARG;
    if (dtype != ORACLE_F32 && dtype != ORACLE_BF16 && dtype != ORACLE_F16) return ORACLE_BAD_ARG;
    for (int64_t i = 0; i < n; ++i) dst[i] = widen(src, i, dtype);
    return ORACLE_OK;
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
