/*
 * pagedattn_mods.h -- the extension point for user-defined mask and score modifications.
 *
 * The paper builds its paged attention out of FlexAttention because that interface lets a caller state the
 * visibility predicate (mask_mod) and a score rewrite (score_mod) as small functions that are compiled into the
 * attention kernel (Sec. II-C; Sec. III-B "FlexAttention Kernel").  This header is that interface for the HIP
 * kernels of this library: a modification is a struct with two static device functions, listed in
 * PA_USER_MODS below; the library's build instantiates every attention kernel (matrix-core decode and prefill,
 * portable kernel) once per listed struct, and a call selects one through pa_attn_mods.user_mod = <its kId>.
 * Adding a family means adding a struct and a line to the list in THIS file (and, for the tests, the same predicate
 * in the CPU oracle); no kernel source changes.
 *
 * Contract.  For query row r of sequence `seq` (absolute position `pos`, context length `len`, query head `head`)
 * and every key j that the length mask (j < len), the causal bound (j <= pos, when the call is causal) and the
 * built-in hooks of pa_attn_mods leave visible, the kernels evaluate
 *     visible(c, j)    -> false removes the key (masked by selection: its slot may hold anything, NaN included)
 *     score(c, j, x)   -> the score that enters the softmax; x = scale * <q, k_j> after the built-in soft cap and
 *                         position bias, in natural units (the kernel converts to its own base-2 domain); a
 *                         template over the score type F: float in the 16-bit kernels, double where fp32 pools
 *                         keep their scores in fp64
 * with c = { user_data, seq, head, pos, len }.  Both must be pure functions of their arguments and of memory that
 * user_data points to (device memory the caller owns; read-only for the kernel).  They run once per (row, key) pair on
 * the hot path: keep them to a few instructions.  A row left without any visible key gets out = 0, lse = -inf.
 * Tiles are not skipped on account of a user mask (only the built-in window and document masks know how to), so a
 * very sparse user mask costs what the unmasked call costs.  Rows under a user modification always carry their
 * softmax weights as two 16-bit terms (a user mask may leave a row a handful of keys).
 */
#ifndef PAGEDATTN_MODS_H
#define PAGEDATTN_MODS_H

#include <stdint.h>

#if defined(__HIPCC__)
#define PA_MOD_FN __device__ __forceinline__ static
#else
#define PA_MOD_FN inline static
#endif

struct pa_mod_ctx {
    const void* user_data;   /* pa_attn_mods.user_data */
    int32_t seq;             /* sequence index of the row */
    int32_t head;            /* query head of the row */
    int32_t pos;             /* absolute position of the query: seq_lens[seq] - q_len + i */
    int32_t len;             /* seq_lens[seq] */
};

/*
 * Prefix-LM (the shipped example, kId 1): the first prefix_len[seq] tokens of a sequence see each other in both
 * directions, everything after them is causal:  key j is visible iff  j <= pos  or  j < prefix_len[seq].  Use it
 * with causal = 0 (a causal call has removed j > pos already).  Its score hook adds prefix_bias to the scores of
 * prefix keys (0 for the plain mask).  user_data points to a pa_prefix_lm_data in device memory.
 */
struct pa_prefix_lm_data {
    const int32_t* prefix_len;   /* device, int32[batch] */
    float prefix_bias;
};

struct pa_mod_prefix_lm {
    static constexpr int32_t kId = 1;
    PA_MOD_FN bool visible(const pa_mod_ctx& c, int32_t j)
    {
        const pa_prefix_lm_data* d = static_cast<const pa_prefix_lm_data*>(c.user_data);
        return j <= c.pos || j < d->prefix_len[c.seq];
    }
    template <typename F>
    PA_MOD_FN F score(const pa_mod_ctx& c, int32_t j, F x)
    {
        const pa_prefix_lm_data* d = static_cast<const pa_prefix_lm_data*>(c.user_data);
        return j < d->prefix_len[c.seq] ? x + (F)d->prefix_bias : x;
    }
};

/* The list the build instantiates: X(struct name), one per line. */
#define PA_USER_MODS(X) \
    X(pa_mod_prefix_lm)

#endif /* PAGEDATTN_MODS_H */
