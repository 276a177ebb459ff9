/*
 * pagedattn.h -- C ABI of the MI355X (gfx950) paged-KV attention library.
 *
 * The library implements the hot path of "Paged Attention Meets FlexAttention"
 * (arXiv 2506.07311): the KV cache of every sequence lives in fixed-size
 * physical pages of two global pools (K and V, Sec. III-B "Paged KV-Manager"),
 * a per-sequence block table of 32-bit entries maps logical block b to a
 * physical page (Algorithm 1), and attention reads the scattered pages in place
 * -- no contiguous copy (Sec. I-A, challenge 2) -- under the length mask of
 * Sec. III-B "FlexAttention Kernel".
 *
 * Conventions common to every entry point
 *   - Every array pointer is a DEVICE pointer owned by the caller.  The
 *     descriptor struct itself and all scalars are host values.
 *   - The library allocates no device memory and never synchronises: work is
 *     enqueued on `stream` (a hipStream_t passed as void*; NULL = the default
 *     stream) and results are valid once the caller has synchronised it.
 *   - Host-checkable violations (NULL pointer, unsupported shape, workspace too
 *     small, ...) are rejected before anything is launched and reported through
 *     the returned pa_status.  Device-side CONTENTS are caller preconditions and
 *     are not checked: block-table entries that are dereferenced lie in
 *     [0, num_pages); positions and lengths fit max_blocks * page_size; one
 *     append call never writes a slot twice.
 *   - batch == 0, T == 0 or total_q == 0 returns PA_OK without launching.
 *   - Index arithmetic is 64-bit: pools beyond 2^31 elements are fine.
 */
#ifndef PAGEDATTN_H
#define PAGEDATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    PA_OK = 0,
    PA_ERR_INVALID_ARG = 1,          /* NULL pointer, negative size, Hq % Hkv != 0, page size not a power of two */
    PA_ERR_UNSUPPORTED = 2,          /* dtype / head_dim / stride combination no kernel is written for            */
    PA_ERR_WORKSPACE_TOO_SMALL = 3,  /* workspace_bytes < paged_attention_workspace_bytes(...)                    */
    PA_ERR_HIP = 4,                  /* a HIP call reported an error                                              */
    PA_ERR_OUT_OF_PAGES = 5,         /* the page pool cannot satisfy a reservation (nothing was changed)          */
    PA_ERR_SCRATCH_LIMIT = 6         /* paged_attention_decode_static: the call needs more scratch than the array holds */
} pa_status;

typedef enum { PA_DTYPE_F32 = 0, PA_DTYPE_BF16 = 1, PA_DTYPE_F16 = 2 } pa_dtype;

/*
 * K and V live in two global pools of pages (Sec. III-B, Paged KV-Manager).
 * Algorithm 1 addresses them by the flat slot p = page * P + o; the literal
 * layout is therefore token-major [num_pages, page_size, num_kv_heads, head_dim]
 * with page_stride = P*Hkv*d, token_stride = Hkv*d, head_stride = d.  Strides
 * are in ELEMENTS and let a head-major pool [NP, Hkv, P, d] be described too.
 * head_dim is innermost and contiguous; every stride must be a multiple of
 * 16 bytes.  page_size must be a power of two (Algorithm 1, Require).
 * Supported: head_dim a multiple of 8 (bf16, fp16) / 4 (fp32), at most 256.
 * fp16 (the paper's own precision, Sec. III-B) computes like bf16: fp32 accumulation, outputs rounded to
 * nearest even.
 */
typedef struct {
    void*    k_cache;
    void*    v_cache;
    int64_t  page_stride;
    int64_t  token_stride;
    int64_t  head_stride;
    int32_t  num_pages;
    int32_t  page_size;
    int32_t  num_kv_heads;
    int32_t  head_dim;
    pa_dtype dtype;
} pa_kv_cache_desc;

/*
 * Algorithm 1, Assign.  For every appended token i in [0, T):
 *     s = seq_ids[i], t = positions[i], b = floor(t / P), o = t mod P,
 *     p = block_table[s][b] * P + o,   K[p] <- k_new[i],   V[p] <- v_new[i].
 * k_new, v_new : [T, Hkv, d] contiguous, cache dtype.  seq_ids, positions :
 * int32[T].  block_table : int32[batch, max_blocks] row-major.  The copy is
 * bytewise (bit-exact).  Writing one slot twice in a call is undefined.
 */
pa_status paged_kv_append(const pa_kv_cache_desc* cache, const void* k_new, const void* v_new,
                          const int32_t* seq_ids, const int32_t* positions, int32_t T,
                          const int32_t* block_table, int32_t batch, int32_t max_blocks, void* stream);

/*
 * Algorithm 1, Gather -- a verification utility; attention itself never makes
 * this copy.  For sequence s and t in [0, seq_lens[s]) the slot's Hkv*d
 * elements are copied bytewise to row cu_seq_lens[s] + t of out_k / out_v
 * ([sum(seq_lens), Hkv, d] contiguous).  cu_seq_lens : int32[batch + 1]
 * exclusive prefix sum of seq_lens.  max_seq_len : host upper bound of
 * seq_lens (sizes the grid without a device read).
 */
pa_status paged_kv_gather(const pa_kv_cache_desc* cache, void* out_k, void* out_v,
                          const int32_t* block_table, const int32_t* seq_lens, const int32_t* cu_seq_lens,
                          int32_t batch, int32_t max_blocks, int32_t max_seq_len, void* stream);

/*
 * Upper bound (pure host function) of the split-KV workspace the two attention
 * entry points need for these sizes: fp32 partial outputs and (max, sum)
 * statistics per (query, head, context chunk).  Pass total_q = batch for
 * decode (the bound then covers the decode entry points only; a prefill call
 * with total_q <= batch that is not plain decode keeps its few-query sequences
 * on the prefill kernel when the workspace has no room for their partials).
 * Always a multiple of 256; never 0.  Depends on the calling thread's
 * pa_set_option knobs and on the current device's compute-unit count.
 */
size_t paged_attention_workspace_bytes(int32_t batch, int32_t num_q_heads, int32_t head_dim,
                                       int32_t total_q, int32_t max_seq_len);

/*
 * Decode: one query token per sequence attends to its whole context.
 *     out[s,h,:] = sum_{j < len_s} softmax_j( scale * <q[s,h,:], K_s[j, floor(h/G), :]> ) V_s[j, floor(h/G), :]
 * where K_s[j] is the slot Algorithm 1 maps (s, j) to and G = Hq / Hkv.  Keys
 * j >= seq_lens[s] are masked by selection (Sec. III-B mask, read 0-based), so
 * unused slots may hold anything, NaN included.  seq_lens counts the tokens
 * already appended for this step.  seq_lens[s] == 0 gives out = 0, lse = -inf.
 * q, out : [batch, Hq, d] contiguous, cache dtype (fp32 accumulation, bf16
 * outputs rounded to nearest even).  lse : NULL or float[batch, Hq], natural
 * log-sum-exp of the scaled scores.  max_seq_len : host upper bound of
 * seq_lens, used to size the grid.  workspace : at least
 * paged_attention_workspace_bytes(batch, Hq, d, batch, max_seq_len) bytes,
 * 256-byte aligned; its contents need not be initialised.
 * Concurrency: calls on different streams may overlap when each has a workspace
 * of its own.  Calls whose plan splits a (sequence, KV head) over several
 * workgroups of one launch (few sequences, contexts of about 1 k - 8 k tokens)
 * also count arrivals in a ring of 16 counter windows inside the library, one
 * window per call in issue order: at most 16 such calls may be in flight on one
 * GPU at a time (a captured HIP graph keeps the window of the call it captured).
 */
pa_status paged_attention_decode(const pa_kv_cache_desc* cache, const void* q, void* out, float* lse,
                                 const int32_t* block_table, const int32_t* seq_lens, int32_t batch,
                                 int32_t num_q_heads, int32_t max_blocks, int32_t max_seq_len, float scale,
                                 void* workspace, size_t workspace_bytes, void* stream);

/*
 * paged_attention_decode for callers that can neither allocate device memory nor bring a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and results as
 * paged_attention_decode (bit-identical: the same kernels and the same plan), without the workspace: the split-KV
 * partials go to a 16 MiB array that lives in the library's device image (one copy per GPU, held until the process
 * ends).  The call allocates and frees nothing.  A call whose plan needs more than the array holds (partials are
 * (workgroups + batch) * Hq * (head_dim + 1) floats; about one workgroup per compute unit) is rejected with
 * PA_ERR_SCRATCH_LIMIT before anything is launched.  Every call on a GPU shares that GPU's array: calls that
 * overlap on one GPU (different streams, different host threads) race and must be serialised by the caller.
 * Nothing in the array needs to start at zero: the kernels write every partial they later read.
 */
pa_status paged_attention_decode_static(const pa_kv_cache_desc* cache, const void* q, void* out, float* lse,
                                        const int32_t* block_table, const int32_t* seq_lens, int32_t batch,
                                        int32_t num_q_heads, int32_t max_blocks, int32_t max_seq_len, float scale,
                                        void* stream);

/*
 * Prefill / general ragged form: sequence s contributes q_len_s =
 * cu_q_lens[s+1] - cu_q_lens[s] packed queries (cu_q_lens : int32[batch + 1],
 * the prefix-sum vector of Sec. III-B).  Query i of sequence s sits at absolute
 * position pos = seq_lens[s] - q_len_s + i and attends to keys
 *     j < seq_lens[s]            (causal == 0)
 *     j <= pos                   (causal != 0).
 * q, out : [total_q, Hq, d]; lse : NULL or float[total_q, Hq].  max_q_len :
 * host upper bound of q_len_s.  Other arguments as for decode (workspace sized
 * with this call's total_q).
 * q_len_s may be anything from 0 to seq_lens[s] and differ per sequence: a
 * chunk of a long prompt on top of cached context, decode rows (q_len 1) and
 * whole prompts can share one call (the jagged batch of Sec. III-B: sequence
 * ids are implied by the prefix sums).  A call with few query rows over a long
 * context is cut along the context and merged through the workspace.
 */
pa_status paged_attention_prefill(const pa_kv_cache_desc* cache, const void* q, void* out, float* lse,
                                  const int32_t* cu_q_lens, int32_t total_q, int32_t max_q_len,
                                  const int32_t* block_table, const int32_t* seq_lens, int32_t batch,
                                  int32_t num_q_heads, int32_t max_blocks, int32_t max_seq_len, float scale,
                                  int32_t causal, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Mask and score modifications in the sense of FlexAttention's mask_mod /
 * score_mod (Sec. II-C; Sec. III-B builds the paged mask out of one), for the
 * families this library builds in.  With pos the query's absolute position
 * (decode: seq_lens[s] - 1), on top of the length mask and the causal bound:
 *   window > 0       key j is visible only if |j - pos| < window            (sliding window)
 *   doc_ids != NULL  ... only if doc_ids[s][j] == doc_ids[s][pos]            (document mask); device
 *                    int32 [batch, doc_stride], indexed by logical position, doc_stride >= max_seq_len
 *   softcap > 0      score x = scale * <q, k> becomes softcap * tanh(x / softcap)
 *   alibi_slopes     then x becomes x + alibi_slopes[h] * (j - pos);  device float[Hq]
 *   user_mod != 0    then the visible() / score() pair of the user modification with that id, compiled into
 *                    every attention kernel from include/pagedattn_mods.h (the extension point: a mask or score
 *                    family is added there, in one header, without touching a kernel); an id the library
 *                    was not built with is PA_ERR_INVALID_ARG
 * A query left without any visible key gets out = 0, lse = -inf.  The kernels
 * are instantiated per combination of hooks at compile time: a call with
 * mods == NULL, or with every field off, runs exactly the unmodified kernels.
 * Sliding windows skip the context before the window instead of masking it.
 */
typedef struct {
    int32_t        window;
    float          softcap;
    const float*   alibi_slopes;
    const int32_t* doc_ids;
    int64_t        doc_stride;
    int32_t        user_mod;    /* 0 = none, else the kId of a modification listed in pagedattn_mods.h */
    const void*    user_data;   /* handed to that modification's hooks (device memory the hooks read) */
} pa_attn_mods;

/* paged_attention_decode / paged_attention_prefill with modifications; all other arguments as there. */
pa_status paged_attention_decode_mod(const pa_kv_cache_desc* cache, const void* q, void* out, float* lse,
                                     const int32_t* block_table, const int32_t* seq_lens, int32_t batch,
                                     int32_t num_q_heads, int32_t max_blocks, int32_t max_seq_len, float scale,
                                     const pa_attn_mods* mods, void* workspace, size_t workspace_bytes,
                                     void* stream);
pa_status paged_attention_prefill_mod(const pa_kv_cache_desc* cache, const void* q, void* out, float* lse,
                                      const int32_t* cu_q_lens, int32_t total_q, int32_t max_q_len,
                                      const int32_t* block_table, const int32_t* seq_lens, int32_t batch,
                                      int32_t num_q_heads, int32_t max_blocks, int32_t max_seq_len, float scale,
                                      int32_t causal, const pa_attn_mods* mods, void* workspace,
                                      size_t workspace_bytes, void* stream);

/*
 * One decode step as one call: Algorithm 1, Assign, for one new token per sequence, then decode over the context
 * that now ends with it.  Equivalent to
 *     paged_kv_append(cache, k_new, v_new, seq_ids = 0 .. batch-1, positions = seq_lens - 1, T = batch, ...)
 *     paged_attention_decode_mod(cache, q, out, lse, ..., mods, ...)
 * and bit-identical to that pair in the pools and in out / lse.  k_new, v_new : [batch, Hkv, d] contiguous, cache
 * dtype, 16-byte aligned; token s lands at position seq_lens[s] - 1 (seq_lens counts it already); a sequence with
 * seq_lens[s] == 0 receives no token and gives out = 0, lse = -inf.  mods may be NULL.  The point of the call is
 * the launch count: a step over short contexts (the range the paper measures, Sec. IV) is bound by launches and
 * memory round trips, and here the append runs inside the decode kernel itself: the wave (or workgroup) that
 * meets a sequence's last key stores the new rows into their slot and reads them from k_new / v_new, on every
 * decode kernel of the library.
 */
pa_status paged_decode_step(const pa_kv_cache_desc* cache, const void* k_new, const void* v_new, const void* q,
                            void* out, float* lse, const int32_t* block_table, const int32_t* seq_lens, int32_t batch,
                            int32_t num_q_heads, int32_t max_blocks, int32_t max_seq_len, float scale,
                            const pa_attn_mods* mods, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Debug utility: checks on the device the preconditions about device-side CONTENTS that the other entry points
 * assume and do not check.  counts (host, int64[3]) receives
 *   [0] block-table entries among the first ceil(seq_lens[s] / page_size) of a row that lie outside [0, num_pages)
 *   [1] sequences whose length is negative or exceeds max_blocks * page_size
 *   [2] appended tokens (seq_ids / positions, both NULL with T = 0) whose sequence id is outside [0, batch) or
 *       whose position is outside [0, max_blocks * page_size)
 * scratch : device memory, at least 32 bytes, 8-byte aligned (e.g. the attention workspace).  The call
 * SYNCHRONISES `stream` and returns PA_OK when the check ran, whatever it found.
 */
pa_status pa_debug_check(const pa_kv_cache_desc* cache, const int32_t* block_table, const int32_t* seq_lens,
                         int32_t batch, int32_t max_blocks, const int32_t* seq_ids, const int32_t* positions, int32_t T,
                         void* scratch, int64_t* counts, void* stream);

const char* pa_status_string(pa_status status);

/*
 * Tuning knobs, kept per host thread: they shape the calls (and the workspace
 * bound) of the thread that set them and nothing else.  name is one of
 *   "decode_chunk_tokens"  context tokens per split-KV workgroup of the portable kernel (0 = heuristic)
 *   "decode_workgroups"    workgroups the MFMA decode kernel spreads the batch's key tiles over
 *                          (0 = one per compute unit)
 *   "prefill_chunk_tokens" context tokens per workgroup of the MFMA prefill kernel (0 = heuristic: no split
 *                          unless the call has too few query rows to fill the machine); size the workspace
 *                          AFTER setting it
 *   "decode_short"         the one-launch decode kernel for short contexts (a workgroup per sequence and KV head,
 *                          no workspace, no merge launch): 0 = taken while the step is small enough for it to
 *                          pay (the default), 1 = whenever it supports the call, -1 = never
 *   "decode_short_splits"  workgroups per (sequence, KV head) of the one-launch decode kernel, 1 .. 16 (0 = as many
 *                          as fill the machine, at least 256 keys each); size the workspace AFTER setting it
 *   "step_append_kernel"   1 = paged_decode_step on the tile-stream kernel appends with a kernel launch of its own
 *                          instead of inside the decode kernel (for comparison)
 *   "no_small_q_route"     1 = the prefill entry point keeps sequences with few queries (q_len * G <= 16) on
 *                          the prefill kernel instead of handing them to the decode kernel
 *   "force_generic"        1 = always take the portable VALU kernels
 * Returns PA_ERR_INVALID_ARG for an unknown name or a value out of range.
 */
pa_status pa_set_option(const char* name, int64_t value);

/*
 * Measurement yardstick (no part of the method): reads bytes_each bytes of each of the two device buffers a and b
 * once, contiguously, 16 bytes per lane, and writes nothing -- the rate the memory system gives the plainest reader,
 * against which the achieved bandwidth of the decode kernels (Sec. IV measures the same step end to end) is judged.
 * bytes_each must be a positive multiple of 64 MiB; a, b and sink (16 bytes of device memory, never written) are
 * 16-byte aligned.  Timed like every other kernel through pa_profile_* under the name "pa_stream_read_kernel".
 */
pa_status pa_stream_read(const void* a, const void* b, size_t bytes_each, void* sink, void* stream);

/*
 * Per-kernel timing for benchmarks.  While enabled, every kernel launch of the
 * library is bracketed by a pair of HIP events recorded on the launch stream.
 * pa_profile_read synchronises those events and returns, for the kernel whose
 * name starts with `kernel_prefix`, the number of launches and their summed
 * duration in milliseconds since the last pa_profile_reset.  Not for use under
 * graph capture.
 */
pa_status pa_profile_enable(int32_t on);
pa_status pa_profile_reset(void);
pa_status pa_profile_read(const char* kernel_prefix, int32_t* launches, double* total_ms);

/*
 * ---------------------------------------------------------------------------
 * KV page manager (Algorithm 1 Reserve; Sec. III-B "Paged KV-Manager"; Sec. I-A
 * challenge 1: grow on demand, reclaim at once, share identical prefixes, all
 * in constant time per page).
 *
 * A pa_pool is a HOST object that owns the bookkeeping of num_pages physical
 * pages of page_size tokens: which pages are free, which sequence maps which
 * logical block to which page, and how many sequences reference each page.  It
 * never touches K/V data except in pa_pool_make_writable.  The free list is
 * lock-free: never-used pages come from an atomic bump pointer, recycled pages
 * from a tagged (ABA-safe) atomic stack, so reserving or releasing one page is
 * O(1) and calls for DIFFERENT sequences may run concurrently from several host
 * threads; calls for the SAME sequence must be serialised by the caller
 * (pa_pool_share_prefix counts as a call for both of its sequences).
 *
 * device_table (optional, may be NULL): the int32 [max_seqs, max_blocks] block
 * table in device memory that the attention entry points read.  Every call
 * that changes a sequence's row enqueues a copy of the changed entries on
 * `stream`, from a pinned staging ring that holds their values as of the call,
 * so the table is current for work enqueued later on the same stream and work
 * enqueued earlier still sees the earlier row.  Use ONE stream for all calls on
 * a pool (the ring's reuse is ordered by events on that stream); a page that
 * was released may be handed out again at once, which is safe for the same
 * reason.  Entries of unmapped blocks are -1.  pa_pool_destroy waits for the
 * device to go idle when a device table is attached.  A call changes the host
 * bookkeeping first and enqueues the row copy last: if that copy fails
 * (PA_ERR_HIP) the bookkeeping stands, the device row is stale for the
 * changed entries, and the next call that changes the same sequence's row
 * delivers them together with its own.
 * ---------------------------------------------------------------------------
 */
typedef struct pa_pool pa_pool;

/* Creates a pool.  num_pages, max_seqs, max_blocks > 0; page_size a power of two.
 * When device_table is given, all of its max_seqs * max_blocks entries are set to -1 (synchronously). */
pa_status pa_pool_create(pa_pool** pool, int32_t num_pages, int32_t page_size, int32_t max_seqs,
                         int32_t max_blocks, int32_t* device_table);
pa_status pa_pool_destroy(pa_pool* pool);

/* Growth policy of pa_pool_reserve.  PA_GROW_EXACT (default) is Algorithm 1 as printed: n = ceil(len / P).
 * PA_GROW_POW2 is the power-of-two cache allocation the paper's memory measurements mention (Sec. IV,
 * "Memory Utilization"): when a sequence must grow, its block count goes to the next power of two >= n
 * (capped at max_blocks), so a sequence growing token by token touches the free list O(log n) times; if the pool
 * runs short the call keeps what it could get as long as that is >= n. */
enum { PA_GROW_EXACT = 0, PA_GROW_POW2 = 1 };
pa_status pa_pool_set_growth(pa_pool* pool, int32_t policy);

/* Algorithm 1, Reserve, incremental: makes sure sequence seq owns n = ceil(len / page_size) blocks, popping
 * the missing ones from the free list (a sequence never shrinks here).  PA_ERR_OUT_OF_PAGES leaves the
 * sequence as it was; PA_ERR_INVALID_ARG if n > max_blocks or seq is out of range. */
pa_status pa_pool_reserve(pa_pool* pool, int32_t seq, int32_t len, void* stream);

/* Drops every block of the sequence; pages whose reference count reaches zero return to the free list. */
pa_status pa_pool_release(pa_pool* pool, int32_t seq, void* stream);

/* Prefix sharing: dst (which must hold no blocks) maps the first floor(prefix_tokens / page_size) blocks of src,
 * whole pages only, and their reference counts grow by one.  No data is copied. */
pa_status pa_pool_share_prefix(pa_pool* pool, int32_t dst_seq, int32_t src_seq, int32_t prefix_tokens, void* stream);

/* Copy-on-write: if the page holding `position` of seq is referenced by more than one sequence, seq gets a
 * private copy (one page of K and of V is copied on `stream` inside the pools `cache` describes) and the shared
 * page loses one reference.  A no-op for a private page.  Call before appending into a page that may be shared. */
pa_status pa_pool_make_writable(pa_pool* pool, const pa_kv_cache_desc* cache, int32_t seq, int32_t position,
                                void* stream);

/* Introspection (host, no synchronisation): free pages; blocks of a sequence; copy of a sequence's row into
 * host_row[0 .. capacity) (returns PA_ERR_INVALID_ARG if capacity is too small); references of a page. */
int32_t   pa_pool_num_free(const pa_pool* pool);
int32_t   pa_pool_num_blocks(const pa_pool* pool, int32_t seq);
pa_status pa_pool_get_row(const pa_pool* pool, int32_t seq, int32_t* host_row, int32_t capacity);
int32_t   pa_pool_refcount(const pa_pool* pool, int32_t page);

#ifdef __cplusplus
}
#endif
#endif /* PAGEDATTN_H */
