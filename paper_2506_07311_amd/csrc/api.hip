// C ABI of the paged-attention library: argument validation, split planning and kernel dispatch.
// Nothing here touches device memory; every check is a host check made before the first launch.
#include <string.h>

#include <mutex>
#include <string>
#include <vector>

#include "common.h"

// Scratch of paged_attention_decode_static: the split-KV partials of a decode call, for callers that cannot bring
// a workspace.  One copy per GPU, held until the process ends.  In host code this name is only a handle for
// hipGetSymbolAddress; kernels receive the address that call returns.
constexpr size_t kStaticScratchBytes = (size_t)16 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace pa {

namespace {

struct Options {
    int64_t decode_chunk_tokens = 0;
    int64_t decode_workgroups = 0;
    int64_t force_generic = 0;
    int64_t prefill_chunk_tokens = 0;
    int64_t no_small_q_route = 0;
    int64_t step_append_kernel = 0;   // 1 = paged_decode_step on the tile stream appends with a kernel of its own
                                      // (0: every decode kernel performs the step's append itself)
    int64_t decode_short = 0;      // 0 = heuristic, 1 = whenever the one-launch kernel supports the call, -1 = never
    int64_t decode_short_splits = 0;   // workgroups per (sequence, KV head) of the one-launch kernel; 0 = heuristic
};
thread_local Options g_opt;       // per host thread: a thread's knobs shape only the calls it makes itself

// Compute units of the current device (the tile-stream decode launches one workgroup per CU by default).
int32_t device_cus()
{
    static int32_t cached[64] = {0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    if (cached[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
        cached[dev] = n;
    }
    return cached[dev];
}

struct ProfileRecord {
    std::string kernel;
    hipEvent_t start;
    hipEvent_t stop;
};
bool g_profile_on = false;
std::vector<ProfileRecord> g_records;
std::vector<hipEvent_t> g_spare_events;   // events of records that were reset, reused instead of created anew
std::mutex g_profile_mutex;

bool take_event(hipEvent_t* e)
{
    if (!g_spare_events.empty()) {
        *e = g_spare_events.back();
        g_spare_events.pop_back();
        return true;
    }
    return hipEventCreate(e) == hipSuccess;
}

inline int elem_bytes(pa_dtype t) { return t == PA_DTYPE_F32 ? 4 : 2; }

bool is_pow2(int32_t x) { return x > 0 && (x & (x - 1)) == 0; }

// Is `id` the kId of a user modification the library was built with?
bool user_mod_known(int32_t id)
{
#define PA_USER_CASE(U) if (id == U::kId) return true;
    PA_USER_MODS(PA_USER_CASE)
#undef PA_USER_CASE
    return false;
}

}  // namespace

pa_status check_cache(const pa_kv_cache_desc* c)
{
    if (!c || !c->k_cache || !c->v_cache) return PA_ERR_INVALID_ARG;
    if (c->dtype != PA_DTYPE_F32 && c->dtype != PA_DTYPE_BF16 && c->dtype != PA_DTYPE_F16) return PA_ERR_UNSUPPORTED;
    if (c->num_pages <= 0 || c->num_kv_heads <= 0 || c->head_dim <= 0) return PA_ERR_INVALID_ARG;
    if (!is_pow2(c->page_size)) return PA_ERR_INVALID_ARG;   // Algorithm 1 requires a power of two
    const int epv = 16 / elem_bytes(c->dtype);
    if (c->head_dim % epv != 0 || c->head_dim > 256) return PA_ERR_UNSUPPORTED;
    if (c->page_stride <= 0 || c->token_stride <= 0 || c->head_stride <= 0) return PA_ERR_INVALID_ARG;
    if (c->page_stride % epv || c->token_stride % epv || c->head_stride % epv) return PA_ERR_UNSUPPORTED;
    if (((uintptr_t)c->k_cache | (uintptr_t)c->v_cache) & 15) return PA_ERR_UNSUPPORTED;
    return PA_OK;
}

namespace {

int32_t nsplit_bound(int32_t max_seq_len)
{
    int64_t n = ((int64_t)max_seq_len + kMinChunk - 1) / kMinChunk;
    if (n < 1) n = 1;
    if (n > kMaxSplits) n = kMaxSplits;
    return (int32_t)n;
}

// Context tokens per split-KV workgroup.  Chunks are a multiple of max(P, 32) so that a chunk starts on a
// page boundary and on a 32-key MFMA tile; their number never exceeds the bound the workspace is sized by.
SplitPlan plan_decode(int32_t batch, int32_t max_seq_len, int32_t page_size)
{
    const int32_t unit = page_size > 32 ? page_size : 32;
    int64_t chunk = g_opt.decode_chunk_tokens;
    if (chunk <= 0) {
        // aim at a few thousand (sequence, chunk) work items so that 256 CUs stay busy and ragged
        // batches balance, but keep chunks long enough to amortise a workgroup's start-up
        const int64_t tokens = (int64_t)batch * max_seq_len;
        chunk = kMinChunk;
        while (chunk < 2048 && tokens / chunk > 4096) chunk *= 2;
    }
    chunk = (chunk + unit - 1) / unit * unit;
    const int32_t bound = nsplit_bound(max_seq_len);
    while (((int64_t)max_seq_len + chunk - 1) / chunk > bound) chunk *= 2;
    SplitPlan p;
    p.chunk = (int32_t)chunk;
    p.nsplit = (int32_t)(((int64_t)max_seq_len + chunk - 1) / chunk);
    if (p.nsplit < 1) p.nsplit = 1;
    return p;
}

size_t align256(size_t x) { return (x + 255) / 256 * 256; }

// Context split of the MFMA prefill kernel.  The kernel gets one workgroup per (128-row tile, head group); the
// host knows only total_q and batch, so it bounds the live tiles by total_q * pack / 128 + batch.  When that fills
// the machine there is no split; a call with few query rows over a long context (a chunk of a long prompt, a
// mixed batch that is mostly decode rows) is cut along the context into chunks of at least kPrefillMinChunk
// tokens until about kPrefillTargetWGs work items exist.  A pure function of its arguments: the workspace size is
// computed from the same rule with the largest packing.
constexpr int32_t kPrefillMinChunk = 1024;
constexpr int64_t kPrefillTargetWGs = 1024;
constexpr int64_t kPrefillFullWGs = 512;

SplitPlan plan_prefill(int32_t batch, int32_t num_q_heads, int32_t log2_pack, int32_t total_q, int32_t max_seq_len,
                       int32_t page_size)
{
    SplitPlan p;
    p.chunk = max_seq_len > 0 ? max_seq_len : 1;
    p.nsplit = 1;
    if (g_opt.prefill_chunk_tokens > 0) {
        const int64_t unit = page_size > 64 ? page_size : 64;
        int64_t chunk = (g_opt.prefill_chunk_tokens + unit - 1) / unit * unit;
        while (((int64_t)max_seq_len + chunk - 1) / chunk > kMaxSplits) chunk *= 2;
        if (chunk < max_seq_len) {
            p.chunk = (int32_t)chunk;
            p.nsplit = (int32_t)(((int64_t)max_seq_len + chunk - 1) / chunk);
        }
        return p;
    }
    const int64_t wgs = (((int64_t)total_q << log2_pack) / 128 + batch) * (num_q_heads >> log2_pack);
    if (wgs >= kPrefillFullWGs || max_seq_len < 2 * kPrefillMinChunk) return p;
    int64_t n = (kPrefillTargetWGs + wgs - 1) / wgs;
    if (n > max_seq_len / kPrefillMinChunk) n = max_seq_len / kPrefillMinChunk;
    if (n > kMaxSplits) n = kMaxSplits;
    if (n < 2) return p;
    const int64_t unit = page_size > 64 ? page_size : 64;
    int64_t chunk = ((int64_t)max_seq_len + n - 1) / n;
    chunk = (chunk + unit - 1) / unit * unit;
    if (chunk >= max_seq_len) return p;
    p.chunk = (int32_t)chunk;
    p.nsplit = (int32_t)(((int64_t)max_seq_len + chunk - 1) / chunk);
    return p;
}

// Largest number of chunks plan_prefill can choose for these sizes, whatever the packing and page size.
int32_t prefill_nsplit_bound(int32_t batch, int32_t num_q_heads, int32_t total_q, int32_t max_seq_len)
{
    if (g_opt.prefill_chunk_tokens > 0) return kMaxSplits;
    int32_t best = 1;
    for (int32_t lg = 0; lg <= 4; ++lg) {
        if (num_q_heads % (1 << lg)) break;
        const SplitPlan p = plan_prefill(batch, num_q_heads, lg, total_q, max_seq_len, 1);
        if (p.nsplit > best) best = p.nsplit;
    }
    return best;
}

// Workgroups along the tile stream for the MFMA decode kernel: one per compute unit and KV-head group, and more when
// that leaves fewer than four waves per compute unit (a workgroup holds one wave per KV head: few KV heads, as on one
// shard of a tensor-parallel model, mean small workgroups; `slices` = grid slices of 16 heads for groups above 16) --
// but never so many that a workgroup gets fewer than two 32-key tiles of the longest possible stream.
int32_t plan_stream_wgs(int32_t batch, int32_t max_seq_len, int32_t head_groups, int32_t num_kv_heads, int32_t slices)
{
    int64_t target = g_opt.decode_workgroups;
    if (target <= 0) {
        target = device_cus() / head_groups;
        const int64_t by_waves = 4LL * device_cus() / ((int64_t)num_kv_heads * (slices < 1 ? 1 : slices));
        if (by_waves > target) target = by_waves;
    }
    if (target < 1) target = 1;
    const int64_t tiles = (int64_t)batch * ((max_seq_len + 31) / 32);
    int64_t n = tiles / 2;
    if (n > target) n = target;
    if (n > kMaxDecodeWGs) n = kMaxDecodeWGs;
    if (n < 1) n = 1;
    return (int32_t)n;
}

// One launch instead of tile stream + merge: pays while a step is bound by launches and memory round trips.  A
// workgroup of the one-launch kernel streams its share of a (sequence, KV head) at about 55 GB/s, so its time is
// about 4 us + 9 us per 512 KB, against a floor of 12-16 us for tile stream + merge.  With few sequences the
// kernel puts several workgroups on a (sequence, KV head) -- as many as fill the machine once (a compute unit holds
// one workgroup of this kernel: its eight waves take the whole register file), at least 256 keys each -- which
// merge through the workspace inside the same launch; the route is taken while a workgroup's share stays within
// 512 KB of K and V rows (1024 tokens at head_dim <= 128, 512 at head_dim 256: rows twice as long).  Beyond that
// the tile stream's whole-row reads and equal split use the memory system better.  Measured, 32 / 8 heads, one box:
// 8 x 1024 tokens 10.6 us with 4 workgroups per (sequence, KV head) against 14.3 with one (15.5 tile stream + merge),
// 8 x 2048 16.9 against 23.6 (20.7), 8 x 4096 26.7 against 41.9 (29.5), 1 x 8192 19.9 against 75 (20.2).
constexpr int64_t kShortMaxRowBytes = 1024 * 512;   // context tokens x bytes of a K row and a V row (>= 512) per workgroup
constexpr int64_t kShortMaxWGsPerCU = 2;
constexpr int32_t kShortMinSplitKeys = 256;

int64_t short_units(const AttnArgs& a)
{
    return (int64_t)a.batch * a.cache.num_kv_heads * ((a.num_q_heads / a.cache.num_kv_heads + 15) / 16);
}

// Workgroups per (sequence, KV head, slice of 16 heads) of the one-launch kernel.
int32_t plan_short_splits(const AttnArgs& a)
{
    const int64_t units = short_units(a);
    if (units > kShortMaxUnits) return 1;
    int64_t n = g_opt.decode_short_splits;
    if (n <= 0) {
        n = device_cus() / units;
        const int64_t by_keys = a.max_seq_len / kShortMinSplitKeys;
        if (n > by_keys) n = by_keys;
    }
    if (n > kShortMaxSplit) n = kShortMaxSplit;
    return n < 1 ? 1 : (int32_t)n;
}

bool short_decode_pays(const AttnArgs& a, int32_t nsplit)
{
    if (g_opt.decode_workgroups > 0) return false;     // the caller shapes the tile stream: keep it
    const int64_t row_bytes = 4LL * (a.cache.head_dim > 128 ? a.cache.head_dim : 128);
    const int64_t share = ((int64_t)a.max_seq_len + nsplit - 1) / nsplit;
    return share * row_bytes <= kShortMaxRowBytes && short_units(a) * nsplit <= kShortMaxWGsPerCU * device_cus();
}

// Partials of the one-launch kernel's workgroups when a call splits: at most kShortMaxWGsPerCU per compute unit
// (or the forced number per unit), 16 rows of head_dim floats plus maxima and sums each.
size_t short_split_workspace_bytes(int32_t batch, int32_t hq, int32_t d)
{
    // units <= batch * hq (group size 1, one slice); the heuristic never exceeds two workgroups per compute unit
    int64_t wgs = kShortMaxWGsPerCU * device_cus();
    if (g_opt.decode_short_splits > 1) wgs = (int64_t)batch * hq * g_opt.decode_short_splits;
    return align256(decode_short_part_floats(wgs, d) * sizeof(float));
}

size_t stream_workspace_bytes(int32_t batch, int32_t hq, int32_t d, int32_t wgs)
{
    const size_t parts = (size_t)wgs + batch;
    return align256(parts * hq * d * sizeof(float)) + align256(parts * hq * sizeof(float)) +
           2 * align256((size_t)batch * sizeof(int32_t));
}

// Workgroups of the decode kernel when it runs the few-query sequences of a prefill call; its partials there take
// 16 rows per KV head, so the count is held to kSmallRouteMaxWGs and to kSmallRouteMaxHeadWGs / Hkv (a workgroup
// holds up to eight KV heads: about one workgroup per compute unit either way).
constexpr int32_t kSmallRouteMaxWGs = 256;
constexpr int32_t kSmallRouteMaxHeadWGs = 2048;

int32_t small_route_wgs_cap(int32_t num_kv_heads)
{
    const int32_t by_heads = kSmallRouteMaxHeadWGs / num_kv_heads;
    return by_heads < 1 ? 1 : by_heads < kSmallRouteMaxWGs ? by_heads : kSmallRouteMaxWGs;
}

size_t small_route_bytes(int32_t wgs, int32_t batch, int32_t num_kv_heads, int32_t d)
{
    const size_t rows = ((size_t)wgs + batch) * num_kv_heads * 16;
    return align256(rows * d * sizeof(float)) + align256(rows * sizeof(float)) +
           2 * align256((size_t)batch * sizeof(int32_t));
}

// Bound of small_route_bytes over every KV-head count that divides hq: wgs * Hkv <= kSmallRouteMaxHeadWGs, Hkv <= hq.
size_t small_route_workspace_bytes(int32_t batch, int32_t hq, int32_t d)
{
    const size_t rows = ((size_t)kSmallRouteMaxHeadWGs + (size_t)batch * hq) * 16;
    return align256(rows * d * sizeof(float)) + align256(rows * sizeof(float)) +
           2 * align256((size_t)batch * sizeof(int32_t));
}

// Largest tile-stream grid plan_stream_wgs can choose for a call with hq query heads: head_groups >= 1 and
// Hkv * slices >= hq / 16.
int32_t stream_wgs_bound(int32_t batch, int32_t hq, int32_t max_seq_len)
{
    int64_t n = g_opt.decode_workgroups;
    if (n <= 0) {
        n = device_cus();
        const int64_t by_waves = 64LL * device_cus() / hq;
        if (by_waves > n) n = by_waves;
    }
    const int64_t tiles = (int64_t)batch * ((max_seq_len + 15) / 16);
    if (n > tiles / 2) n = tiles / 2;
    if (n > kMaxDecodeWGs) n = kMaxDecodeWGs;
    return n < 1 ? 1 : (int32_t)n;
}

size_t part_o_bytes(int64_t rows, int32_t hq, int32_t d, int32_t nsplit)
{
    return align256((size_t)rows * hq * nsplit * d * sizeof(float));
}

size_t part_lse_bytes(int64_t rows, int32_t hq, int32_t nsplit)
{
    return align256((size_t)rows * hq * nsplit * sizeof(float));
}

// The workspace of a call.  The public entry points promise the bound paged_attention_workspace_bytes() and are
// checked against it (bound = true); the entry point that brings its own scratch array is checked against what the
// call's plan really uses.
struct Workspace {
    void* ptr;
    size_t bytes;
    bool bound;
};

pa_status run_attention(const pa_kv_cache_desc* cache, const void* q, void* out, float* lse,
                        const int32_t* cu_q_lens, int32_t total_q, int32_t max_q_len, const int32_t* block_table,
                        const int32_t* seq_lens, int32_t batch, int32_t num_q_heads, int32_t max_blocks,
                        int32_t max_seq_len, float scale, int32_t causal, const pa_attn_mods* mods,
                        const Workspace& ws, void* stream, bool decode, const void* k_new = nullptr,
                        const void* v_new = nullptr)
{
    pa_status st = check_cache(cache);
    if (st != PA_OK) return st;
    if (batch < 0 || total_q < 0 || max_blocks < 0 || max_seq_len < 0 || max_q_len < 0) return PA_ERR_INVALID_ARG;
    if (num_q_heads <= 0 || num_q_heads % cache->num_kv_heads != 0) return PA_ERR_INVALID_ARG;
    if (batch == 0 || total_q == 0) return PA_OK;
    if (!q || !out || !block_table || !seq_lens || (!decode && !cu_q_lens)) return PA_ERR_INVALID_ARG;
    if (((uintptr_t)q | (uintptr_t)out) & 15) return PA_ERR_UNSUPPORTED;
    if ((int64_t)max_blocks * cache->page_size < max_seq_len) return PA_ERR_INVALID_ARG;
    if (!(scale == scale)) return PA_ERR_INVALID_ARG;
    ModArgs m = {0, 0.f, nullptr, nullptr, 0, 0, nullptr};
    if (mods) {
        if (mods->window < 0 || !(mods->softcap >= 0.f) || mods->softcap > 3.0e38f) return PA_ERR_INVALID_ARG;
        if (mods->doc_ids && mods->doc_stride < max_seq_len) return PA_ERR_INVALID_ARG;
        if (mods->user_mod != 0 && !user_mod_known(mods->user_mod)) return PA_ERR_INVALID_ARG;
        m.user_mod = mods->user_mod;
        m.user_data = mods->user_mod ? mods->user_data : nullptr;
        m.window = mods->window;
        m.softcap = mods->softcap;
        m.alibi_slopes = mods->alibi_slopes;
        m.doc_ids = mods->doc_ids;
        m.doc_stride = mods->doc_ids ? mods->doc_stride : 0;
    }
    if (ws.bound) {
        const size_t need = paged_attention_workspace_bytes(batch, num_q_heads, cache->head_dim, total_q, max_seq_len);
        if (!ws.ptr || ws.bytes < need) return PA_ERR_WORKSPACE_TOO_SMALL;
    }
    if ((uintptr_t)ws.ptr & 255) return PA_ERR_INVALID_ARG;
    // a prefill call whose every sequence brings exactly one query is a decode call (its causal bound is the length
    // mask: the query sits at the last position)
    if (!decode && max_q_len == 1 && total_q == batch) decode = true;

    AttnArgs a;
    a.cache = make_view(cache);
    a.dtype = cache->dtype;
    a.q = q;
    a.out = out;
    a.lse = lse;
    a.cu_q_lens = decode ? nullptr : cu_q_lens;
    a.block_table = block_table;
    a.seq_lens = seq_lens;
    a.batch = batch;
    a.total_q = total_q;
    a.max_q_len = max_q_len;
    a.num_q_heads = num_q_heads;
    a.max_blocks = max_blocks;
    a.max_seq_len = max_seq_len;
    a.scale = scale;
    a.causal = causal ? 1 : 0;
    a.plan.chunk = max_seq_len > 0 ? max_seq_len : 1;
    a.plan.nsplit = 1;
    a.part_o = nullptr;
    a.part_lse = nullptr;
    a.stream_split = 0;
    a.num_wgs = 0;
    a.seg_first = a.seg_last = nullptr;
    a.skip_small = 0;
    a.mods = m;
    a.has_mods = m.window > 0 || m.softcap > 0.f || m.alibi_slopes || m.doc_ids || m.user_mod != 0;
    a.k_new = k_new;
    a.v_new = v_new;
    a.short_nsplit = 1;
    a.short_part = nullptr;
    a.short_arrive = nullptr;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    char* const base = reinterpret_cast<char*>(ws.ptr);
    const int32_t d = cache->head_dim;

    // tile-stream partials of the decode kernel at `p`: outputs, LSEs, first / last workgroup per sequence
    auto place_stream = [&](AttnArgs& b, char* p, size_t rows) {
        b.part_o = reinterpret_cast<float*>(p);
        p += align256(rows * d * sizeof(float));
        b.part_lse = reinterpret_cast<float*>(p);
        p += align256(rows * sizeof(float));
        b.seg_first = reinterpret_cast<int32_t*>(p);
        p += align256((size_t)batch * sizeof(int32_t));
        b.seg_last = reinterpret_cast<int32_t*>(p);
    };

    if (decode) {
        if (!g_opt.force_generic && g_opt.decode_short >= 0 && decode_short_supported(a)) {
            const int32_t nsplit = plan_short_splits(a);
            if (g_opt.decode_short > 0 || short_decode_pays(a, nsplit)) {
                a.short_nsplit = nsplit;
                a.short_part = reinterpret_cast<float*>(base);
                if (nsplit > 1 &&
                    ws.bytes < decode_short_part_floats(short_units(a) * nsplit, d) * sizeof(float))
                    return PA_ERR_WORKSPACE_TOO_SMALL;
                return launch_decode_short(a, s);          // with k_new / v_new: the append happens in this launch
            }
        }
        const bool stream_route = !g_opt.force_generic && decode_mfma_supported(a);
        if (stream_route) {
            const int32_t head_groups = cache->num_kv_heads / decode_mfma_heads_per_wg(cache->num_kv_heads, d);
            a.stream_split = 1;
            a.num_wgs = plan_stream_wgs(batch, max_seq_len, head_groups, cache->num_kv_heads,
                                        (num_q_heads / cache->num_kv_heads + 15) / 16);
            if (ws.bytes < stream_workspace_bytes(batch, num_q_heads, d, a.num_wgs)) return PA_ERR_WORKSPACE_TOO_SMALL;
            place_stream(a, base, ((size_t)a.num_wgs + batch) * num_q_heads);
            if (a.k_new && g_opt.step_append_kernel) {     // append as a launch of its own, then attend
                st = launch_kv_append_last(cache, k_new, v_new, seq_lens, block_table, batch, max_blocks, s);
                if (st != PA_OK) return st;
                a.k_new = a.v_new = nullptr;
            }                                              // (otherwise the decode kernel appends by itself)
            st = launch_decode_mfma(a, s);
            if (st != PA_OK) return st;
            return launch_merge(a, s);
        }
        a.plan = plan_decode(batch, max_seq_len, cache->page_size);
        const size_t po = part_o_bytes(batch, num_q_heads, d, a.plan.nsplit);
        if (a.plan.nsplit > 1 && ws.bytes < po + part_lse_bytes(batch, num_q_heads, a.plan.nsplit))
            return PA_ERR_WORKSPACE_TOO_SMALL;
        a.part_o = reinterpret_cast<float*>(base);
        a.part_lse = reinterpret_cast<float*>(base + po);
        st = launch_attention_generic(a, s);
        if (st != PA_OK) return st;
        if (a.plan.nsplit > 1) st = launch_merge(a, s);
        return st;
    }
    if (!g_opt.force_generic && prefill_mfma_supported(a)) {
        // Jagged batch: sequences with few queries (q_len * G <= 16: decode rows, a few speculative tokens) are
        // bound by streaming their context once, which the decode kernel's equal-work tile stream does best; the
        // others go to the prefill kernel.  Both kernels decide per sequence from cu_q_lens on the device; the
        // host only skips a launch that cannot find work.
        const int32_t G = num_q_heads / cache->num_kv_heads;
        const bool uniform_q = (int64_t)batch * max_q_len == total_q;      // every sequence has max_q_len queries
        bool may_have_small = !g_opt.no_small_q_route && decode_mfma_supported(a) && G <= 16 &&
                              !(uniform_q && (int64_t)max_q_len * G > 16);
        const SplitPlan pp = plan_prefill(batch, num_q_heads, prefill_mfma_log2_pack(num_q_heads, cache->num_kv_heads),
                                          total_q, max_seq_len, cache->page_size);
        const size_t split_bytes =
            pp.nsplit > 1 ? part_o_bytes(total_q, num_q_heads, d, pp.nsplit) + part_lse_bytes(total_q, num_q_heads, pp.nsplit)
                          : 0;
        int32_t small_wgs = 0;
        if (may_have_small) {
            const int32_t head_groups = cache->num_kv_heads / decode_mfma_heads_per_wg(cache->num_kv_heads, d);
            small_wgs = plan_stream_wgs(batch, max_seq_len, head_groups, cache->num_kv_heads, 1);
            const int32_t cap = small_route_wgs_cap(cache->num_kv_heads);
            if (small_wgs > cap) small_wgs = cap;
            // The route is an optimisation: a workspace without room for its partials (a call with total_q == batch
            // is promised the decode bound only) keeps those sequences on the prefill kernel.
            if (ws.bytes < split_bytes + small_route_bytes(small_wgs, batch, cache->num_kv_heads, d))
                may_have_small = false;
        }
        const bool may_have_large = (int64_t)max_q_len * G > 16 || !may_have_small;
        if (ws.bytes < split_bytes) return PA_ERR_WORKSPACE_TOO_SMALL;
        if (may_have_large) {
            AttnArgs b = a;
            b.skip_small = may_have_small ? 1 : 0;
            b.plan = pp;
            b.part_o = reinterpret_cast<float*>(base);
            b.part_lse = reinterpret_cast<float*>(base + part_o_bytes(total_q, num_q_heads, d, pp.nsplit));
            st = launch_prefill_mfma(b, s);
            if (st != PA_OK) return st;
        }
        if (may_have_small) {
            AttnArgs b = a;
            b.stream_split = 1;
            b.num_wgs = small_wgs;
            place_stream(b, base + split_bytes, ((size_t)small_wgs + batch) * cache->num_kv_heads * 16);
            st = launch_decode_mfma(b, s);
            if (st != PA_OK) return st;
            st = launch_merge(b, s);
        }
        return st;
    }
    return launch_attention_generic(a, s);
}

// Device address of this GPU's copy of `scratch`, looked up once per device with that device current.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

pa_status static_scratch(void** ptr)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return PA_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return PA_ERR_HIP;
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return PA_OK;
}

}  // namespace


void profile_begin(const char* kernel, hipStream_t stream)
{
    if (!g_profile_on) return;
    std::lock_guard<std::mutex> lock(g_profile_mutex);
    ProfileRecord r;
    r.kernel = kernel;
    if (!take_event(&r.start)) return;
    if (!take_event(&r.stop)) {
        g_spare_events.push_back(r.start);
        return;
    }
    (void)hipEventRecord(r.start, stream);
    g_records.push_back(r);
}

void profile_end(hipStream_t stream)
{
    if (!g_profile_on) return;
    std::lock_guard<std::mutex> lock(g_profile_mutex);
    if (!g_records.empty()) (void)hipEventRecord(g_records.back().stop, stream);
}

}  // namespace pa

using namespace pa;

extern "C" {

pa_status paged_kv_append(const pa_kv_cache_desc* cache, const void* k_new, const void* v_new,
                          const int32_t* seq_ids, const int32_t* positions, int32_t T, const int32_t* block_table,
                          int32_t batch, int32_t max_blocks, void* stream)
{
    pa_status st = check_cache(cache);
    if (st != PA_OK) return st;
    if (T < 0 || batch < 0 || max_blocks < 0) return PA_ERR_INVALID_ARG;
    if (T == 0) return PA_OK;
    if (!k_new || !v_new || !seq_ids || !positions || !block_table || batch == 0 || max_blocks == 0)
        return PA_ERR_INVALID_ARG;
    if (((uintptr_t)k_new | (uintptr_t)v_new) & 15) return PA_ERR_UNSUPPORTED;
    return launch_kv_append(cache, k_new, v_new, seq_ids, positions, T, block_table, max_blocks,
                            reinterpret_cast<hipStream_t>(stream));
}

pa_status paged_kv_gather(const pa_kv_cache_desc* cache, void* out_k, void* out_v, const int32_t* block_table,
                          const int32_t* seq_lens, const int32_t* cu_seq_lens, int32_t batch, int32_t max_blocks,
                          int32_t max_seq_len, void* stream)
{
    pa_status st = check_cache(cache);
    if (st != PA_OK) return st;
    if (batch < 0 || max_blocks < 0 || max_seq_len < 0) return PA_ERR_INVALID_ARG;
    if (batch == 0 || max_seq_len == 0) return PA_OK;
    if (!out_k || !out_v || !block_table || !seq_lens || !cu_seq_lens) return PA_ERR_INVALID_ARG;
    if ((int64_t)max_blocks * cache->page_size < max_seq_len) return PA_ERR_INVALID_ARG;
    if (((uintptr_t)out_k | (uintptr_t)out_v) & 15) return PA_ERR_UNSUPPORTED;
    return launch_kv_gather(cache, out_k, out_v, block_table, seq_lens, cu_seq_lens, batch, max_blocks, max_seq_len,
                            reinterpret_cast<hipStream_t>(stream));
}

pa_status pa_debug_check(const pa_kv_cache_desc* cache, const int32_t* block_table, const int32_t* seq_lens,
                         int32_t batch, int32_t max_blocks, const int32_t* seq_ids, const int32_t* positions, int32_t T,
                         void* scratch, int64_t* counts, void* stream)
{
    pa_status st = check_cache(cache);
    if (st != PA_OK) return st;
    if (batch < 0 || max_blocks < 0 || T < 0 || !counts || !scratch) return PA_ERR_INVALID_ARG;
    if (((uintptr_t)scratch & 7) || (batch > 0 && (!block_table || !seq_lens)) || (T > 0 && (!seq_ids || !positions)))
        return PA_ERR_INVALID_ARG;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    st = launch_debug_check(cache, block_table, seq_lens, batch, max_blocks, seq_ids, positions, T, scratch, s);
    if (st != PA_OK) return st;
    unsigned long long host[4] = {0, 0, 0, 0};
    if (hipMemcpyAsync(host, scratch, sizeof(host), hipMemcpyDeviceToHost, s) != hipSuccess) return PA_ERR_HIP;
    if (hipStreamSynchronize(s) != hipSuccess) return PA_ERR_HIP;
    for (int i = 0; i < 3; ++i) counts[i] = (int64_t)host[i];
    return PA_OK;
}

size_t paged_attention_workspace_bytes(int32_t batch, int32_t num_q_heads, int32_t head_dim, int32_t total_q,
                                       int32_t max_seq_len)
{
    if (batch <= 0 || num_q_heads <= 0 || head_dim <= 0 || total_q <= 0) return 256;
    if (total_q <= batch) {
        // decode: partials of the portable kernel's chunks, or of the tile stream's workgroups
        const int32_t ns = nsplit_bound(max_seq_len);
        const size_t chunked = part_o_bytes(batch, num_q_heads, head_dim, ns) + part_lse_bytes(batch, num_q_heads, ns);
        const size_t stream = stream_workspace_bytes(batch, num_q_heads, head_dim,
                                                     stream_wgs_bound(batch, num_q_heads, max_seq_len));
        const size_t split = short_split_workspace_bytes(batch, num_q_heads, head_dim);
        const size_t need = chunked > stream ? chunked : stream;
        return need > split ? need : split;
    }
    // prefill: partials of the context split, when the sizes make it split, and of the few-query route
    const int32_t np = prefill_nsplit_bound(batch, num_q_heads, total_q, max_seq_len);
    const size_t split = np > 1 ? part_o_bytes(total_q, num_q_heads, head_dim, np) + part_lse_bytes(total_q, num_q_heads, np)
                                : 0;
    return split + small_route_workspace_bytes(batch, num_q_heads, head_dim);
}

pa_status paged_attention_decode(const pa_kv_cache_desc* cache, const void* q, void* out, float* lse,
                                 const int32_t* block_table, const int32_t* seq_lens, int32_t batch,
                                 int32_t num_q_heads, int32_t max_blocks, int32_t max_seq_len, float scale,
                                 void* workspace, size_t workspace_bytes, void* stream)
{
    return run_attention(cache, q, out, lse, nullptr, batch, 1, block_table, seq_lens, batch, num_q_heads, max_blocks,
                         max_seq_len, scale, 0, nullptr, Workspace{workspace, workspace_bytes, true}, stream, true);
}

pa_status paged_attention_decode_mod(const pa_kv_cache_desc* cache, const void* q, void* out, float* lse,
                                     const int32_t* block_table, const int32_t* seq_lens, int32_t batch,
                                     int32_t num_q_heads, int32_t max_blocks, int32_t max_seq_len, float scale,
                                     const pa_attn_mods* mods, void* workspace, size_t workspace_bytes, void* stream)
{
    return run_attention(cache, q, out, lse, nullptr, batch, 1, block_table, seq_lens, batch, num_q_heads, max_blocks,
                         max_seq_len, scale, 0, mods, Workspace{workspace, workspace_bytes, true}, stream, true);
}

pa_status paged_attention_decode_static(const pa_kv_cache_desc* cache, const void* q, void* out, float* lse,
                                        const int32_t* block_table, const int32_t* seq_lens, int32_t batch,
                                        int32_t num_q_heads, int32_t max_blocks, int32_t max_seq_len, float scale,
                                        void* stream)
{
    void* ptr = nullptr;
    if (batch > 0) {
        const pa_status st = static_scratch(&ptr);
        if (st != PA_OK) return st;
    }
    const pa_status st = run_attention(cache, q, out, lse, nullptr, batch, 1, block_table, seq_lens, batch, num_q_heads,
                                       max_blocks, max_seq_len, scale, 0, nullptr,
                                       Workspace{ptr, kStaticScratchBytes, false}, stream, true);
    return st == PA_ERR_WORKSPACE_TOO_SMALL ? PA_ERR_SCRATCH_LIMIT : st;
}

pa_status paged_decode_step(const pa_kv_cache_desc* cache, const void* k_new, const void* v_new, const void* q,
                            void* out, float* lse, const int32_t* block_table, const int32_t* seq_lens, int32_t batch,
                            int32_t num_q_heads, int32_t max_blocks, int32_t max_seq_len, float scale,
                            const pa_attn_mods* mods, void* workspace, size_t workspace_bytes, void* stream)
{
    if (batch > 0 && (!k_new || !v_new)) return PA_ERR_INVALID_ARG;
    if (((uintptr_t)k_new | (uintptr_t)v_new) & 15) return PA_ERR_UNSUPPORTED;
    return run_attention(cache, q, out, lse, nullptr, batch, 1, block_table, seq_lens, batch, num_q_heads, max_blocks,
                         max_seq_len, scale, 0, mods, Workspace{workspace, workspace_bytes, true}, stream, true, k_new, v_new);
}

pa_status paged_attention_prefill_mod(const pa_kv_cache_desc* cache, const void* q, void* out, float* lse,
                                      const int32_t* cu_q_lens, int32_t total_q, int32_t max_q_len,
                                      const int32_t* block_table, const int32_t* seq_lens, int32_t batch,
                                      int32_t num_q_heads, int32_t max_blocks, int32_t max_seq_len, float scale,
                                      int32_t causal, const pa_attn_mods* mods, void* workspace,
                                      size_t workspace_bytes, void* stream)
{
    return run_attention(cache, q, out, lse, cu_q_lens, total_q, max_q_len, block_table, seq_lens, batch, num_q_heads,
                         max_blocks, max_seq_len, scale, causal, mods, Workspace{workspace, workspace_bytes, true}, stream, false);
}

pa_status paged_attention_prefill(const pa_kv_cache_desc* cache, const void* q, void* out, float* lse,
                                  const int32_t* cu_q_lens, int32_t total_q, int32_t max_q_len,
                                  const int32_t* block_table, const int32_t* seq_lens, int32_t batch,
                                  int32_t num_q_heads, int32_t max_blocks, int32_t max_seq_len, float scale,
                                  int32_t causal, void* workspace, size_t workspace_bytes, void* stream)
{
    return run_attention(cache, q, out, lse, cu_q_lens, total_q, max_q_len, block_table, seq_lens, batch, num_q_heads,
                         max_blocks, max_seq_len, scale, causal, nullptr, Workspace{workspace, workspace_bytes, true}, stream, false);
}

const char* pa_status_string(pa_status status)
{
    switch (status) {
        case PA_OK: return "ok";
        case PA_ERR_INVALID_ARG: return "invalid argument";
        case PA_ERR_UNSUPPORTED: return "unsupported dtype, shape or alignment";
        case PA_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
        case PA_ERR_HIP: return "HIP call failed";
        case PA_ERR_OUT_OF_PAGES: return "page pool exhausted";
        case PA_ERR_SCRATCH_LIMIT: return "the call's split-KV partials exceed the 16 MiB static scratch array";
    }
    return "unknown status";
}

pa_status pa_set_option(const char* name, int64_t value)
{
    if (!name) return PA_ERR_INVALID_ARG;
    if (!strcmp(name, "decode_chunk_tokens")) {
        if (value < 0 || value > (1 << 24)) return PA_ERR_INVALID_ARG;
        g_opt.decode_chunk_tokens = value;
        return PA_OK;
    }
    if (!strcmp(name, "decode_workgroups")) {
        if (value < 0 || value > kMaxDecodeWGs) return PA_ERR_INVALID_ARG;
        g_opt.decode_workgroups = value;
        return PA_OK;
    }
    if (!strcmp(name, "prefill_chunk_tokens")) {
        if (value < 0 || value > (1 << 24)) return PA_ERR_INVALID_ARG;
        g_opt.prefill_chunk_tokens = value;
        return PA_OK;
    }
    if (!strcmp(name, "no_small_q_route")) {
        if (value != 0 && value != 1) return PA_ERR_INVALID_ARG;
        g_opt.no_small_q_route = value;
        return PA_OK;
    }
    if (!strcmp(name, "step_append_kernel")) {
        if (value != 0 && value != 1) return PA_ERR_INVALID_ARG;
        g_opt.step_append_kernel = value;
        return PA_OK;
    }
    if (!strcmp(name, "decode_short")) {
        if (value < -1 || value > 1) return PA_ERR_INVALID_ARG;
        g_opt.decode_short = value;
        return PA_OK;
    }
    if (!strcmp(name, "decode_short_splits")) {
        if (value < 0 || value > kShortMaxSplit) return PA_ERR_INVALID_ARG;
        g_opt.decode_short_splits = value;
        return PA_OK;
    }
    if (!strcmp(name, "force_generic")) {
        if (value != 0 && value != 1) return PA_ERR_INVALID_ARG;
        g_opt.force_generic = value;
        return PA_OK;
    }
    return PA_ERR_INVALID_ARG;
}

pa_status pa_stream_read(const void* a, const void* b, size_t bytes_each, void* sink, void* stream)
{
    if (!a || !b || !sink || (((uintptr_t)a | (uintptr_t)b | (uintptr_t)sink) & 15)) return PA_ERR_INVALID_ARG;
    return launch_stream_read(a, b, bytes_each, sink, reinterpret_cast<hipStream_t>(stream));
}

pa_status pa_profile_enable(int32_t on)
{
    std::lock_guard<std::mutex> lock(g_profile_mutex);
    g_profile_on = on != 0;
    return PA_OK;
}

pa_status pa_profile_reset(void)
{
    std::lock_guard<std::mutex> lock(g_profile_mutex);
    for (auto& r : g_records) {
        (void)hipEventSynchronize(r.stop);
        g_spare_events.push_back(r.start);
        g_spare_events.push_back(r.stop);
    }
    g_records.clear();
    return PA_OK;
}

pa_status pa_profile_read(const char* kernel_prefix, int32_t* launches, double* total_ms)
{
    if (!kernel_prefix || !launches || !total_ms) return PA_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lock(g_profile_mutex);
    const size_t n = strlen(kernel_prefix);
    int32_t count = 0;
    double sum = 0.0;
    for (auto& r : g_records) {
        if (r.kernel.compare(0, n, kernel_prefix) != 0) continue;
        if (hipEventSynchronize(r.stop) != hipSuccess) return PA_ERR_HIP;
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, r.start, r.stop) != hipSuccess) return PA_ERR_HIP;
        sum += ms;
        ++count;
    }
    *launches = count;
    *total_ms = sum;
    return PA_OK;
}

}  // extern "C"
