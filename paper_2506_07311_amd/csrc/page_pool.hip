// KV page manager (Algorithm 1 Reserve; Sec. III-B "Paged KV-Manager"): host bookkeeping of the physical pages.
//
// Free list = atomic bump pointer over never-used pages + tagged Treiber stack of recycled pages; both are
// lock-free, so one page is reserved or returned in O(1) without a lock.  Per-sequence state (its row of the block
// table and its block count) is owned by whoever drives that sequence; reference counts make pages shareable.
// The device-resident block table is kept current by copying the changed entries of a row on the caller's stream.
// The copy's source is a pinned staging ring that holds the values as they were when the call was made: the host
// mirror itself may change again (a release right after a reserve) before the stream reaches the copy.
#include <atomic>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "common.h"

struct pa_pool {
    int32_t num_pages = 0;
    int32_t page_size = 0;
    int32_t log2_page = 0;
    int32_t max_seqs = 0;
    int32_t max_blocks = 0;
    int32_t* device_table = nullptr;
    int32_t* host_table = nullptr;          // [max_seqs, max_blocks] host mirror
    std::vector<int32_t> num_blocks;        // per sequence
    // per sequence: entries [stale_lo, stale_hi) of the device row whose copy failed (PA_ERR_HIP); the next call that
    // changes the sequence's row copies them again from the mirror together with its own
    std::vector<int32_t> stale_lo, stale_hi;
    std::atomic<int32_t>* next = nullptr;   // free-stack links
    std::atomic<int32_t>* refs = nullptr;   // per page
    std::atomic<int32_t> fresh{0};          // bump pointer: pages [fresh, num_pages) were never handed out
    std::atomic<uint64_t> head{0};          // free stack: low 32 bits = page index + 1 (0 = empty), high 32 = tag
    std::atomic<int32_t> free_count{0};
    int32_t growth = PA_GROW_EXACT;

    // Staging ring for row updates (only with a device table): kQuarters segments of kQuarterInts entries; a
    // segment is reused only after the event recorded when it was left has completed.
    static constexpr int kQuarters = 4;
    static constexpr int32_t kQuarterInts = 1 << 16;
    int32_t* stage = nullptr;
    hipEvent_t stage_done[kQuarters] = {};
    bool stage_recorded[kQuarters] = {};
    int stage_quarter = 0;
    int32_t stage_pos = 0;
    std::mutex stage_mu;
};

namespace {

// O(1), lock-free: recycled pages first, then the bump pointer.  Returns -1 when the pool is exhausted.
int32_t pop_page(pa_pool* p)
{
    uint64_t h = p->head.load(std::memory_order_acquire);
    while ((uint32_t)h != 0) {
        const int32_t page = (int32_t)(uint32_t)h - 1;
        const uint64_t nh = ((h >> 32) + 1) << 32 | (uint32_t)(p->next[page].load(std::memory_order_relaxed) + 1);
        if (p->head.compare_exchange_weak(h, nh, std::memory_order_acq_rel, std::memory_order_acquire)) {
            p->free_count.fetch_sub(1, std::memory_order_relaxed);
            return page;
        }
    }
    int32_t f = p->fresh.load(std::memory_order_relaxed);
    while (f < p->num_pages) {
        if (p->fresh.compare_exchange_weak(f, f + 1, std::memory_order_relaxed)) {
            p->free_count.fetch_sub(1, std::memory_order_relaxed);
            return f;
        }
    }
    // the bump pointer is spent: a page may have been pushed meanwhile
    h = p->head.load(std::memory_order_acquire);
    while ((uint32_t)h != 0) {
        const int32_t page = (int32_t)(uint32_t)h - 1;
        const uint64_t nh = ((h >> 32) + 1) << 32 | (uint32_t)(p->next[page].load(std::memory_order_relaxed) + 1);
        if (p->head.compare_exchange_weak(h, nh, std::memory_order_acq_rel, std::memory_order_acquire)) {
            p->free_count.fetch_sub(1, std::memory_order_relaxed);
            return page;
        }
    }
    return -1;
}

void push_page(pa_pool* p, int32_t page)
{
    uint64_t h = p->head.load(std::memory_order_acquire);
    for (;;) {
        p->next[page].store((int32_t)(uint32_t)h - 1, std::memory_order_relaxed);
        const uint64_t nh = ((h >> 32) + 1) << 32 | (uint32_t)(page + 1);
        if (p->head.compare_exchange_weak(h, nh, std::memory_order_acq_rel, std::memory_order_acquire)) break;
    }
    p->free_count.fetch_add(1, std::memory_order_relaxed);
}

void unref_page(pa_pool* p, int32_t page)
{
    if (p->refs[page].fetch_sub(1, std::memory_order_acq_rel) == 1) push_page(p, page);
}

pa_status copy_row(pa_pool* p, int32_t seq, int32_t b0, int32_t b1, void* stream);

// Copy entries [b0, b1) of the sequence's row to the device table, together with entries an earlier call failed to
// deliver.  On PA_ERR_HIP the host mirror is ahead of the device row for the recorded range until a later call for
// the same sequence succeeds.
pa_status sync_row(pa_pool* p, int32_t seq, int32_t b0, int32_t b1, void* stream)
{
    if (!p->device_table) return PA_OK;
    if (p->stale_hi[seq] > p->stale_lo[seq]) {
        const bool own = b1 > b0;                            // the union of this call's entries and the stale ones
        b0 = own && b0 < p->stale_lo[seq] ? b0 : p->stale_lo[seq];
        b1 = own && b1 > p->stale_hi[seq] ? b1 : p->stale_hi[seq];
    }
    if (b1 <= b0) return PA_OK;
    const pa_status st = copy_row(p, seq, b0, b1, stream);
    if (st == PA_OK) {
        p->stale_lo[seq] = p->stale_hi[seq] = 0;
    } else {
        p->stale_lo[seq] = b0;
        p->stale_hi[seq] = b1;
    }
    return st;
}

pa_status copy_row(pa_pool* p, int32_t seq, int32_t b0, int32_t b1, void* stream)
{
    const size_t off = (size_t)seq * p->max_blocks + b0;
    const int32_t n = b1 - b0;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    if (n > pa_pool::kQuarterInts) {   // larger than a ring segment: copy from the mirror and wait for it
        if (hipMemcpyAsync(p->device_table + off, p->host_table + off, (size_t)n * sizeof(int32_t),
                           hipMemcpyHostToDevice, st) != hipSuccess)
            return PA_ERR_HIP;
        return hipStreamSynchronize(st) == hipSuccess ? PA_OK : PA_ERR_HIP;
    }
    std::lock_guard<std::mutex> lock(p->stage_mu);
    if (p->stage_pos + n > pa_pool::kQuarterInts) {
        if (hipEventRecord(p->stage_done[p->stage_quarter], st) != hipSuccess) return PA_ERR_HIP;
        p->stage_recorded[p->stage_quarter] = true;
        p->stage_quarter = (p->stage_quarter + 1) % pa_pool::kQuarters;
        p->stage_pos = 0;
        if (p->stage_recorded[p->stage_quarter]) {
            if (hipEventSynchronize(p->stage_done[p->stage_quarter]) != hipSuccess) return PA_ERR_HIP;
            p->stage_recorded[p->stage_quarter] = false;
        }
    }
    int32_t* src = p->stage + (size_t)p->stage_quarter * pa_pool::kQuarterInts + p->stage_pos;
    std::memcpy(src, p->host_table + off, (size_t)n * sizeof(int32_t));
    p->stage_pos += n;
    return hipMemcpyAsync(p->device_table + off, src, (size_t)n * sizeof(int32_t), hipMemcpyHostToDevice, st) ==
                   hipSuccess
               ? PA_OK
               : PA_ERR_HIP;
}

bool seq_ok(const pa_pool* p, int32_t seq) { return p && seq >= 0 && seq < p->max_seqs; }

}  // namespace

extern "C" {

pa_status pa_pool_create(pa_pool** out, int32_t num_pages, int32_t page_size, int32_t max_seqs, int32_t max_blocks,
                         int32_t* device_table)
{
    if (!out || num_pages <= 0 || max_seqs <= 0 || max_blocks <= 0) return PA_ERR_INVALID_ARG;
    if (page_size <= 0 || (page_size & (page_size - 1)) != 0) return PA_ERR_INVALID_ARG;   // Algorithm 1: power of two
    pa_pool* p = new pa_pool;
    p->num_pages = num_pages;
    p->page_size = page_size;
    while ((1 << p->log2_page) < page_size) ++p->log2_page;
    p->max_seqs = max_seqs;
    p->max_blocks = max_blocks;
    p->device_table = device_table;
    const size_t entries = (size_t)max_seqs * max_blocks;
    p->host_table = new int32_t[entries];
    for (size_t i = 0; i < entries; ++i) p->host_table[i] = -1;
    p->num_blocks.assign(max_seqs, 0);
    p->stale_lo.assign(max_seqs, 0);
    p->stale_hi.assign(max_seqs, 0);
    p->next = new std::atomic<int32_t>[num_pages];
    p->refs = new std::atomic<int32_t>[num_pages];
    for (int32_t i = 0; i < num_pages; ++i) {
        p->next[i].store(-1, std::memory_order_relaxed);
        p->refs[i].store(0, std::memory_order_relaxed);
    }
    p->free_count.store(num_pages);
    if (device_table) {
        bool ok = hipHostMalloc(reinterpret_cast<void**>(&p->stage),
                                (size_t)pa_pool::kQuarters * pa_pool::kQuarterInts * sizeof(int32_t),
                                hipHostMallocDefault) == hipSuccess;
        for (int q = 0; ok && q < pa_pool::kQuarters; ++q)
            ok = hipEventCreateWithFlags(&p->stage_done[q], hipEventDisableTiming) == hipSuccess;
        ok = ok && hipMemcpy(device_table, p->host_table, entries * sizeof(int32_t), hipMemcpyHostToDevice) == hipSuccess;
        if (!ok) {
            pa_pool_destroy(p);
            return PA_ERR_HIP;
        }
    }
    *out = p;
    return PA_OK;
}

pa_status pa_pool_set_growth(pa_pool* p, int32_t policy)
{
    if (!p || (policy != PA_GROW_EXACT && policy != PA_GROW_POW2)) return PA_ERR_INVALID_ARG;
    p->growth = policy;
    return PA_OK;
}

pa_status pa_pool_destroy(pa_pool* p)
{
    if (!p) return PA_ERR_INVALID_ARG;
    for (int q = 0; q < pa_pool::kQuarters; ++q)
        if (p->stage_done[q]) {
            if (p->stage_recorded[q]) (void)hipEventSynchronize(p->stage_done[q]);
            (void)hipEventDestroy(p->stage_done[q]);
        }
    if (p->stage) {
        (void)hipDeviceSynchronize();   // row copies still in flight read the ring
        (void)hipHostFree(p->stage);
    }
    delete[] p->host_table;
    delete[] p->next;
    delete[] p->refs;
    delete p;
    return PA_OK;
}

pa_status pa_pool_reserve(pa_pool* p, int32_t seq, int32_t len, void* stream)
{
    if (!seq_ok(p, seq) || len < 0) return PA_ERR_INVALID_ARG;
    const int64_t n = ((int64_t)len + p->page_size - 1) >> p->log2_page;   // n = ceil(len / P)
    if (n > p->max_blocks) return PA_ERR_INVALID_ARG;
    const int32_t have = p->num_blocks[seq];
    if (n <= have) return PA_OK;
    int64_t want = n;   // PA_GROW_POW2: capacity in blocks rounded up to a power of two, as far as pages last
    if (p->growth == PA_GROW_POW2) {
        want = 1;
        while (want < n) want <<= 1;
        if (want > p->max_blocks) want = p->max_blocks;
    }
    int32_t* row = p->host_table + (size_t)seq * p->max_blocks;
    int32_t got = have;
    for (; got < (int32_t)want; ++got) {
        const int32_t page = pop_page(p);
        if (page < 0) break;
        p->refs[page].store(1, std::memory_order_release);
        row[got] = page;
    }
    if (got < (int32_t)n) {   // give back what this call took: the sequence stays as it was
        for (int32_t u = have; u < got; ++u) {
            unref_page(p, row[u]);
            row[u] = -1;
        }
        return PA_ERR_OUT_OF_PAGES;
    }
    p->num_blocks[seq] = got;
    return sync_row(p, seq, have, got, stream);
}

pa_status pa_pool_release(pa_pool* p, int32_t seq, void* stream)
{
    if (!seq_ok(p, seq)) return PA_ERR_INVALID_ARG;
    const int32_t have = p->num_blocks[seq];
    int32_t* row = p->host_table + (size_t)seq * p->max_blocks;
    for (int32_t b = 0; b < have; ++b) {
        unref_page(p, row[b]);
        row[b] = -1;
    }
    p->num_blocks[seq] = 0;
    return sync_row(p, seq, 0, have, stream);
}

pa_status pa_pool_share_prefix(pa_pool* p, int32_t dst, int32_t src, int32_t prefix_tokens, void* stream)
{
    if (!seq_ok(p, dst) || !seq_ok(p, src) || dst == src || prefix_tokens < 0) return PA_ERR_INVALID_ARG;
    if (p->num_blocks[dst] != 0) return PA_ERR_INVALID_ARG;
    const int32_t nb = prefix_tokens >> p->log2_page;    // whole pages only
    if (nb > p->num_blocks[src]) return PA_ERR_INVALID_ARG;
    int32_t* drow = p->host_table + (size_t)dst * p->max_blocks;
    const int32_t* srow = p->host_table + (size_t)src * p->max_blocks;
    for (int32_t b = 0; b < nb; ++b) {
        p->refs[srow[b]].fetch_add(1, std::memory_order_acq_rel);
        drow[b] = srow[b];
    }
    p->num_blocks[dst] = nb;
    return sync_row(p, dst, 0, nb, stream);
}

pa_status pa_pool_make_writable(pa_pool* p, const pa_kv_cache_desc* cache, int32_t seq, int32_t position, void* stream)
{
    if (!seq_ok(p, seq) || position < 0) return PA_ERR_INVALID_ARG;
    const pa_status desc = pa::check_cache(cache);           // dtype, strides, 16-byte alignment of the pools
    if (desc != PA_OK) return desc;
    if (cache->page_size != p->page_size || cache->num_pages < p->num_pages) return PA_ERR_INVALID_ARG;
    const int32_t b = position >> p->log2_page;
    if (b >= p->num_blocks[seq]) return PA_ERR_INVALID_ARG;
    int32_t* row = p->host_table + (size_t)seq * p->max_blocks;
    const int32_t old_page = row[b];
    if (p->refs[old_page].load(std::memory_order_acquire) <= 1) return PA_OK;   // already private
    const int32_t page = pop_page(p);
    if (page < 0) return PA_ERR_OUT_OF_PAGES;
    p->refs[page].store(1, std::memory_order_release);
    const pa_status st = pa::launch_kv_copy_page(cache, old_page, page, reinterpret_cast<hipStream_t>(stream));
    if (st != PA_OK) {
        unref_page(p, page);
        return st;
    }
    row[b] = page;
    unref_page(p, old_page);
    return sync_row(p, seq, b, b + 1, stream);
}

int32_t pa_pool_num_free(const pa_pool* p) { return p ? p->free_count.load(std::memory_order_relaxed) : -1; }

int32_t pa_pool_num_blocks(const pa_pool* p, int32_t seq) { return seq_ok(p, seq) ? p->num_blocks[seq] : -1; }

pa_status pa_pool_get_row(const pa_pool* p, int32_t seq, int32_t* host_row, int32_t capacity)
{
    if (!seq_ok(p, seq) || !host_row || capacity < p->num_blocks[seq]) return PA_ERR_INVALID_ARG;
    const int32_t* row = p->host_table + (size_t)seq * p->max_blocks;
    for (int32_t b = 0; b < capacity; ++b) host_row[b] = b < p->max_blocks ? row[b] : -1;
    return PA_OK;
}

int32_t pa_pool_refcount(const pa_pool* p, int32_t page)
{
    return (p && page >= 0 && page < p->num_pages) ? p->refs[page].load(std::memory_order_acquire) : -1;
}

}  // extern "C"
