// Host-side page pool for the paged KV cache of one layer, with page recycling for
// sliding-window layers.
//
// A window layer attends to the most recent W positions only, so its KV footprint per sequence
// is bounded by W instead of growing with the context (paper Section 2, "Window attention for
// long-context inference": the per-layer KV-cache footprint becomes proportional to W).  The pool
// makes that bound real: when a sequence grows, pages that lie entirely before its window are
// handed back to the free list, so a window layer needs at most pz_window_pages() physical pages
// per sequence however long the context becomes.  The attention kernel never uses block-table
// entries of pages that hold no attended position, so the stale entries of recycled pages are
// harmless.
//
// Pure host code (no HIP calls): the caller owns the device block table and mirrors the updates
// that pz_page_pool_drain_updates() hands out.
#include <stdint.h>

#include <new>
#include <vector>

#include "pz.h"

struct pz_page_pool {
    int32_t num_pages, page_size, max_seqs, max_pages_per_seq, window;
    std::vector<int32_t> free_list;                    // stack of free physical pages
    std::vector<int32_t> table;                        // [max_seqs][max_pages_per_seq], -1 = none
    std::vector<int32_t> seq_len;                      // [max_seqs]
    std::vector<int32_t> first_page;                   // [max_seqs]: first logical page still held
    std::vector<int32_t> upd_index, upd_value;         // pending block-table updates (flat index, value)
};

namespace {

// Records a block-table change.  The caller has made room in the update lists (reserve_updates), so
// nothing here allocates and a half-recorded change cannot happen.
void set_entry(pz_page_pool *p, int32_t seq, int32_t logical_page, int32_t value) {
    const int32_t idx = seq * p->max_pages_per_seq + logical_page;
    p->table[idx] = value;
    p->upd_index.push_back(idx);
    p->upd_value.push_back(value);
}

// Room for n more pending updates in both lists; false when host memory is exhausted (nothing changed).
bool reserve_updates(pz_page_pool *p, size_t n) {
    try {
        p->upd_index.reserve(p->upd_index.size() + n);
        p->upd_value.reserve(p->upd_value.size() + n);
    } catch (...) {
        return false;
    }
    return true;
}

}  // namespace

extern "C" {

int32_t pz_window_pages(int32_t window, int32_t page_size) {
    if (window <= 0 || page_size <= 0) return 0;
    // positions [L - W, L) touch pages floor((L-W)/P) .. floor((L-1)/P): at most this many
    return (window + page_size - 2) / page_size + 1;
}

pz_page_pool *pz_page_pool_create(int32_t num_pages, int32_t page_size, int32_t max_seqs,
                                  int32_t max_pages_per_seq, int32_t window) {
    if (num_pages <= 0 || page_size <= 0 || max_seqs <= 0 || max_pages_per_seq <= 0 || window < 0) return nullptr;
    if ((int64_t)max_seqs * max_pages_per_seq > 0x7fffffffLL) return nullptr;     // flat table indices are 32-bit
    pz_page_pool *p = new (std::nothrow) pz_page_pool;
    if (p == nullptr) return nullptr;
    p->num_pages = num_pages;
    p->page_size = page_size;
    p->max_seqs = max_seqs;
    p->max_pages_per_seq = max_pages_per_seq;
    p->window = window;
    try {
        // the free list never holds more than num_pages entries: sized once, push_back never reallocates
        p->free_list.reserve(num_pages);
        p->free_list.resize(num_pages);
        for (int32_t i = 0; i < num_pages; ++i) p->free_list[i] = num_pages - 1 - i;   // page 0 is handed out first
        p->table.assign((size_t)max_seqs * max_pages_per_seq, -1);
        p->seq_len.assign(max_seqs, 0);
        p->first_page.assign(max_seqs, 0);
    } catch (...) {                                    // out of host memory: no exception crosses the C boundary
        delete p;
        return nullptr;
    }
    return p;
}

void pz_page_pool_destroy(pz_page_pool *pool) { delete pool; }

int64_t pz_page_pool_append(pz_page_pool *p, int32_t seq) {
    if (p == nullptr) return PZ_ERR_NULL;
    if (seq < 0 || seq >= p->max_seqs) return PZ_ERR_SHAPE;
    const int32_t pos = p->seq_len[seq];
    const int32_t lp = pos / p->page_size;
    if (lp >= p->max_pages_per_seq) return PZ_ERR_SHAPE;
    const int32_t new_len = pos + 1;
    const bool opens_page = pos % p->page_size == 0;
    // pages entirely before the window of the grown sequence go back to the pool first
    const int32_t keep_from = (p->window > 0 && new_len > p->window) ? (new_len - p->window) / p->page_size : 0;
    const int32_t n_drop = keep_from > p->first_page[seq] ? keep_from - p->first_page[seq] : 0;
    // every failure is found before anything changes: no page to open (the pages this very step hands
    // back count), or no host memory for the update records
    if (opens_page && p->free_list.empty() && n_drop == 0) return PZ_ERR_WORKSPACE;
    if (!reserve_updates(p, (size_t)n_drop + 1)) return PZ_ERR_WORKSPACE;
    while (p->first_page[seq] < keep_from) {
        const int32_t old = p->first_page[seq]++;
        const int32_t phys = p->table[(size_t)seq * p->max_pages_per_seq + old];
        if (phys >= 0) {
            p->free_list.push_back(phys);
            set_entry(p, seq, old, -1);
        }
    }
    if (opens_page) {                                  // the new position opens a page
        if (p->free_list.empty()) return PZ_ERR_WORKSPACE;         // not reached: a held page was just handed back
        const int32_t phys = p->free_list.back();
        p->free_list.pop_back();
        set_entry(p, seq, lp, phys);
    }
    p->seq_len[seq] = new_len;
    const int32_t phys = p->table[(size_t)seq * p->max_pages_per_seq + lp];
    return (int64_t)phys * p->page_size + pos % p->page_size;
}

pz_status pz_page_pool_release(pz_page_pool *p, int32_t seq) {
    if (p == nullptr) return PZ_ERR_NULL;
    if (seq < 0 || seq >= p->max_seqs) return PZ_ERR_SHAPE;
    const int32_t end = (p->seq_len[seq] + p->page_size - 1) / p->page_size;
    if (end > p->first_page[seq] && !reserve_updates(p, (size_t)(end - p->first_page[seq]))) return PZ_ERR_WORKSPACE;
    for (int32_t lp = p->first_page[seq]; lp < end; ++lp) {
        const int32_t phys = p->table[(size_t)seq * p->max_pages_per_seq + lp];
        if (phys >= 0) {
            p->free_list.push_back(phys);
            set_entry(p, seq, lp, -1);
        }
    }
    p->seq_len[seq] = 0;
    p->first_page[seq] = 0;
    return PZ_OK;
}

int32_t pz_page_pool_seq_len(const pz_page_pool *p, int32_t seq) {
    return (p == nullptr || seq < 0 || seq >= p->max_seqs) ? -1 : p->seq_len[seq];
}

int32_t pz_page_pool_free_pages(const pz_page_pool *p) { return p == nullptr ? -1 : (int32_t)p->free_list.size(); }

const int32_t *pz_page_pool_block_table(const pz_page_pool *p) { return p == nullptr ? nullptr : p->table.data(); }

int32_t pz_page_pool_drain_updates(pz_page_pool *p, int32_t *index_out, int32_t *value_out, int32_t capacity) {
    if (p == nullptr || capacity < 0 || (capacity > 0 && (index_out == nullptr || value_out == nullptr))) return -1;
    const int32_t pending = (int32_t)p->upd_index.size();
    const int32_t n = pending < capacity ? pending : capacity;
    for (int32_t i = 0; i < n; ++i) {
        index_out[i] = p->upd_index[i];
        value_out[i] = p->upd_value[i];
    }
    p->upd_index.erase(p->upd_index.begin(), p->upd_index.begin() + n);
    p->upd_value.erase(p->upd_value.begin(), p->upd_value.begin() + n);
    return n;
}

int32_t pz_page_pool_pending_updates(const pz_page_pool *p) { return p == nullptr ? -1 : (int32_t)p->upd_index.size(); }

}  // extern "C"
