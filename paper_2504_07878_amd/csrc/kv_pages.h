// Host bookkeeping of the paged KV cache: one page table row per slot, a reference count per page, a free list.
// Plain C++, no device calls: the scheduler asks it what a write would cost, lets it update the tables, and then makes the
// page copies and table uploads it reports. Pages are shared between slots after a fork and copied before the first
// write into a shared page (positions already cached are never rewritten, so full shared pages stay shared for good).
#pragma once
#include <stddef.h>
#include <unordered_map>
#include <vector>

namespace tr {

struct KvPages {
    struct Copy { int from, to; };   // page `from` must be copied to page `to` on the device before the next kernel writes

    int page = 0, maxp = 0, pool = 0;
    std::vector<int> table;    // [slots][maxp]: page of positions i*page .. (i+1)*page-1; entries past npages are stale
    std::vector<int> npages;   // pages a slot refers to
    std::vector<int> refc;     // slots referring to a page
    std::vector<int> free_;    // stack of unused pages

    void init(int slots, int page_len, int pages_per_slot, int pool_pages)
    {
        page = page_len; maxp = pages_per_slot; pool = pool_pages;
        table.assign((size_t)slots * maxp, 0);
        npages.assign((size_t)slots, 0);
        refc.assign((size_t)pool, 0);
        free_.clear();
        for (int p = pool - 1; p >= 0; --p) free_.push_back(p);   // page 0 is handed out first
    }
    int pages_for(int len) const { return (len + page - 1) / page; }
    int free_count() const { return (int)free_.size(); }
    const int *row(int slot) const { return table.data() + (size_t)slot * maxp; }

    // Pages the writes [old_len, new_len) of the listed slots would take from the free list: new pages past what a slot
    // has, and private copies of pages it shares. A page shared only among the listed slots is counted for all but the
    // last of them (the last one keeps the original).
    int demand(int n, const int *slots, const int *old_len, const int *new_len) const
    {
        std::unordered_map<int, int> left;   // references still on a shared page while the listed slots take their copies
        int need = 0;
        for (int i = 0; i < n; ++i) {
            if (new_len[i] <= old_len[i]) continue;
            const int s = slots[i], first = old_len[i] / page, last = (new_len[i] - 1) / page;
            for (int k = first; k <= last; ++k) {
                if (k >= npages[(size_t)s]) { ++need; continue; }
                const int pg = table[(size_t)s * maxp + k];
                auto it = left.find(pg);
                int &r = it == left.end() ? (left[pg] = refc[(size_t)pg]) : it->second;
                if (r > 1) { ++need; --r; }
            }
        }
        return need;
    }

    // Performs the write's bookkeeping for one slot (the caller has checked demand() against free_count()); copies to make
    // are appended. Returns true if the slot's table row changed.
    bool grow(int s, int old_len, int new_len, std::vector<Copy> &copies)
    {
        if (new_len <= old_len) return false;
        bool changed = false;
        const int first = old_len / page, last = (new_len - 1) / page;
        for (int k = first; k <= last; ++k) {
            int &entry = table[(size_t)s * maxp + k];
            if (k >= npages[(size_t)s]) {
                entry = take();
                npages[(size_t)s] = k + 1;
                changed = true;
            } else if (refc[(size_t)entry] > 1) {
                const int fresh = take();
                copies.push_back(Copy{entry, fresh});
                refc[(size_t)entry] -= 1;
                entry = fresh;
                changed = true;
            }
        }
        return changed;
    }

    // gives back the pages that hold no position below new_len
    void shrink(int s, int new_len)
    {
        const int keep = pages_for(new_len);
        for (int k = keep; k < npages[(size_t)s]; ++k) drop(table[(size_t)s * maxp + k]);
        if (npages[(size_t)s] > keep) npages[(size_t)s] = keep;
    }

    // dst, emptied before, refers to the pages of src
    void share(int src, int dst)
    {
        for (int k = 0; k < npages[(size_t)src]; ++k) {
            const int pg = table[(size_t)src * maxp + k];
            table[(size_t)dst * maxp + k] = pg;
            refc[(size_t)pg] += 1;
        }
        npages[(size_t)dst] = npages[(size_t)src];
    }

private:
    int take()
    {
        const int pg = free_.back();
        free_.pop_back();
        refc[(size_t)pg] = 1;
        return pg;
    }
    void drop(int pg)
    {
        if (--refc[(size_t)pg] == 0) free_.push_back(pg);
    }
};

}  // namespace tr
