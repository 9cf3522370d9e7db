// Host tier (paper Sec. V-A, V-C: all clusters are offloaded to CPU memory and
// fetched on demand as retrieval units; Sec. VII-B: transfers overlap compute).
//
// Pinned host memory holds, per unit, a pool of slabs of `SF` frame pages.  A
// cluster owns a chain of slabs, so its pages are contiguous in runs of SF
// ([SF K pages][SF V pages]) and a fetch streams a few large contiguous regions.  The GPU side keeps, per unit, a cache of slab-sized blocks with
// least-recently-used replacement at cluster granularity; the attention kernels
// read cache slots through the same page list they use in the HBM tier.
//
// All bookkeeping (slab chains, cache directory, LRU) is plain host code; the
// data moves by device stores into pinned memory (ingest, k_offload) and by
// device loads from pinned memory (fetch, k_fetch).
#include <algorithm>

#include "../../include/mosaic.h"
#include "host_tier.h"

namespace mosaic {

void HostTier::init(int U_, int C_, int SF_, int slabs_per_unit_, int cache_blocks_, int max_clusters_,
                    size_t kpage_, size_t vpage_) {
    U = U_; C = C_; SF = SF_; slabs_per_unit = slabs_per_unit_; cache_blocks = cache_blocks_;
    max_clusters = max_clusters_; kpage = kpage_; vpage = vpage_;
    units.assign(U, Unit());
    reset();
}

void HostTier::reset() {
    for (Unit &un : units) {
        un.slabs.assign(C, {});
        un.frames.assign(C, {});
        un.n.assign(C, 0);
        un.next_slab = 0;
        un.cache.assign(C, Entry());
        un.free_blocks.clear();
        for (int b = cache_blocks - 1; b >= 0; --b) un.free_blocks.push_back(b);
        un.n_cached = 0;
    }
    clock = 0;
}

// Frame f of unit u joins cluster c; returns the host page (within the unit's
// pool) it must be stored at, or -1 if the pool is exhausted.
int HostTier::append(int u, int f, int c) {
    Unit &un = units[u];
    const int slot = un.n[c] % SF;
    if (slot == 0) {
        if (un.next_slab >= slabs_per_unit) return -1;
        un.slabs[c].push_back(un.next_slab++);
    }
    un.n[c] += 1;
    un.frames[c].push_back(f);
    return un.slabs[c].back() * SF + slot;
}

// (With `prefetch` the ids are a prediction for a coming layer, see mosaic_prefetch: the same
// cache work, counted apart.)
// Make clusters ids[0..n_ids) of unit u resident: decide what must move (LRU at
// cluster granularity), append the moves as (host page, cache page) pairs to
// `moves`, and append the cache pages of the selection, in gather order, to
// `pages`.  The data itself is moved afterwards by ONE fetch kernel per retrieve
// that reads the pinned slabs directly over PCIe (measured at the rate of a
// large DMA copy, without a per-copy API cost).  Returns MOSAIC_OK or
// MOSAIC_ECAPACITY.
int HostTier::fetch(int u, const int *ids, int n_ids, std::vector<int> &moves, std::vector<int> &pages,
                    bool prefetch) {
    Unit &un = units[u];
    std::vector<char> pinned(C, 0);
    for (int i = 0; i < n_ids; ++i) pinned[ids[i]] = 1;
    for (int i = 0; i < n_ids; ++i) {
        const int c = ids[i];
        Entry &e = un.cache[c];
        const int have = e.present ? e.pages : 0;
        const int want = un.n[c];
        const bool complete = e.present && have == want;
        if (prefetch) {                      // a guess for a coming layer: not a retrieval's hit or miss
            if (!complete) { pf_fetched += 1; e.by_prefetch = true; }
        } else {
            if (complete) { hits += 1; if (e.by_prefetch) pf_useful += 1; } else misses += 1;
            e.by_prefetch = false;
        }
        const int need_blocks = (want + SF - 1) / SF;
        // room: enough free blocks, and not more resident clusters than allowed
        while ((int)un.free_blocks.size() < need_blocks - (int)e.blocks.size() ||
               (!e.present && un.n_cached >= max_clusters)) {
            int victim = -1;
            for (int j = 0; j < C; ++j)
                if (un.cache[j].present && !pinned[j] &&
                    (victim < 0 || un.cache[j].stamp < un.cache[victim].stamp)) victim = j;
            if (victim < 0) {
                fail_need = need_blocks; fail_free = (int)un.free_blocks.size(); fail_cached = un.n_cached;
                fail_sel_pages = 0;
                for (int q = 0; q < n_ids; ++q) fail_sel_pages += un.n[ids[q]];
                return MOSAIC_ECAPACITY;
            }
            Entry &v = un.cache[victim];
            for (int b : v.blocks) un.free_blocks.push_back(b);
            v.blocks.clear(); v.pages = 0; v.present = false; v.by_prefetch = false;
            un.n_cached -= 1;
            evictions += 1;
        }
        if (!e.present) { e.present = true; un.n_cached += 1; }
        while ((int)e.blocks.size() < need_blocks) {
            e.blocks.push_back(un.free_blocks.back());
            un.free_blocks.pop_back();
        }
        for (int p = have; p < want; ++p) {          // pages still in host memory only
            moves.push_back(un.slabs[c][p / SF] * SF + p % SF);
            moves.push_back(e.blocks[p / SF] * SF + p % SF);
        }
        h2d_bytes += (long long)(want - have) * (kpage + vpage);
        e.pages = want;
        e.stamp = ++clock;
        for (int p = 0; p < want; ++p) pages.push_back(e.blocks[p / SF] * SF + p % SF);
    }
    return MOSAIC_OK;
}

} // namespace mosaic
