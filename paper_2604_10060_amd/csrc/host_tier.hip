// Host tier (paper Sec. V-A, V-C: all clusters are offloaded to CPU memory and
// fetched on demand as retrieval units; Sec. VII-B: transfers overlap compute).
//
// Pinned host memory holds, per unit, a pool of slabs of `SF` frame pages
// ([SF K pages][SF V pages]).  A cluster appends its frames to a slab of its own and
// opens a new one when that is full, so a cluster's pages lie in runs of SF frames and
// a fetch streams a few large contiguous regions.  The GPU side keeps, per unit, a
// cache of page slots with least-recently-used replacement at cluster granularity
// (a cluster is fetched, counted and evicted as a whole; its slots need not be
// adjacent); the attention kernels read cache slots through the same page list they
// use in the HBM tier.
//
// The self-adaptive maintainer (Sec. VI) changes membership under the cache: a split hands
// part of a cluster's frames to a new id, a deferred split first parks states as singleton
// entries.  Pages never move for that: a frame keeps its host page and its cache slot, and
// the cache state is kept per frame (slot, time of last use, fetched-ahead mark); what the
// directory says about an entry -- resident, complete, time of last use -- is derived from
// its frames, so both halves of a split inherit the parent's residency and recency.
//
// All bookkeeping (frame lists, slab placement, cache directory, LRU) is plain host
// code over arrays sized at creation; the data moves by device stores into pinned
// memory (ingest, k_offload) and by device loads from pinned memory (fetch, k_fetch).
#include <algorithm>

#include "../../include/mosaic.h"
#include "host_tier.h"

namespace mosaic {

void HostTier::init(int U_, int C_, int n_entries, int F_, int SF_, int slabs_per_unit_, int cache_pages_,
                    int max_clusters_, int top_k_, size_t kpage_, size_t vpage_) {
    U = U_; C = C_; E = n_entries; F = F_; SF = SF_; slabs_per_unit = slabs_per_unit_; cache_pages = cache_pages_;
    max_clusters = max_clusters_; top_k = top_k_; kpage = kpage_; vpage = vpage_;
    units.assign(U, Unit());
    pinned.assign(E, 0);
    seen_splits.assign((size_t)U * 2, 0);
    seen_nbuf.assign(U, 0);
    for (Unit &un : units) {
        un.n.resize(E); un.head_f.resize(E); un.tail_f.resize(E);
        un.next_f.resize(F);
        un.open_slab.resize(C); un.open_fill.resize(C);
        un.host_page.resize(F);
        un.slot.resize(F); un.fstamp.resize(F); un.ahead.resize(F);
        un.free_slots.reserve(cache_pages);
        un.cached.resize(E); un.stamp.resize(E); un.by_prefetch.resize(E);
        un.last_ids.resize(std::max(top_k, 1));
        un.last_frames.resize(F);
    }
    reset();
}

void HostTier::reset() {
    for (Unit &un : units) {
        std::fill(un.n.begin(), un.n.end(), 0);
        std::fill(un.head_f.begin(), un.head_f.end(), -1);
        std::fill(un.tail_f.begin(), un.tail_f.end(), -1);
        std::fill(un.next_f.begin(), un.next_f.end(), -1);
        std::fill(un.open_slab.begin(), un.open_slab.end(), -1);
        std::fill(un.open_fill.begin(), un.open_fill.end(), 0);
        std::fill(un.host_page.begin(), un.host_page.end(), -1);
        std::fill(un.slot.begin(), un.slot.end(), -1);
        std::fill(un.fstamp.begin(), un.fstamp.end(), 0);
        std::fill(un.ahead.begin(), un.ahead.end(), 0);
        un.next_slab = 0;
        un.free_slots.clear();
        for (int s = cache_pages - 1; s >= 0; --s) un.free_slots.push_back(s);
        std::fill(un.cached.begin(), un.cached.end(), 0);
        std::fill(un.stamp.begin(), un.stamp.end(), 0);
        std::fill(un.by_prefetch.begin(), un.by_prefetch.end(), 0);
        un.n_cached = 0;
        un.n_last = 0;
        un.n_last_frames = 0;
        un.resident_dirty = true;
    }
    std::fill(seen_splits.begin(), seen_splits.end(), 0);
    std::fill(seen_nbuf.begin(), seen_nbuf.end(), 0);
    clock = 0;
}

// Host page for frame f of unit u, filed with cluster c (the cluster it was assigned to, or the
// owner on whose behalf it is buffered): the next free place of c's open slab.  Returns the page
// (within the unit's pool), or -1 if the pool is exhausted.
int HostTier::place(int u, int f, int c) {
    Unit &un = units[u];
    if (un.open_slab[c] < 0 || un.open_fill[c] == SF) {
        if (un.next_slab >= slabs_per_unit) return -1;
        un.open_slab[c] = un.next_slab++;
        un.open_fill[c] = 0;
    }
    const int hp = un.open_slab[c] * SF + un.open_fill[c]++;
    un.host_page[f] = hp;
    return hp;
}

// Frame f (larger than every frame the entry holds) joins entry e.
void HostTier::join(int u, int f, int e) {
    Unit &un = units[u];
    un.next_f[f] = -1;
    if (un.tail_f[e] < 0) un.head_f[e] = f; else un.next_f[un.tail_f[e]] = f;
    un.tail_f[e] = f;
    un.n[e] += 1;
}

// Membership changed under the cache (splits, deferred splits carried out, states buffered or
// released): rebuild unit u's frame lists from the frame -> cluster map (negative: in no cluster)
// and the buffered singletons, and derive every entry's cache state from its frames.
void HostTier::rebuild(int u, const int *assign, int n_frames, const int *buf_frame, int n_buf) {
    Unit &un = units[u];
    std::fill(un.n.begin(), un.n.end(), 0);
    std::fill(un.head_f.begin(), un.head_f.end(), -1);
    std::fill(un.tail_f.begin(), un.tail_f.end(), -1);
    for (int f = 0; f < n_frames; ++f)
        if (assign[f] >= 0 && assign[f] < C) join(u, f, assign[f]);
    for (int b = 0; b < n_buf && C + b < E; ++b) join(u, buf_frame[b], C + b);
    un.n_cached = 0;
    for (int e = 0; e < E; ++e) {
        int have = 0;
        long long st = 0;
        char ah = 0;
        for (int f = un.head_f[e]; f >= 0; f = un.next_f[f])
            if (un.slot[f] >= 0) { ++have; st = std::max(st, un.fstamp[f]); ah |= un.ahead[f]; }
        un.cached[e] = have; un.stamp[e] = st; un.by_prefetch[e] = ah;
        un.n_cached += have > 0;
    }
    un.resident_dirty = true;
}

// Can entries ids[0..n_ids) of unit u be resident together?  Everything that is not part of
// the selection may be evicted, so the answer depends only on the selection's own footprint
// in pages and on its entry count.  Fills the fail_* fields when the answer is no.
bool HostTier::fits(int u, const int *ids, int n_ids) {
    const Unit &un = units[u];
    long long need = 0;
    for (int i = 0; i < n_ids; ++i) need += un.n[ids[i]];
    if (need <= cache_pages && n_ids <= std::max(max_clusters, 1)) return true;
    fail_need = (int)need; fail_free = (int)un.free_slots.size(); fail_cached = un.n_cached;
    fail_sel_pages = (int)need;
    return false;
}

// (With `prefetch` the ids are a prediction for a coming layer, see mosaic_prefetch: the same
// cache work, counted apart.)
// Make entries ids[0..n_ids) of unit u resident: decide what must move (LRU at cluster
// granularity, the selection itself is never evicted; entries used at the same time -- the
// halves of a split -- go lowest id first), write the moves as (host page, cache slot) pairs
// to `moves` (room for 2 ints per frame of the unit) and the cache slots of the selection, in
// gather order (entries as listed, frames ascending), to `pages` (room for one int per frame);
// the counts come back in *n_moves / *n_pages.  A selection that cannot be resident together
// (fits()) changes nothing and returns MOSAIC_ECAPACITY: the directory only ever describes
// data that a fetch kernel was given to move.  The data itself is moved afterwards by ONE
// fetch kernel per retrieve that reads the pinned slabs directly over PCIe (measured at the
// rate of a large DMA copy, without a per-copy API cost).  Allocates nothing.
int HostTier::fetch(int u, const int *ids, int n_ids, int *moves, int *n_moves, int *pages, int *n_pages,
                    bool prefetch) {
    Unit &un = units[u];
    *n_moves = 0; *n_pages = 0;
    if (!fits(u, ids, n_ids)) return MOSAIC_ECAPACITY;
    std::fill(pinned.begin(), pinned.end(), 0);
    for (int i = 0; i < n_ids; ++i) pinned[ids[i]] = 1;
    int nm = 0, np = 0;
    if (!prefetch) un.n_last_frames = 0;
    for (int i = 0; i < n_ids; ++i) {
        const int c = ids[i];
        const int have = un.cached[c];
        const int want = un.n[c];
        const bool complete = have == want;
        if (prefetch) {                      // a guess for a coming layer: not a retrieval's hit or miss
            if (!complete) pf_fetched += 1;
        } else {
            if (complete) { hits += 1; if (un.by_prefetch[c]) pf_useful += 1; } else misses += 1;
        }
        // room: enough free slots, and not more resident entries than allowed
        while ((int)un.free_slots.size() < want - have || (have == 0 && un.n_cached >= max_clusters)) {
            int victim = -1;
            for (int j = 0; j < E; ++j)
                if (un.cached[j] > 0 && !pinned[j] && (victim < 0 || un.stamp[j] < un.stamp[victim])) victim = j;
            if (victim < 0) {                 // cannot happen after fits(); kept as a guard
                fail_need = want - have; fail_free = (int)un.free_slots.size(); fail_cached = un.n_cached;
                fail_sel_pages = 0;
                for (int q = 0; q < n_ids; ++q) fail_sel_pages += un.n[ids[q]];
                return MOSAIC_ECAPACITY;
            }
            for (int f = un.head_f[victim]; f >= 0; f = un.next_f[f])
                if (un.slot[f] >= 0) { un.free_slots.push_back(un.slot[f]); un.slot[f] = -1; un.ahead[f] = 0; }
            un.cached[victim] = 0; un.by_prefetch[victim] = 0;
            un.n_cached -= 1;
            evictions += 1;
            un.resident_dirty = true;
        }
        if (have == 0 && want > 0) { un.n_cached += 1; un.resident_dirty = true; }
        const long long now = ++clock;
        for (int f = un.head_f[c]; f >= 0; f = un.next_f[f]) {
            if (un.slot[f] < 0) {                     // still in host memory only
                un.slot[f] = un.free_slots.back();
                un.free_slots.pop_back();
                moves[2 * nm] = un.host_page[f];
                moves[2 * nm + 1] = un.slot[f];
                ++nm;
            }
            un.fstamp[f] = now;
            un.ahead[f] = prefetch ? (char)(un.ahead[f] | !complete) : (char)0;
            pages[np++] = un.slot[f];
            if (!prefetch) un.last_frames[un.n_last_frames++] = f;
        }
        h2d_bytes += (long long)(want - have) * (long long)(kpage + vpage);
        un.cached[c] = want;
        un.stamp[c] = now;
        un.by_prefetch[c] = prefetch ? (char)(un.by_prefetch[c] | !complete) : (char)0;
    }
    *n_moves = nm; *n_pages = np;
    return MOSAIC_OK;
}

} // namespace mosaic
