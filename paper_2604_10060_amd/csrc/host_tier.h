// Host-side bookkeeping of the pinned-host tier: slab chains per cluster and the
// per-unit GPU cluster cache (LRU at cluster granularity).  See host_tier.hip.
#pragma once
#include <hip/hip_runtime.h>
#include <vector>

namespace mosaic {

struct HostTier {
    struct Entry {
        std::vector<int> blocks;   // cache blocks (of SF pages) holding the cluster, in slab order
        int pages = 0;             // frames of the cluster that are resident
        long long stamp = 0;       // last use (LRU)
        bool present = false;
        bool by_prefetch = false;  // brought in (or completed) by a prefetch and not used by a retrieval yet
    };
    struct Unit {
        std::vector<std::vector<int>> slabs;    // per cluster: its host slabs in arrival order
        std::vector<std::vector<int>> frames;   // per cluster: member frame ids, ascending
        std::vector<int> n;                     // per cluster: frames
        int next_slab = 0;                      // bump allocator of the unit's host pool
        std::vector<Entry> cache;               // per cluster
        std::vector<int> free_blocks;
        int n_cached = 0;
    };
    int U = 0, C = 0, SF = 8, slabs_per_unit = 0, cache_blocks = 0, max_clusters = 0;
    size_t kpage = 0, vpage = 0;                // bytes of one K / V page
    std::vector<Unit> units;
    long long clock = 0;
    int fail_need = 0, fail_free = 0, fail_cached = 0, fail_sel_pages = 0;   // context of the last ECAPACITY
    long long hits = 0, misses = 0, evictions = 0, h2d_bytes = 0, h2d_copies = 0;
    // cross-layer prefetch: clusters a prefetch had to fetch, and how many of them a retrieval then used
    long long pf_calls = 0, pf_fetched = 0, pf_useful = 0;
    // streams and events owned by the context
    hipStream_t sel_stream = nullptr;    // selection kernel + read-back of the ids
    hipStream_t copy_stream = nullptr;   // fetch kernel, page-list upload, `ready` events
    hipEvent_t main_mark = nullptr;                 // marks the caller's stream at each retrieve
    std::vector<hipEvent_t> ready, attend_done;     // per layer
    std::vector<char> attend_recorded, ready_recorded;
    std::vector<hipEvent_t> busy_ev;                // pairs around each retrieve's copies
    double busy_ms = 0.0;
    // latest selection per unit, kept for the observer
    std::vector<std::vector<int>> last_ids;

    void init(int U, int C, int SF, int slabs_per_unit, int cache_blocks, int max_clusters,
              size_t kpage, size_t vpage);
    void reset();
    int append(int u, int f, int c);
    int fetch(int u, const int *ids, int n_ids, std::vector<int> &moves, std::vector<int> &pages,
              bool prefetch = false);
};

} // namespace mosaic
