// Host-side bookkeeping of the pinned-host tier: where every frame's page lives in pinned
// memory (cluster-contiguous slab chains), which frames are in the GPU cluster cache, and
// the least-recently-used replacement at cluster granularity.  See host_tier.hip.
// Every array is sized when the context is created: nothing here allocates afterwards.
#pragma once
#include <hip/hip_runtime.h>
#include <vector>

namespace mosaic {

struct HostTier {
    struct Unit {
        // entries = cluster ids [0, C) and, with the deferred-split maintainer, the buffered
        // singletons [C, C + buf_max) (Alg. 1 line 10: a buffered state is a cluster of its own)
        // entries as ascending frame lists (singly linked through next_f)
        std::vector<int> n, head_f, tail_f;      // [E]
        std::vector<int> next_f;                 // [F]
        // pinned-host placement: a cluster appends to its open slab; host_page[f] = slab * SF + slot
        std::vector<int> open_slab, open_fill;   // [C]  -1 / frames already in the open slab
        std::vector<int> host_page;              // [F]
        int next_slab = 0;                       // bump allocator of the unit's slab pool
        // GPU cluster cache, state per frame: its page slot, when it was last used, and whether a
        // prefetch brought it in and no retrieval has used it since
        std::vector<int> slot;                   // [F]  cache slot of the frame, -1 = not cached
        std::vector<long long> fstamp;           // [F]
        std::vector<char> ahead;                 // [F]
        std::vector<int> free_slots;             // stack of free slots
        // ... and per entry, derived from its frames (kept up to date by fetch(), recomputed by rebuild())
        std::vector<int> cached;                 // [E]  member frames that are in the cache (> 0: resident)
        std::vector<long long> stamp;            // [E]  last use: the latest of its cached frames'
        std::vector<char> by_prefetch;           // [E]  some cached member frame was fetched ahead and not used yet
        int n_cached = 0;                        // resident entries
        // latest selection, kept for the observer: ids, and the frames in gather order as the query saw them
        std::vector<int> last_ids;               // [top_k]
        int n_last = 0;
        std::vector<int> last_frames;            // [F]
        int n_last_frames = 0;
        bool resident_dirty = false;             // the device's copy of the residency flags is out of date
    };
    int U = 0, C = 0, E = 0, F = 0, SF = 8, slabs_per_unit = 0, cache_pages = 0, max_clusters = 0, top_k = 0;
    size_t kpage = 0, vpage = 0;                // bytes of one K / V page
    std::vector<Unit> units;
    std::vector<char> pinned;                   // [E] scratch of fetch(): the current selection
    long long clock = 0;
    int fail_need = 0, fail_free = 0, fail_cached = 0, fail_sel_pages = 0;   // context of the last ECAPACITY
    long long hits = 0, misses = 0, evictions = 0, h2d_bytes = 0, h2d_copies = 0;
    // cross-layer prefetch: clusters a prefetch had to fetch, and how many of them a retrieval then used
    long long pf_calls = 0, pf_fetched = 0, pf_useful = 0;
    // streams and events owned by the context
    hipStream_t sel_stream = nullptr;    // selection kernel + read-back of the ids
    hipStream_t copy_stream = nullptr;   // fetch kernel, page-list upload, `ready` events
    hipEvent_t main_mark = nullptr;                 // marks the caller's stream at each retrieve
    // ingest: the offload of a staged batch runs on the copy stream while the caller's stream goes on with the
    // next batch; two slab tables (host and device) used in turn, an event per table for "offload finished",
    // and the frames each still-counted offload read from the staging ring
    hipEvent_t off_ready = nullptr, off_done[2] = {nullptr, nullptr};
    bool off_used[2] = {false, false};
    long long off_f0[2] = {0, 0}, off_f1[2] = {0, 0};
    long long off_idx = 0;
    // eager maintainer: splits since the host last followed a layer's units (followed when the layer is next queried)
    std::vector<char> follow_dirty;              // [L]
    std::vector<hipEvent_t> ready, attend_done;     // per layer
    std::vector<char> attend_recorded, ready_recorded;
    // timing of the fetch kernels while profiling is on: a fixed pool of event pairs, folded into
    // busy_ms when it is full or when the statistics are read
    std::vector<hipEvent_t> busy_ev;
    size_t busy_used = 0;
    double busy_ms = 0.0;
    // maintainer on the host tier: what the host last saw of each unit's counters (splits on insertion,
    // deferred splits) and buffer fill, to tell when its frame lists are out of date
    std::vector<long long> seen_splits;          // [U][2]
    std::vector<int> seen_nbuf;                  // [U]

    void init(int U, int C, int n_entries, int F, int SF, int slabs_per_unit, int cache_pages, int max_clusters,
              int top_k, size_t kpage, size_t vpage);
    void reset();
    int place(int u, int f, int c);
    void join(int u, int f, int e);
    void rebuild(int u, const int *assign, int n_frames, const int *buf_frame, int n_buf);
    bool fits(int u, const int *ids, int n_ids);
    int fetch(int u, const int *ids, int n_ids, int *moves, int *n_moves, int *pages, int *n_pages,
              bool prefetch = false);
};

} // namespace mosaic
