/*
 * libmosaic -- cluster-driven KV-cache management for streaming long-video
 * VLM inference on one MI355X (gfx950): C ABI.
 *
 * The calls mirror the two-stage workflow of the paper's problem statement
 * (Sec. V-A "Setup"): Frame Encoding = mosaic_ingest_frame (update the
 * layer-wise KV cache and its cluster structure as frames arrive), Query
 * Retrieval = mosaic_retrieve + mosaic_attend (select the relevant clusters
 * and run attention over them only).
 *
 * Vocabulary.  L layers, Hq query heads, Hkv KV heads, G = Hq/Hkv, D head_dim,
 * T tokens per frame, C clusters, k = top_k.  A "unit" is one (layer, KV head)
 * pair, index u = layer*Hkv + head; units never interact.  The thing that is
 * clustered is the frame: its state is the mean of its T key vectors, and all
 * T tokens (keys and values) follow the frame into its cluster.
 *
 * Conventions.
 *  - Every function returns a mosaic_status; nothing throws or aborts across
 *    the boundary.  mosaic_last_error() gives the text of the last failure.
 *  - "device pointer" = HIP device memory of the GPU current at mosaic_create;
 *    "host pointer" = ordinary host memory.  Stated per argument.
 *  - All device work is enqueued on config.stream (a hipStream_t passed as
 *    void*).  ingest / retrieve / attend / reset do not synchronise; the
 *    mosaic_get_* observers do (they copy to host memory).
 *  - The library allocates no device memory: the caller provides one arena
 *    (size from mosaic_workspace_size) which is borrowed until
 *    mosaic_destroy.  Input buffers passed to a call must stay valid until
 *    the stream has passed that call.
 *  - A handle is not thread-safe; distinct handles are independent.
 *  - Decision arithmetic (frame summaries, cosine similarities, representative
 *    updates, query scores, top-k) is fp64 on the device; attention
 *    accumulates in fp32.
 */
#ifndef MOSAIC_H
#define MOSAIC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct mosaic_ctx mosaic_ctx; /* one per video stream */

typedef enum {
    MOSAIC_OK = 0,
    MOSAIC_EINVAL = -1,    /* bad argument or unsupported shape */
    MOSAIC_ENOMEM = -2,    /* arena too small */
    MOSAIC_ECAPACITY = -3, /* more than max_frames frames, or an output buffer too small */
    MOSAIC_ENOTREADY = -4, /* retrieve before the initial clustering, or attend before retrieve */
    MOSAIC_EHIP = -5       /* a HIP call failed (text in mosaic_last_error) */
} mosaic_status;

enum { MOSAIC_FP32 = 0, MOSAIC_BF16 = 1 };
enum { MOSAIC_TIER_HBM = 0, MOSAIC_TIER_HOST = 1 };
enum { MOSAIC_ATTEND_AUTO = 0, /* bf16 -> MFMA kernel, fp32 -> vector-ALU kernel */
       MOSAIC_ATTEND_VALU = 1, /* vector-ALU kernel for either dtype */
       MOSAIC_ATTEND_MFMA = 2  /* MFMA kernel (bf16 only) */ };

typedef struct {
    int32_t n_layers, n_q_heads, n_kv_heads;
    int32_t head_dim;         /* 64 or 128 */
    int32_t tokens_per_frame; /* T >= 1 */
    int32_t max_frames;       /* capacity of the stream */
    int32_t n_clusters;       /* C, 1..1024, fixed */
    int32_t top_k;            /* 1..C */
    int32_t kv_dtype;         /* MOSAIC_FP32 | MOSAIC_BF16: dtype of K, V, q and the attention output */
    int32_t warmup_frames;    /* W; 0 -> 2*C.  The first W frames are buffered, then the initial clustering runs */
    int32_t lloyd_iters;      /* rounds of the cosine K-means used at init and re-clustering; 0 -> 8 */
    int32_t recluster_every;  /* 0 = never; else a warm-started full re-clustering whenever the frame
                                 count reaches a multiple of it beyond the warm-up */
    int32_t score_mode;       /* 0 cosine (paper Sec. V-B criterion), 1 plain dot product */
    int32_t max_q_tokens;     /* largest n_q_tokens retrieve/attend will be given; 0 -> 256 */
    int32_t attend_impl;      /* MOSAIC_ATTEND_* */
    int32_t tier;             /* MOSAIC_TIER_HBM: all K/V pages stay in the device arena;
                                 MOSAIC_TIER_HOST: pages are offloaded to pinned host memory in
                                 cluster-contiguous slabs and fetched cluster by cluster into a GPU
                                 cluster cache (paper Sec. V-A, V-C: clusters live in CPU memory and
                                 are the retrieval units) */
    void *dev_arena;          /* device pointer, 256-byte aligned, borrowed */
    size_t dev_arena_bytes;
    void *stream;             /* hipStream_t, borrowed; NULL = the null stream */
    /* host tier only (ignored for MOSAIC_TIER_HBM) */
    int32_t slab_frames;          /* frames per host slab (a cluster's pages are contiguous in runs of
                                     this many frames, keys then values); 0 -> 8 */
    int32_t cache_pages_per_unit; /* GPU cluster-cache capacity per unit, in frame pages; 0 -> 3 *
                                     max(cache_fraction, top_k/C) * max_frames + top_k, at most the
                                     whole stream.  A selection whose clusters hold more frames than
                                     this cannot be attended: mosaic_retrieve then fails (ECAPACITY) */
    float cache_fraction;         /* at most floor(cache_fraction * C) clusters (but at least top_k) are
                                     cached per unit, least recently used evicted first; 0 -> 0.10 */
    int32_t decode_fused_max_mib; /* (any tier; sits here for alignment) mosaic_decode_step runs its single
                                     fused kernel (equal splits) while the expected K/V volume of the step is
                                     at most this many MiB; 0 -> 48; -2: always the two calls; -1: never that
                                     kernel but, wherever it applies, the one-launch form with proportional
                                     splits (an option kept for measurement: slower than the two calls) */
    void *host_arena;             /* HOST pointer to pinned (hipHostMalloc) memory, 256-byte aligned,
                                     borrowed; size from mosaic_workspace_size */
    size_t host_arena_bytes;
    /* Self-adaptive maintainer (paper Sec. VI); excludes recluster_every.  In the host tier a split
     * moves no page: a frame keeps its place in pinned memory and its slot in the GPU cluster cache,
     * the host follows the new membership (it reads the unit's frame -> cluster map back when the
     * unit's split counters or buffer fill have moved), and both halves inherit what the cache holds
     * of the parent and its time of last use.
     * Every insertion updates the cluster's running variance (Eq. 4) next to its representative
     * (Eq. 3); a cluster whose variance exceeds the size-adaptive threshold (Eq. 5, evaluated at
     * its size before the insertion) is refined by a two-way Split (two-means under the cosine
     * criterion, seeds = the two members with the lowest mutual cosine).  n_clusters is then the
     * capacity of the cluster table: the initial K-means builds init_clusters clusters and every
     * split adds one (no free id left: the state is absorbed without refinement). */
    int32_t maint_mode;           /* MOSAIC_MAINT_OFF | _EAGER | _DEFERRED */
    int32_t init_clusters;        /* 1..n_clusters; 0 -> max(1, n_clusters / 2); warmup_frames 0 -> 2 * init_clusters */
    int32_t split_iters;          /* two-means rounds of Split; 0 -> 4 */
    int32_t buffer_max;           /* _DEFERRED: capacity of the per-unit buffer of singletons (Alg. 1, B);
                                     0 -> 32; n_clusters + buffer_max <= 1024.  A full buffer: absorbed */
    double tau_min, tau_max;      /* Eq. 5: threshold for large / for small clusters (squared distance) */
    double tau_n0;                /* Eq. 5: transition rate N0 > 0 */
    /* Retrieval augmentation (paper Sec. V-C, "Retrieval Augmentation"); MOSAIC_TIER_HBM only, not
     * with MOSAIC_MAINT_DEFERRED.  mosaic_attend then attends over the retrieved clusters AND
     *  (1) aug_global_reps = 1: one pseudo token per non-empty cluster, key = its representative
     *      (Eq. 1), value = the mean of its members' value vectors (a compact global view);
     *  (2) aug_window_frames = w > 0: all tokens of the w most recent frames (local window).
     * Every real token is attended once: a window frame that also belongs to a selected cluster
     * is listed with the window only.  The three parts are one softmax (merged exactly through
     * their log-sum-exp). */
    int32_t aug_global_reps;
    int32_t aug_window_frames;
    /* mosaic_prefetch (host tier): how many of the predicted top-k clusters are fetched ahead,
     * best first; 0 -> top_k (the paper's scheme).  A smaller number wastes less PCIe time on
     * marginal predictions that the actual query may not confirm. */
    int32_t prefetch_top_k;
    /* Nested visual-semantic hierarchy and two-stage retrieval (paper Sec. V-B "Nested Hierarchy",
     * Sec. V-C "Two-Stage Retrieval"); n_partitions = 0: flat index.  MOSAIC_TIER_HBM only, without
     * the maintainer, periodic re-clustering and augmentation.  With P = n_partitions > 0:
     *  - frames are ingested with mosaic_ingest_frame_visual, which also takes the frame's visual
     *    embedding (visual_dim floats).  The visual level clusters these embeddings once per stream
     *    with the same modified K-means as the semantic level (warm-up of W frames, then P-means with
     *    seeds = embeddings of frames floor(p*W/P), then greedy cosine assignment and Eq. 3), and
     *    gives every frame a partition;
     *  - n_clusters must be a multiple of P: partition p owns the cluster ids [p*Cs, (p+1)*Cs),
     *    Cs = n_clusters / P.  A unit's K-means runs inside each partition (a partition with np
     *    warm-up members starts min(Cs, np) clusters from its members floor(j*np/min(Cs, np))), and a
     *    new frame is compared with the non-empty clusters of its own partition only;
     *  - mosaic_retrieve first scores, per unit, the P partition representatives (mean key summary
     *    of the partition's frames: the query lives in the layer's key space, not the vision
     *    encoder's), keeps the top_partitions best, then scores only the clusters of those and
     *    keeps the top_k of them. */
    int32_t n_partitions;         /* P, 0..64 */
    int32_t visual_dim;           /* Dv, 1..4096 */
    int32_t top_partitions;       /* 1..P; 0 -> max(1, P / 4) */
    /* Batched matching, overlapped (paper Sec. VII-A: frame encoding is pipelined; the assignment of
     * frame t depends on frame t-1, its page store does not).  1: the order-dependent part of
     * mosaic_ingest_frame -- assignment chain, initial clustering, re-clustering -- runs on a stream
     * the context owns, after the call's page stores (an event), while the caller's stream goes on
     * with the next call's page stores.  Every mosaic_* call that reads or changes the index first
     * makes the caller's stream wait for that work, so results are the same bit for bit; work the
     * caller enqueues on its stream by itself (or a synchronisation of that stream alone) is NOT
     * ordered after it: call mosaic_ingest_join first.  MOSAIC_TIER_HBM, n_partitions = 0 and calls
     * of more than one frame only (other calls run wholly on the caller's stream, as with 0). */
    int32_t ingest_overlap;
} mosaic_config;

/* maint_mode.  _EAGER: every cluster counts as GPU resident, an invalid cluster is split at once
 * (Alg. 1 lines 4-6).  _DEFERRED: Alg. 1 in full.  "GPU resident" means, in the host tier, that
 * the GPU cluster cache holds frames of the cluster (the split itself needs only the frame
 * summaries, which never leave the GPU); in the HBM tier, where everything is resident, it is
 * emulated as "selected by the unit's latest mosaic_retrieve" (the working set such a cache would
 * hold).  An invalid cluster that is not resident gets a lazy-split flag and the new state is kept in the buffer as a singleton
 * cluster that retrieval can select (id n_clusters + buffer slot); the split is carried out when
 * mosaic_retrieve next selects the flagged cluster (lines 12-17), after that query's page list
 * has been built. */
enum { MOSAIC_MAINT_OFF = 0, MOSAIC_MAINT_EAGER = 1, MOSAIC_MAINT_DEFERRED = 2 };

typedef struct {
    int64_t frames_ingested;
    int64_t lloyd_runs;        /* initial clustering + re-clusterings */
    int64_t retrieve_calls, attend_calls;
    int64_t kv_bytes_stored;   /* K+V bytes written into the arena so far */
    int32_t ready;             /* 1 once the initial clustering has run */
    int32_t attend_impl;       /* the kernel family in use (MOSAIC_ATTEND_VALU or _MFMA) */
    int32_t last_n_splits;     /* average KV splits per unit used by the latest attend */
    int32_t last_decode_fused; /* what the latest mosaic_decode_step ran: 0 = mosaic_retrieve + mosaic_attend,
                                  1 = the single fused kernel (equal splits), 2 = selection inside the attention
                                  launch with size-proportional splits */
    /* host tier */
    int64_t cache_hits, cache_misses;   /* selected clusters found in / missing from the GPU cache */
    int64_t h2d_bytes, h2d_copies;      /* cluster fetches: bytes moved host-to-device and fetch-kernel launches */
    double h2d_busy_ms;                 /* time of those fetch kernels (event pairs around each launch while
                                           mosaic_profile_enable is on; filled by mosaic_get_stats, which
                                           synchronises) */
    /* cross-layer prefetch (host tier) */
    int64_t prefetch_calls;             /* mosaic_prefetch calls */
    int64_t prefetch_fetched;           /* clusters a prefetch had to bring into the GPU cache */
    int64_t prefetch_useful;            /* of those, clusters that the layer's retrieval then selected */
    /* maintainer, summed over the units (filled by mosaic_get_stats, which synchronises) */
    int64_t splits_immediate;           /* invalid clusters split on insertion */
    int64_t splits_deferred;            /* deferred splits carried out at retrieval */
    int64_t deferred_inserts;           /* states put into the singleton buffer */
    int64_t forced_absorbs;             /* invalid, but absorbed: no free cluster id, degenerate split, or full buffer */
    int64_t sync_timeouts;              /* nonzero if a bounded wait inside a kernel (the selection exchange of
                                           mosaic_decode_step's one-launch form) ever ran out: results of that
                                           step are then undefined (filled by mosaic_get_stats) */
} mosaic_stats;

/* Bytes of device arena and of pinned host arena (0 for MOSAIC_TIER_HBM) a
 * context with this configuration needs (the arena fields of cfg are
 * ignored).  dev_bytes, host_bytes: host pointers; host_bytes may be NULL. */
int32_t mosaic_workspace_size(const mosaic_config *cfg, size_t *dev_bytes, size_t *host_bytes);

/* Pinned, device-mapped host memory of exactly `bytes` bytes for config.host_arena (hipHostMalloc in
 * the HIP runtime the library itself uses), and its release.  A convenience for callers whose own
 * pinned allocator rounds sizes up; any hipHostMalloc memory serves as host_arena.  out: host
 * pointer to a host pointer.  Errors: EINVAL, ENOMEM (the runtime refused; text in
 * mosaic_last_error(NULL)). */
int32_t mosaic_host_alloc(size_t bytes, void **out);
int32_t mosaic_host_free(void *p);

/* One context per video stream: the "layer-wise KVCache" that Frame Encoding updates and Query
 * Retrieval reads (Sec. V-A "Setup"), with the state Alg. 1 lists per cluster (representative,
 * variance, lazy-split flag, GPU buffer, representative set).  Validates cfg, carves the arena;
 * the only device work it enqueues clears the maintainer's counters.  out: host pointer.
 * Host tier: the library creates two default-priority streams of its own (selection; fetches)
 * and per-layer events, because the overlap of Sec. VII-B is between the library's own fetch of
 * layer l+1 and the caller's attention of layer l: the caller hands over one stream and the
 * library orders its internal streams against it with events, never with a host wait on the
 * caller's stream.  Errors: EINVAL, ENOMEM (arena too small), EHIP. */
int32_t mosaic_create(const mosaic_config *cfg, mosaic_ctx **out);
/* Waits for the context's streams, releases the library's streams and events; the arenas stay
 * the caller's. */
int32_t mosaic_destroy(mosaic_ctx *ctx);

/* A new video stream on the same context (Sec. V-A: the cache is built per stream): forget all
 * frames, clusters, maintainer state (Alg. 1 "State") and cache contents; keep the arenas and the
 * configuration.  Stream-ordered in the HBM tier; the host tier waits for its streams first. */
int32_t mosaic_reset(mosaic_ctx *ctx);

/* Frame Encoding (Sec. V-A (1); Sec. VI-A greedy assignment and Eq. 3; Sec. VII-A
 * batched matching when n_frames > 1).
 * k_dev, v_dev: device pointers, [n_frames][L][Hkv][T][D] in kv_dtype, the
 * keys and values of the next n_frames frames in stream order.  For every
 * frame and unit: the K and V pages are copied into the arena, the frame's
 * key summary is formed, and -- once W frames are in -- the frame is assigned
 * to the non-empty cluster with the most similar representative (cosine; ties
 * to the lowest id) whose representative is then updated by Eq. 3.  The result
 * is identical to n_frames calls with one frame each.
 * Errors: EINVAL (NULL, n_frames < 1), ECAPACITY (max_frames exceeded; nothing
 * is ingested).
 * Host tier: the pages are written to a device staging ring, the batch's
 * assignments are read back (this call then synchronises the stream once), and
 * a kernel stores each page into its cluster's slab in the pinned host arena.
 * Re-clustering (recluster_every > 0) is not available in the host tier. */
int32_t mosaic_ingest_frame(mosaic_ctx *ctx, const void *k_dev, const void *v_dev,
                            int32_t n_frames);

/* Makes the context's stream (mosaic_config.stream) wait for the order-dependent part of earlier
 * mosaic_ingest_frame calls that ingest_overlap = 1 put on the context's own stream.  Enqueues a
 * wait, does not block the host; no-op when nothing is pending.  Sec. VII-A (pipelined encoding). */
int32_t mosaic_ingest_join(mosaic_ctx *ctx);

/* Frame Encoding under the nested hierarchy (Sec. V-B; config.n_partitions > 0, where it replaces
 * mosaic_ingest_frame, which then fails with EINVAL -- and vice versa).  k_dev, v_dev, n_frames
 * as for mosaic_ingest_frame; e_dev: device pointer, fp32 [n_frames][visual_dim], 16-byte
 * aligned, the frames' visual embeddings.  Identical to n_frames calls with one frame each. */
int32_t mosaic_ingest_frame_visual(mosaic_ctx *ctx, const void *k_dev, const void *v_dev,
                                   const float *e_dev, int32_t n_frames);

/* Query Retrieval, selection part (Sec. V-C "Cluster Indexing" / second stage
 * of "Two-Stage Retrieval"; top-K of Sec. VII-B).
 * layer >= 0: that layer only, q_dev is [Tq][Hq][D]; layer == -1: all layers,
 * q_dev is [L][Tq][Hq][D].  q_dev: device pointer, kv_dtype.
 * Per unit: mean query over the Tq tokens and the unit's G query heads;
 * score_j = (mean query . r_j)/|r_j| for non-empty clusters; the top_k best by
 * (score descending, id ascending); then the page list of those clusters
 * (clusters in selection order, member frames ascending).  The selection stays
 * in the context until the next retrieve for that layer or the next ingest.
 * Errors: ENOTREADY before W frames are in; EINVAL (layer, n_q_tokens out of
 * range, NULL).
 * Host tier (layer >= 0 only): scoring and top-k run on an internal selection
 * stream, the ids are read back (the call waits for that small copy only), and
 * every page of a selected cluster that is missing from the unit's GPU cache is
 * moved by one fetch kernel per call on an internal copy stream (the kernel
 * reads the pinned slabs over PCIe), so that the fetch for layer l+1 overlaps
 * mosaic_attend of layer l when retrieve(l+1) is issued before attend(l).
 * ECAPACITY if the selection does not fit the cache: the cache and its directory are then left
 * exactly as they were and the layer has no current selection. */
int32_t mosaic_retrieve(mosaic_ctx *ctx, int32_t layer, const void *q_dev,
                        int32_t n_q_tokens);

/* Overlap-aware prefetch (paper Sec. VII-B), host tier only.  While layer l is being computed,
 * its query q^(l) serves as a proxy for the next layer's: the call selects the top-k clusters of
 * `layer` (= l + 1) with q_proxy_dev -- same shape and dtype as mosaic_retrieve's q_dev, one layer --
 * and starts fetching those that are not in the GPU cluster cache, asynchronously on the library's
 * copy stream, so that the transfer overlaps whatever the caller enqueues next (layer l's
 * attention).  It does not make a selection: the later mosaic_retrieve(layer, q^(l+1)) verifies the
 * prediction against the actual query and fetches whatever is still missing (the completion
 * step); results never depend on whether, or with which proxy, mosaic_prefetch was called.
 * Contains the same short host wait as the host tier's mosaic_retrieve (read-back of k ids).
 * Errors: EINVAL (not the host tier, layer < 0, NULL, n_q_tokens out of range); ENOTREADY;
 * ECAPACITY if the predicted clusters do not fit the cache (nothing is fetched or evicted then). */
int32_t mosaic_prefetch(mosaic_ctx *ctx, int32_t layer, const void *q_proxy_dev, int32_t n_q_tokens);

/* Query Retrieval, attention part (Sec. V-A (2)): softmax(q K^T/sqrt(D)) V over
 * the tokens of the clusters chosen by the latest mosaic_retrieve for `layer`
 * (same `layer` convention), query head hq reading KV head hq / G, no mask.
 * q_dev as in mosaic_retrieve; out_dev [.][Tq][Hq][D] in kv_dtype and lse_dev
 * [.][Tq][Hq] fp32 (natural-log sum of exponentials of the scaled logits; may
 * be NULL) are device pointers.
 * Errors: ENOTREADY if no selection is current for the layer; EINVAL.
 * Host tier: the stream first waits (on the device) for the layer's fetches. */
int32_t mosaic_attend(mosaic_ctx *ctx, int32_t layer, const void *q_dev,
                      int32_t n_q_tokens, void *out_dev, float *lse_dev);

/* mosaic_attend for callers that cannot allocate or be handed scratch memory sized per call: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * results and errors as mosaic_attend (the same kernels run), but the per-split attention partials
 * live in a 16 MiB buffer that is part of the library's device image (one per GPU, held until the
 * process ends) instead of in the arena; the call allocates nothing on the host or the device and
 * ignores mosaic_profile_enable.  A call needs units x row tiles partial entries at the least
 * (units = n_kv_heads, or L * n_kv_heads for layer == -1; row tiles = ceil(n_q_tokens * G / 16);
 * an entry is 16 * head_dim * 4 + 192 bytes: 2001 entries at head_dim 128, 3912 at 64) and takes
 * fewer KV splits when the buffer is short; ECAPACITY if even one split per row tile does not fit.
 * Nothing in the buffer has to survive or be cleared between calls (every entry a call reads it has
 * written itself), but all handles on one GPU share it: calls whose kernels may overlap on that GPU
 * (different streams, no ordering between them) race and must be serialised by the caller. */
int32_t mosaic_attend_static(mosaic_ctx *ctx, int32_t layer, const void *q_dev, int32_t n_q_tokens,
                             void *out_dev, float *lse_dev);

/* One decode step in one call: mosaic_retrieve(layer, q) followed by mosaic_attend(layer, q) --
 * same arguments, errors, selection left behind (ids, scores, page list: the observers and a
 * later mosaic_attend see it) and the same output up to the order in which fp32 partial sums are
 * merged.  Where it applies -- MOSAIC_TIER_HBM, bf16 MFMA attention, layer >= 0, at most 16 query
 * rows per KV head (n_q_tokens * Hq/Hkv <= 16), n_clusters <= 256, maintainer, augmentation and
 * nested index off, and an expected K/V volume of the step (frames * top_k / n_clusters pages per
 * KV head) of at most decode_fused_max_mib (default 48) MiB, i.e. a step that is bound by launch and memory latency rather than
 * by bandwidth -- the selection and the attention over the selected clusters run in ONE kernel
 * (every attention workgroup repeats its unit's selection for itself, which is cheaper than a
 * launch boundary and the dependent loads after it; KV splits are then equal per unit instead of
 * proportional to the retrieved size).  Everywhere else the call simply makes the two calls.
 * With decode_fused_max_mib = -1, under the same conditions otherwise (and n_kv_heads <= 64), the
 * selection moves into the attention launch but is made once per unit: the launch's first Hkv
 * workgroups select for one KV head each and publish the result through memory, all workgroups
 * wait for that (a bounded wait on workgroups that are started first and wait for nobody;
 * sync_timeouts in the statistics counts waits that ran out) and then share out the retrieved pages
 * in proportion to the units' sizes, as mosaic_attend does.  Same results bit for bit; measured
 * slower than the two calls, because what the waiting workgroups read has to bypass the L2s. */
int32_t mosaic_decode_step(mosaic_ctx *ctx, int32_t layer, const void *q_dev, int32_t n_q_tokens,
                           void *out_dev, float *lse_dev);

/* Observers for parity checks: the clustering state of Sec. V-B / Sec. VI (frame -> cluster
 * map, representatives of Eq. 1 / Eq. 3, per-frame states) as the library holds it.  All
 * outputs are HOST pointers, caller-allocated; each call synchronises the stream.  NULL
 * outputs are skipped. */

/* frame_to_cluster [L*Hkv][n_frames_ingested] (row stride = frames ingested);
 * -1 for frames still buffered before the initial clustering. */
int32_t mosaic_get_assignments(mosaic_ctx *ctx, int32_t *frame_to_cluster);
/* r [L*Hkv][C][D] fp64 representatives, n [L*Hkv][C] cluster sizes in frames. */
int32_t mosaic_get_centroids(mosaic_ctx *ctx, double *r, int32_t *n);
/* summaries [L*Hkv][n_frames_ingested][D] fp64 per-frame key summaries. */
int32_t mosaic_get_summaries(mosaic_ctx *ctx, double *summaries);

/* Maintainer state (paper Sec. VI), maint_mode != MOSAIC_MAINT_OFF only.  All arguments are
 * HOST pointers, any may be NULL: var [L*Hkv][C] running variances (Eq. 2 after a K-means run or
 * a split, Eq. 4 after an insertion); lazy, resident [L*Hkv][C] flags of Alg. 1; n_slots [L*Hkv]
 * cluster ids in use; n_buf [L*Hkv] and buf_frame, buf_owner [L*Hkv][buffer_max] the buffered
 * singletons (frame, cluster it was assigned to).  mosaic_get_assignments reports a buffered
 * frame as -2 - owner.  Synchronises the stream. */
int32_t mosaic_get_maintainer(mosaic_ctx *ctx, double *var, int32_t *lazy, int32_t *resident,
                              int32_t *n_slots, int32_t *n_buf, int32_t *buf_frame, int32_t *buf_owner);

/* Nested hierarchy (n_partitions > 0 only).  HOST pointers, any may be NULL; synchronises.
 * frame_to_partition [n_frames_ingested] (-1 before the visual level's initial clustering);
 * visual_r [P][visual_dim] fp64 visual centroids, visual_n [P] their sizes in frames;
 * part_r [L*Hkv][P][D] fp64 per-unit partition representatives (key space), part_n [L*Hkv][P]. */
int32_t mosaic_get_partitions(mosaic_ctx *ctx, int32_t *frame_to_partition, double *visual_r,
                              int32_t *visual_n, double *part_r, int32_t *part_n);
/* First stage of the latest two-stage selection of one layer: part_ids [Hkv][top_partitions]
 * (-1 padded) in (score descending, id ascending) order, n_part_ids [Hkv], part_scores [Hkv][P]
 * (-inf for empty partitions).  mosaic_get_selection's scores are -inf for the clusters of
 * partitions that were not chosen. */
int32_t mosaic_get_partition_selection(mosaic_ctx *ctx, int32_t layer, int32_t *part_ids,
                                       int32_t *n_part_ids, double *part_scores);

/* Latest selection of one layer (layer >= 0): ids [Hkv][top_k] (-1 padded),
 * n_ids [Hkv], scores [Hkv][C] fp64 (-inf for empty clusters; with
 * MOSAIC_MAINT_DEFERRED the rows have C + buffer_max columns, column C + b
 * being buffered singleton b, and ids >= C name singletons), tok_idx
 * [Hkv][tok_cap] global token indices f*T+t in gather order, n_tok [Hkv].
 * ECAPACITY if a unit retrieved more than tok_cap tokens. */
int32_t mosaic_get_selection(mosaic_ctx *ctx, int32_t layer, int32_t *ids, int32_t *n_ids,
                             double *scores, int32_t *tok_idx, int64_t tok_cap,
                             int32_t *n_tok);
/* Host tier: directory of the GPU cluster cache (the "small working set" of Sec. V-A that stays
 * on the GPU).  cached_pages: HOST pointer, [L*Hkv][C]; -1 = the cluster is not resident, else the
 * number of its frames that are (fewer than its size if it grew since it was fetched).  Reads
 * host-side bookkeeping only; does not synchronise.  EINVAL outside the host tier. */
int32_t mosaic_get_cache_directory(mosaic_ctx *ctx, int32_t *cached_pages);

/* Counters of the path: frames, K-means runs (Sec. V-B), cache hits / misses and bytes moved
 * host-to-device (Sec. V-C, VII-B), prefetch accounting (Sec. VII-B), split counts of Alg. 1. */
int32_t mosaic_get_stats(mosaic_ctx *ctx, mosaic_stats *stats);

/* Kernel timing for benchmarks: when enabled, the split-KV attention kernel of
 * every mosaic_attend is launched with a HIP start/stop event pair that receives
 * the kernel's own begin and end timestamps on the context's stream.  The event
 * pairs come from a fixed pool that mosaic_profile_enable(on) creates (the query
 * calls create none); when the pool is used up the next timed call waits for the
 * stream and folds the times read so far into the running sum.
 * mosaic_profile_read synchronises and returns the summed kernel time and the
 * number of launches since the last read (host pointers), then clears them. */
int32_t mosaic_profile_enable(mosaic_ctx *ctx, int32_t on);
int32_t mosaic_profile_read(mosaic_ctx *ctx, double *attend_kernel_ms, int64_t *launches);

/* Counter calibration for profilers: a plain grid-stride copy of `bytes` bytes
 * (multiple of 16; both device pointers 16-byte aligned) on `stream` (hipStream_t
 * as void*).  It reads and writes exactly `bytes` bytes, so a hardware byte
 * counter read for this kernel gives the counter's scale.  Not part of the path. */
int32_t mosaic_calibration_copy(void *dst_dev, const void *src_dev, size_t bytes, void *stream);

/* Text of the last error on this handle (never NULL).  ctx may be NULL: then
 * the text of the last failed mosaic_create / mosaic_workspace_size. */
const char *mosaic_last_error(const mosaic_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* MOSAIC_H */
