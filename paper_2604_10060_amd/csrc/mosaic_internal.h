// Internal declarations shared by the HIP sources of libmosaic (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>
#include <string>
#include <vector>

#include "../../include/mosaic.h"

namespace mosaic {

constexpr int kBlock = 256;       // threads per workgroup (4 wavefronts of 64)
constexpr int kRowTile = 16;      // query rows per attention tile
constexpr int kChunk = 32;        // tokens per attention step, always inside one page
constexpr int kMaxSplits = 64;    // KV splits per (unit, row tile), average over the units of a launch
constexpr int kMaxUnitSplits = 256; // ... and the most one unit can be given when the units retrieve unequal amounts
constexpr int kPrefillTiles = 2;  // row tiles per wavefront in the multi-tile MFMA kernel
constexpr int kPrefillWaves = 4;  // wavefronts per workgroup of that kernel (64 * kPrefillTiles * 4 = 128 query rows)
constexpr int kMlRows = 3;        // rows of 16 floats per attention partial besides O: max, normaliser, exact-weight sum

// Device-side view of one context: plain pointers into the caller's arena.
struct DeviceView {
    // geometry
    int L, Hq, Hkv, G, D, T, Tp, F, C, k, U;
    int esize;        // bytes per KV element
    int v_transposed; // 1: V pages stored [Tp/32][D][32] (MFMA path, Tp = T rounded up to 32); 0: [T][D]
    int chunks_per_page;
    int tier;         // MOSAIC_TIER_*
    int PU;           // pages per unit in k_store / v_store: F (HBM tier) or the cluster-cache capacity (host tier)
    int SN;           // host tier: frames in the staging ring
    // KV pages the attention kernels read, addressed through k_page()/v_page() below: two arrays,
    //   k_store [U][PU] K pages, v_store [U][PU] V pages.
    // HBM tier: page p = frame id (arrival order).  Host tier: page p = a slot of the unit's GPU
    //   cluster cache (slots are handed out frame by frame; a cluster's frames need not be adjacent).
    // A K page is [T][D]; a V page is [T][D] or, for the MFMA path, [Tp/32][D][32].
    char *k_store;
    char *v_store;
    size_t kpage, vpage;           // bytes of one K / V page
    size_t k_ustride, v_ustride;   // bytes between units, K array / V array
    // host tier: staging ring the ingest kernel writes (frame f at slot f % SN), and the
    // device-visible address of the pinned host pools the offload kernel writes
    char *stage_k, *stage_v;   // [SN][U][page]
    char *host_k, *host_v;     // pinned pools: [U][HP/SFh] slabs of [SFh K pages][SFh V pages]
    size_t h_ustride, h_bstride;
    int SFh;                   // frames per host slab
    int HP;                    // host pages per unit
    int *dest;                 // [U][SN] host page of each staged frame of the current batch
    // fetch work lists, written by the host into pinned memory and read by k_fetch over PCIe
    const int *moves;          // [U][F][2] (host page, cache page)
    const int *n_moves;        // [U]
    // clustering state (decision arithmetic in fp64)
    double *summ;     // [U][F][D]   per-frame key summaries
    double *r;        // [U][C][D]   representatives
    double *rnorm;    // [U][C]      |r_j|
    int *n;           // [U][C]      sizes in frames
    int *assign;      // [U][F]      frame -> cluster
    int *pos;         // [U][F]      rank of the frame among its cluster's members (ascending frame order)
    long long *sel_flag;   // [U]    (launch number << 32 | retrieved pages) of the unit's last selection published inside a launch (k_decode_layer)
    int *sync_err;    // [1]         set if a bounded in-kernel wait ever ran out
    int *lloyd_moved; // [U][3]      frames moved by the K-means rounds it-1, it, it+1 (mod 3): converged units skip the rest;
                      //             behind it [U][3] rows of 16 frames the rounds' bound tests left alive
    int *lloyd_live;  // [U][ceil(F/16)] those rows (index of the row's first frame / 16), in order of arrival
    int *lloyd_changed; // [U][C]    1 = a frame entered or left the cluster in the current round (its sums must be rebuilt)
    double *lloyd_delta; // [U][C]   chord by which the last update moved the representative's direction
    double *lloyd_ub, *lloyd_lb; // [U][F]  chord bounds of a frame: to its own representative from above, to any other from below
    // self-adaptive maintainer (paper Sec. VI); maint_mode 0 = off (the arrays are then empty)
    int maint_mode, c_init, split_iters, buf_max;
    int SC;           // score columns per unit: C + buf_max
    double tau_min, tau_max, tau_n0;
    double *var;      // [U][C]      running intra-cluster variance (Eq. 2 / Eq. 4)
    int *lazy;        // [U][C]      lazy-split flag
    int *resident;    // [U][C]      1 = selected by the unit's latest retrieval
    int *n_slots;     // [U]         cluster ids in use: [0, n_slots)
    int *buf_frame;   // [U][buf_max] buffered singletons: frame
    int *buf_owner;   // [U][buf_max]                       cluster they were assigned to
    int *n_buf;       // [U]
    long long *mt_cnt;// [U][4]      splits on insertion, deferred splits, buffered inserts, forced absorbs
    int *mt_mem, *mt_side;   // [U][F] scratch of Split
    double *mt_nrm;          // [U][F]
    // retrieval augmentation (paper Sec. V-C); both 0 = off
    int aug_reps, aug_window, nt_max;
    double *vsumm;    // [U][F][D]   per-frame value summaries (mean of the frame's T value vectors)
    double *rvsum;    // [U][C][D]   per-cluster sums of them (value representative = rvsum / n)
    float *rep_k, *rep_v;   // [U][C][D] fp32 pseudo-token tables: representative, value representative
    float *aug_o;     // [U][nt_max][16][D]  partial of the representatives' part, same form as part_o
    float *aug_ml;    // [U][nt_max][2][16]
    // nested visual-semantic hierarchy (paper Sec. V-B, V-C); P = 0: flat index
    int P, Cs, Dv, top_p;
    double *vemb;     // [F][Dv]     visual embeddings of the frames (the visual level's states)
    double *vr;       // [P][Dv]     visual centroids
    double *vrn;      // [P]         their norms
    int *vn;          // [P]         their sizes in frames
    int *part;        // [F]         frame -> visual partition (shared by all units)
    double *pr;       // [U][P][D]   partition representatives in the unit's key space
    double *prn;      // [U][P]
    int *pn;          // [U][P]
    double *pscores;  // [U][P]      first-stage scores of the latest retrieval
    int *pids;        // [U][top_p]  partitions it kept
    int *n_pids;      // [U]
    // latest selection per unit
    double *scores;   // [U][SC]
    int *ids;         // [U][k]
    int *n_ids;       // [U]
    int *sel_pages;   // [U][F]      frames of the selected clusters, gather order
    int *n_sel;       // [U]         number of selected frames
    int *tok_scratch; // [Hkv][F*T]  token-index expansion for the observer
    // attention partials: entry e = base_slot(unit)*NT + tile*S(unit) + split, see split_slot()
    float *part_o;    // [entries][16][D]
    float *part_ml;   // [entries][3][16]  running max (log2 domain), sum of the weights the value contraction
                      //                   used (bf16-rounded in the MFMA kernels), sum of the unrounded weights
    long long part_entries;
};

struct HostTier;   // host_tier.hip

struct Ctx {
    mosaic_config cfg;
    DeviceView dv;
    hipStream_t stream;
    int device;
    int W;               // warm-up frames
    int iters;
    int impl;            // MOSAIC_ATTEND_VALU | MOSAIC_ATTEND_MFMA
    long long n_frames;  // ingested so far (host-side count)
    std::vector<long long> sel_epoch; // per layer: epoch at which the selection was made
    std::vector<int> sel_tq;
    long long epoch;     // bumped by ingest and reset
    int launch_epoch;    // numbers the launches that publish a selection inside the kernel (never 0)
    long long rv_epoch;  // epoch the value representatives were last computed at
    mosaic_stats stats;
    std::string err;
    void *static_scratch; // device address, on this context's GPU, of the library's static partial buffer
    HostTier *host;      // non-null in the host tier
    // host tier: host-side views of the pinned arena
    char *h_k, *h_v;     // slab pools
    int *h_sel, *h_nsel; // page lists / counts staged for upload, [U][F] / [U]
    int *h_moves, *h_nmoves; // fetch work lists, [U][F][2] / [U]
    int *h_ids, *h_nids; // selections read back, [U][k] / [U]
    int *h_assign, *h_dest; // staged batch: assignments read back / slab positions, [U][SN]
    int *h_assign_full;      // maintainer: a unit's whole frame -> cluster map read back, [U][F]
    long long *h_cnt;        // ... its counters, [U][4]
    int *h_nbuf, *h_buf_frame, *h_buf_owner;   // ... its singleton buffer, [U] / [U][buf_max]
    int *h_resident;         // residency flags on their way to the device, [U][C]
    // ingest_overlap: the order-dependent part of batched ingest calls runs here, after `stored`;
    // `assigned` marks its end and the caller's stream waits for it before anything touches the index
    hipStream_t assign_stream;
    hipEvent_t stored, assigned;
    bool assign_pending;
    // profiling
    bool profile;
    std::vector<hipEvent_t> ev;      // pool of pairs, created by mosaic_profile_enable
    size_t ev_used;
    double prof_ms;                  // kernel time and launches folded out of the pool so far
    long long prof_n;
};

// ---- launchers (each checks its own launch; returns hipError_t) ----
hipError_t launch_store_summary(const DeviceView &dv, const void *k_in, const void *v_in,
                                int f0, int n_frames, hipStream_t s);
// pages, summary, assignment and Eq. 3 of one frame in one launch (HBM tier, maintainer off,
// C <= 128, frame f beyond the warm-up)
hipError_t launch_ingest_one(const DeviceView &dv, const void *k_in, const void *v_in, int f, hipStream_t s);
hipError_t launch_assign_update(const DeviceView &dv, int f0, int f1, hipStream_t s);
hipError_t launch_lloyd(const DeviceView &dv, int n_frames, int iters, bool seed_from_warmup,
                        hipStream_t s);
// nested hierarchy: embeddings of frames f0.. into the visual level's state array
hipError_t launch_visual_store(const DeviceView &dv, const float *e_in, int f0, int n_frames, hipStream_t s);
// visual level: initial P-means over the first W embeddings / greedy assignment of frames f0..f1-1
hipError_t launch_visual_lloyd(const DeviceView &dv, int W, int iters, hipStream_t s);
// (e_in: fp32 embeddings of frames f0..f1-1, which the kernel also files in the state array)
hipError_t launch_visual_assign(const DeviceView &dv, const float *e_in, int f0, int f1, hipStream_t s);
// per-unit partition representatives recomputed from the member lists (after a K-means run)
hipError_t launch_partition_reps(const DeviceView &dv, int n_frames, hipStream_t s);
// write_pages = false (host tier): only scores and ids; the page list comes from the host
hipError_t launch_retrieve(const DeviceView &dv, int u0, int n_units, const void *q, int Tq,
                           int n_frames, int score_mode, bool write_pages, hipStream_t s);
// deferred-split maintainer: singletons take part, residency and deferred splits follow the selection
hipError_t launch_retrieve_deferred(const DeviceView &dv, int u0, int n_units, const void *q, int Tq,
                                    int n_frames, int score_mode, hipStream_t s);
// host tier: copy staged frames f0..f0+n-1 of every unit to host page dest[u][f - f0]
hipError_t launch_offload(const DeviceView &dv, int f0, int n, hipStream_t s);
// host tier: move the pages listed in moves[u0..u0+n_units) from the pinned slabs into the cache
hipError_t launch_fetch(const DeviceView &dv, int u0, int n_units, int max_moves, hipStream_t s);
hipError_t launch_expand_tok_idx(const DeviceView &dv, int u0, int n_units, hipStream_t s);
// n_splits = average splits per unit chosen by the caller (B = n_units * n_splits split
// workgroups are shared out by split_slot); partial entries needed = B * NT
// ev0/ev1 (may be null) receive the kernel's own start/stop timestamps
hipError_t launch_attend_prefill(const DeviceView &dv, int u0, int n_units, const unsigned short *q, int Tq,
                                 int n_splits, hipStream_t s, hipEvent_t ev0, hipEvent_t ev1);
hipError_t launch_attend_valu(const DeviceView &dv, int u0, int n_units, const void *q, int Tq,
                              int n_splits, hipStream_t s, hipEvent_t ev0, hipEvent_t ev1);
// stream_kv: the decode-shape kernels load K/V with the non-temporal hint (stores far beyond the caches)
hipError_t launch_attend_mfma(const DeviceView &dv, int u0, int n_units, const void *q, int Tq,
                              int n_splits, bool stream_kv, hipStream_t s, hipEvent_t ev0, hipEvent_t ev1);
// uniform: every unit has exactly n_splits splits at slots unit * n_splits + split (fused decode step)
hipError_t launch_attend_combine(const DeviceView &dv, int u0, int n_units, int Tq, int n_splits,
                                 void *out, float *lse, hipStream_t s, bool uniform = false);
// selection + attention of one decode step of one layer in one launch with size-proportional splits: the
// first n_units workgroups select for one unit each and publish the result, all workgroups then share
// out the retrieved pages (one row tile, bf16, C <= 256).  epoch: a number no earlier launch on this
// context has used.  B = total workgroups (>= n_units)
hipError_t launch_decode_layer(const DeviceView &dv, int u0, int n_units, const void *q, int Tq, int B, int n_frames,
                               int score_mode, int epoch, bool stream_kv, hipStream_t s, hipEvent_t ev0, hipEvent_t ev1);
// selection + attention of one decode step in one launch (one row tile, bf16, C <= 256, uniform splits)
hipError_t launch_decode_fused(const DeviceView &dv, int u0, int n_units, const void *q, int Tq, int n_splits,
                               int n_frames, int score_mode, bool stream_kv, hipStream_t s, hipEvent_t ev0,
                               hipEvent_t ev1);
// retrieval augmentation: per-cluster value sums of all units (after the clustering changed); the
// attention partial over the representatives is computed by extra workgroups of the attention launches
hipError_t launch_value_reps(const DeviceView &dv, int n_frames, hipStream_t s);

// A kernel launch that carries a HIP start/stop event pair when one is given (the events receive the
// kernel's own begin and end timestamps) and is a plain launch otherwise, which a caller may also
// record into a HIP graph.
template <typename K, typename... A>
inline void launch_timed(K kern, dim3 grid, dim3 block, size_t lds, hipStream_t s, hipEvent_t ev0, hipEvent_t ev1,
                         A... args) {
    if (ev0 || ev1) hipExtLaunchKernelGGL(kern, grid, block, (unsigned)lds, s, ev0, ev1, 0, args...);
    else hipLaunchKernelGGL(kern, grid, block, (unsigned)lds, s, args...);
}

// ---- small device helpers ----
__device__ __forceinline__ const char *k_page(const DeviceView &dv, int u, int p) {
    return dv.k_store + (size_t)u * dv.k_ustride + (size_t)p * dv.kpage;
}
__device__ __forceinline__ const char *v_page(const DeviceView &dv, int u, int p) {
    return dv.v_store + (size_t)u * dv.v_ustride + (size_t)p * dv.vpage;
}
__device__ __forceinline__ float bf16_to_f32(unsigned short h) {
    return __uint_as_float(((unsigned int)h) << 16);
}
__device__ __forceinline__ unsigned short f32_to_bf16_rne(float f) {
    unsigned int u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (unsigned short)((u >> 16) | 0x40); // NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (unsigned short)(u >> 16);
}


// ---------------------------------------------------------------------------
// Reductions over the 16 lanes of a DPP row (lanes 16k .. 16k + 15) with data-parallel
// primitives instead of LDS permutes: a butterfly over the lane-index masks 8, 7, 3, 1
// (row_ror:8, row_half_mirror, quad_perm [3,2,1,0], quad_perm [1,0,3,2]), which span all
// 16 lanes.  Every step adds a lane's partner symmetrically, so all 16 lanes end with the
// same bits.  About 80 cycles for a double against about 500 with ds_bpermute.
// ---------------------------------------------------------------------------
template <int CTRL> __device__ __forceinline__ int dpp_i32(int x) {
    // bound_ctrl on: a source lane that is out of range or switched off reads as 0, which is also what the old value 0
    // would leave, and the compiler need not clear the destination first (two instructions fewer per 64-bit step)
    return __builtin_amdgcn_update_dpp(0, x, CTRL, 0xf, 0xf, true);
}
template <int CTRL> __device__ __forceinline__ double dpp_f64(double x) {
    const long long b = __double_as_longlong(x);
    const int lo = dpp_i32<CTRL>((int)b), hi = dpp_i32<CTRL>((int)(b >> 32));
    return __longlong_as_double(((long long)hi << 32) | (long long)(unsigned int)lo);
}
constexpr int kDppXor8 = 0x128, kDppXor7 = 0x141, kDppXor3 = 0x1B, kDppXor1 = 0xB1;
__device__ __forceinline__ double row16_sum(double x) {
    x += dpp_f64<kDppXor8>(x);
    x += dpp_f64<kDppXor7>(x);
    x += dpp_f64<kDppXor3>(x);
    x += dpp_f64<kDppXor1>(x);
    return x;
}
// Sum over the 64 lanes of a wavefront (all lanes active), the same bits in every lane: the four rows'
// sums are read from their first lanes and added in a fixed order.
__device__ __forceinline__ double wave64_sum(double x) {
    x = row16_sum(x);
    const long long b = __double_as_longlong(x);
    const int lo = (int)b, hi = (int)(b >> 32);
    double r[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int l = __builtin_amdgcn_readlane(lo, 16 * i), h = __builtin_amdgcn_readlane(hi, 16 * i);
        r[i] = __longlong_as_double(((long long)h << 32) | (long long)(unsigned int)l);
    }
    return (r[0] + r[1]) + (r[2] + r[3]);
}


// ---------------------------------------------------------------------------
// Load-balanced KV splits.  An attend launch has B split workgroups (per row
// block) for the n_units units of the call.  Units retrieve different numbers
// of tokens, so the splits are shared out in proportion to the selected page
// counts: unit i gets (n_sel_i > 0) + floor((B - n_units) * n_sel_i / total),
// capped at kMaxUnitSplits, contiguous workgroup ids, in unit order.  The attention
// kernels (by workgroup id) and the combine kernel (by unit) evaluate the same
// function of the same device-resident sizes, so they agree without any
// host round trip.  Every lane of the calling wavefront gets the result.
// ---------------------------------------------------------------------------
struct SplitSlot {
    int uc;      // unit within the call, -1: this workgroup has no work
    int split;   // split index within the unit
    int S;       // number of splits of the unit
    int base;    // first split slot of the unit (partials are indexed by slot)
    int n;       // the unit's retrieved size (n_sel), so that the caller need not load it again
};

// Agent-scope (write-through / cache-bypassing) accesses for values that one workgroup publishes and
// others of the SAME launch read: an ordinary store may sit in the writing XCD's L2 until the kernel ends.
// Workgroup barrier that orders LDS accesses only: does not wait for outstanding global loads and stores.
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}
__device__ __forceinline__ void st_agent(int *p, int v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ int ld_agent(const int *p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void st_agent(long long *p, long long v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ long long ld_agent(const long long *p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

template <bool BY_UNIT>
__device__ __forceinline__ SplitSlot split_slot(const int *n_sel_call, int n_units, int B, int key) {
    const int lane = threadIdx.x % 64;
    if (n_units <= 8) {
        // A layer's few units (the per-layer decode chain, where this sits at the head of two launches' dependent
        // chains): sizes, shares and offsets as wave-uniform scalars read from the first lanes, one 32-bit
        // division per lane where the product fits, no cross-lane scans.  Same shares as the general path below.
        const int ns = lane < n_units ? n_sel_call[lane] : 0;
        long long total = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) total += __builtin_amdgcn_readlane(ns, i);
        int want = 0;
        if (ns > 0) {
            const long long prod = (long long)(B - n_units) * ns;      // total >= ns > 0 here
            want = 1 + (prod < (1ll << 32) && total < (1ll << 32) ? (int)((unsigned int)prod / (unsigned int)total)
                                                                  : (int)(prod / total));
            want = min(want, kMaxUnitSplits);
        }
        SplitSlot r{-1, 0, 0, 0, 0};
        int run = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int w = __builtin_amdgcn_readlane(want, i);
            const bool hit = BY_UNIT ? (i == key) : (key >= run && key < run + w);
            if (hit && r.uc < 0 && i < n_units) {
                r.uc = i; r.S = w; r.base = run; r.split = BY_UNIT ? 0 : key - run;
                r.n = __builtin_amdgcn_readlane(ns, i);
            }
            run += w;
        }
        return r;
    }
    long long total = 0;
    for (int i = lane; i < n_units; i += 64) total += n_sel_call[i];
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) total += __shfl_xor(total, o, 64);
    SplitSlot r{-1, 0, 0, 0, 0};
    int run = 0;
    for (int i0 = 0; i0 < n_units; i0 += 64) {
        const int i = i0 + lane;
        const int ns = i < n_units ? n_sel_call[i] : 0;
        int want = 0;
        if (i < n_units && ns > 0) {
            want = 1 + (int)(((long long)(B - n_units) * ns) / (total > 0 ? total : 1));
            want = min(want, kMaxUnitSplits);
        }
        int incl = want;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int t = __shfl_up(incl, o, 64);
            if (lane >= o) incl += t;
        }
        const int excl = run + incl - want;
        const bool hit = BY_UNIT ? (i == key) : (key >= excl && key < excl + want);
        const unsigned long long mask = __ballot(hit);
        if (mask) {
            const int src = __ffsll((long long)mask) - 1;
            r.uc = i0 + src;
            r.S = __shfl(want, src, 64);
            r.base = __shfl(excl, src, 64);
            r.n = __shfl(ns, src, 64);
            r.split = BY_UNIT ? 0 : key - r.base;
        }
        run += __shfl(incl, 63, 64);
    }
    return r;
}

} // namespace mosaic
