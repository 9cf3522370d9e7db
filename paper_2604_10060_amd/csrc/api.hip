// C ABI of libmosaic: configuration checks, arena carving, host-side sequencing
// of the kernels.  All frame counting is done on the host from call arguments,
// so no call on the hot path waits for the device.
#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>

#include "mosaic_internal.h"
#include "host_tier.h"

using namespace mosaic;

struct mosaic_ctx : public Ctx {};

namespace {

thread_local std::string g_create_err = "";

size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

// Attention partials for callers that cannot allocate (mosaic_attend_static): one buffer per GPU,
// in the library's image, shared by every handle on that GPU.  In host code the array's name is
// only a handle for hipGetSymbolAddress; the address kernels are given is looked up once per device.
constexpr size_t kStaticScratchBytes = 16u << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void *g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on `device`, which must be the current device.
hipError_t static_scratch(int device, void **out) {
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[device]) {
        void *ptr = nullptr;
        const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!ptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[device] = ptr;
    }
    *out = g_scratch_ptr[device];
    return hipSuccess;
}

int fail(mosaic_ctx *ctx, int code, const std::string &msg) {
    if (ctx) ctx->err = msg; else g_create_err = msg;
    return code;
}
int fail_hip(mosaic_ctx *ctx, hipError_t e, const char *what) {
    return fail(ctx, MOSAIC_EHIP, std::string(what) + ": " + hipGetErrorString(e));
}

struct Layout {
    size_t k_store, v_store, summ, r, rnorm, n, assign, pos, lloyd_moved, lloyd_delta, lloyd_ub, lloyd_lb, lloyd_live, sel_flag, sync_err, scores, ids, n_ids, sel_pages, n_sel,
        tok_scratch, part_o, part_ml, stage_k, stage_v, dest, var, lazy, resident, n_slots, buf_frame,
        buf_owner, n_buf, mt_cnt, mt_mem, mt_side, mt_nrm, vsumm, rvsum, rep_k, rep_v, aug_o, aug_ml,
        vemb, vr, vrn, vn, part, pr, prn, pn, pscores, pids, n_pids, total;
    size_t host_k, host_v, host_sel, host_nsel, host_ids, host_nids, host_moves, host_nmoves, host_assign, host_dest,
        host_assign_full, host_cnt, host_nbuf, host_buf_frame, host_buf_owner, host_resident, host_total;   // offsets into the pinned host arena
    long long part_entries;
    int Tp, impl, v_transposed;
    int nt_max;
    int c_init, split_iters, buf_max, W;   // maintainer (c_init = C, buf_max = 0 when off); warm-up frames
    // host tier geometry
    int SF, slabs_per_unit, HP, PU, SN, max_clusters;
    size_t kpage, vpage;
};

// resolved defaults of the maintainer fields and of the warm-up length
int init_clusters_of(const mosaic_config &c) {
    if (c.maint_mode == MOSAIC_MAINT_OFF) return c.n_clusters;
    return c.init_clusters > 0 ? c.init_clusters : std::max(1, c.n_clusters / 2);
}
int buffer_max_of(const mosaic_config &c) {
    if (c.maint_mode != MOSAIC_MAINT_DEFERRED) return 0;
    return c.buffer_max > 0 ? c.buffer_max : 32;
}
int top_partitions_of(const mosaic_config &c) {
    if (c.n_partitions <= 0) return 0;
    return c.top_partitions > 0 ? c.top_partitions : std::max(1, c.n_partitions / 4);
}
int warmup_of(const mosaic_config &c) {
    return c.warmup_frames > 0 ? c.warmup_frames : 2 * init_clusters_of(c);
}

int check_config(const mosaic_config *c, std::string &why) {
    if (!c) { why = "config is NULL"; return MOSAIC_EINVAL; }
    if (c->n_layers < 1 || c->n_kv_heads < 1 || c->n_q_heads < 1) { why = "layer/head counts must be positive"; return MOSAIC_EINVAL; }
    if (c->n_q_heads % c->n_kv_heads) { why = "n_q_heads must be a multiple of n_kv_heads"; return MOSAIC_EINVAL; }
    if (c->head_dim != 64 && c->head_dim != 128) { why = "head_dim must be 64 or 128"; return MOSAIC_EINVAL; }
    if (c->tokens_per_frame < 1 || c->max_frames < 1) { why = "tokens_per_frame and max_frames must be positive"; return MOSAIC_EINVAL; }
    if (c->n_clusters < 1 || c->n_clusters > 1024) { why = "n_clusters must be in 1..1024"; return MOSAIC_EINVAL; }
    if (c->top_k < 1 || c->top_k > c->n_clusters) { why = "top_k must be in 1..n_clusters"; return MOSAIC_EINVAL; }
    if (c->kv_dtype != MOSAIC_FP32 && c->kv_dtype != MOSAIC_BF16) { why = "kv_dtype must be MOSAIC_FP32 or MOSAIC_BF16"; return MOSAIC_EINVAL; }
    if (c->warmup_frames < 0 || c->lloyd_iters < 0 || c->recluster_every < 0 || c->max_q_tokens < 0) { why = "negative count"; return MOSAIC_EINVAL; }
    if (c->maint_mode < MOSAIC_MAINT_OFF || c->maint_mode > MOSAIC_MAINT_DEFERRED) { why = "maint_mode out of range"; return MOSAIC_EINVAL; }
    if (c->maint_mode != MOSAIC_MAINT_OFF) {
        if (c->recluster_every != 0) { why = "the maintainer and periodic re-clustering exclude each other"; return MOSAIC_EINVAL; }
        if (c->init_clusters < 0 || c->init_clusters > c->n_clusters) { why = "init_clusters must be in 0..n_clusters"; return MOSAIC_EINVAL; }
        if (c->split_iters < 0 || c->buffer_max < 0) { why = "negative maintainer count"; return MOSAIC_EINVAL; }
        if (!(c->tau_n0 > 0.0)) { why = "tau_n0 must be positive"; return MOSAIC_EINVAL; }
        if (!(c->tau_min == c->tau_min) || !(c->tau_max == c->tau_max)) { why = "tau_min / tau_max is NaN"; return MOSAIC_EINVAL; }
        if (c->n_clusters + buffer_max_of(*c) > 1024) { why = "n_clusters + buffer_max must not exceed 1024"; return MOSAIC_EINVAL; }
    }
    if (c->prefetch_top_k < 0 || c->prefetch_top_k > c->top_k) { why = "prefetch_top_k must be in 0..top_k"; return MOSAIC_EINVAL; }
    if (c->aug_global_reps < 0 || c->aug_global_reps > 1 || c->aug_window_frames < 0) { why = "aug_global_reps must be 0 or 1, aug_window_frames >= 0"; return MOSAIC_EINVAL; }
    if (c->aug_window_frames > 1024) { why = "aug_window_frames must not exceed 1024"; return MOSAIC_EINVAL; }
    if (c->aug_global_reps || c->aug_window_frames) {
        if (c->tier != MOSAIC_TIER_HBM) { why = "retrieval augmentation is available in the HBM tier only"; return MOSAIC_EINVAL; }
        if (c->maint_mode == MOSAIC_MAINT_DEFERRED) { why = "retrieval augmentation is not available with MOSAIC_MAINT_DEFERRED"; return MOSAIC_EINVAL; }
    }
    if (c->n_partitions < 0 || c->n_partitions > 64) { why = "n_partitions must be in 0..64"; return MOSAIC_EINVAL; }
    if (c->n_partitions > 0) {
        if (c->tier != MOSAIC_TIER_HBM) { why = "the nested hierarchy is available in the HBM tier only"; return MOSAIC_EINVAL; }
        if (c->maint_mode != MOSAIC_MAINT_OFF || c->recluster_every != 0) { why = "the nested hierarchy excludes the maintainer and periodic re-clustering"; return MOSAIC_EINVAL; }
        if (c->aug_global_reps || c->aug_window_frames) { why = "the nested hierarchy is not combined with retrieval augmentation"; return MOSAIC_EINVAL; }
        if (c->n_clusters % c->n_partitions) { why = "n_clusters must be a multiple of n_partitions"; return MOSAIC_EINVAL; }
        if (c->visual_dim < 1 || c->visual_dim > 4096) { why = "visual_dim must be in 1..4096"; return MOSAIC_EINVAL; }
        if (c->top_partitions < 0 || c->top_partitions > c->n_partitions) { why = "top_partitions must be in 0..n_partitions"; return MOSAIC_EINVAL; }
    }
    const int W = warmup_of(*c);
    if (W < init_clusters_of(*c)) { why = "warmup_frames must be at least the number of initial clusters (one seed per cluster)"; return MOSAIC_EINVAL; }
    if (c->score_mode != 0 && c->score_mode != 1) { why = "score_mode must be 0 or 1"; return MOSAIC_EINVAL; }
    if (c->attend_impl < MOSAIC_ATTEND_AUTO || c->attend_impl > MOSAIC_ATTEND_MFMA) { why = "attend_impl out of range"; return MOSAIC_EINVAL; }
    if (c->attend_impl == MOSAIC_ATTEND_MFMA && c->kv_dtype != MOSAIC_BF16) { why = "the MFMA attention kernel needs bf16 KV"; return MOSAIC_EINVAL; }
    if ((long long)c->max_frames * c->tokens_per_frame > 0x7fffffffLL) { why = "max_frames * tokens_per_frame must fit in int32"; return MOSAIC_EINVAL; }
    if (c->decode_fused_max_mib < -2) { why = "decode_fused_max_mib must be >= -2"; return MOSAIC_EINVAL; }
    if (c->ingest_overlap != 0 && c->ingest_overlap != 1) { why = "ingest_overlap must be 0 or 1"; return MOSAIC_EINVAL; }
    if (c->tier != MOSAIC_TIER_HBM && c->tier != MOSAIC_TIER_HOST) { why = "tier must be MOSAIC_TIER_HBM or MOSAIC_TIER_HOST"; return MOSAIC_EINVAL; }
    if (c->tier == MOSAIC_TIER_HOST) {
        if (c->recluster_every != 0) { why = "re-clustering is not available in the host tier (pages would have to move between slabs)"; return MOSAIC_EINVAL; }
        if (c->slab_frames < 0 || c->cache_pages_per_unit < 0) { why = "negative host-tier size"; return MOSAIC_EINVAL; }
        if (c->cache_fraction < 0.f || c->cache_fraction > 1.f) { why = "cache_fraction must be in 0..1"; return MOSAIC_EINVAL; }
    }
    return MOSAIC_OK;
}

Layout make_layout(const mosaic_config &c) {
    Layout L{};
    const size_t U = (size_t)c.n_layers * c.n_kv_heads, F = c.max_frames, T = c.tokens_per_frame,
                 D = c.head_dim, C = c.n_clusters, k = c.top_k;
    const size_t e = c.kv_dtype == MOSAIC_FP32 ? 4 : 2;
    L.impl = c.attend_impl == MOSAIC_ATTEND_AUTO
                 ? (c.kv_dtype == MOSAIC_BF16 ? MOSAIC_ATTEND_MFMA : MOSAIC_ATTEND_VALU)
                 : c.attend_impl;
    L.v_transposed = L.impl == MOSAIC_ATTEND_MFMA;
    L.Tp = (int)((T + kChunk - 1) / kChunk * kChunk);   // value pages are padded to whole 32-token chunks
    const int G = c.n_q_heads / c.n_kv_heads;
    const int maxq = c.max_q_tokens > 0 ? c.max_q_tokens : 256;
    const long long nt_max = ((long long)maxq * G + kRowTile - 1) / kRowTile;
    L.part_entries = std::max<long long>(4096, (long long)U * nt_max * 2);
    L.nt_max = (int)nt_max;
    L.kpage = T * D * e;
    L.vpage = D * (L.v_transposed ? (size_t)L.Tp : T) * e;
    const bool host = c.tier == MOSAIC_TIER_HOST;
    L.PU = (int)F; L.SN = 1;
    if (host) {
        const int W = warmup_of(c);
        L.SF = c.slab_frames > 0 ? c.slab_frames : 8;
        L.slabs_per_unit = (int)((F + L.SF - 1) / L.SF + C);
        L.HP = L.slabs_per_unit * L.SF;
        const float frac = c.cache_fraction > 0.f ? c.cache_fraction : 0.10f;
        L.max_clusters = std::max<int>((int)k, (int)(frac * (float)C));
        // default capacity: three times the average footprint of the clusters that may be resident
        const double share = std::max((double)frac, (double)k / (double)C);
        const long long cp = c.cache_pages_per_unit > 0
                                 ? std::min<long long>(c.cache_pages_per_unit, (long long)F)
                                 : std::min<long long>((long long)(3.0 * share * (double)F) + (long long)k, (long long)F);
        L.PU = (int)std::max<long long>(cp, 1);
        L.SN = std::max(W, 128);                // staging ring: the warm-up, or two batches (one being offloaded, one being staged)
    }
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
    L.k_store = take(U * (size_t)L.PU * L.kpage);     // (host tier: PU = page slots of the cluster cache)
    L.v_store = take(U * (size_t)L.PU * L.vpage);
    L.stage_k = take(host ? (size_t)L.SN * U * L.kpage : 0);
    L.stage_v = take(host ? (size_t)L.SN * U * L.vpage : 0);
    L.dest = take(host ? 2 * U * (size_t)L.SN * 4 : 0);      // two slab tables, used in turn
    L.summ = take(U * F * D * 8);
    L.r = take(U * C * D * 8);
    L.rnorm = take(U * C * 8);
    L.n = take(U * C * 4);
    L.assign = take(U * F * 4);
    L.pos = take(U * F * 4);
    L.lloyd_moved = take(U * 6 * 4 + U * C * 4);      // + the live-row counters and the clusters' changed flags
    L.lloyd_live = take(U * ((F + 15) / 16) * 4);
    L.lloyd_delta = take(U * C * 8);
    L.lloyd_ub = take(U * F * 8);
    L.lloyd_lb = take(U * F * 8);
    L.sel_flag = take(U * 8);
    L.sync_err = take(4);
    L.c_init = init_clusters_of(c); L.buf_max = buffer_max_of(c); L.W = warmup_of(c);
    L.split_iters = c.split_iters > 0 ? c.split_iters : 4;
    const bool mt = c.maint_mode != MOSAIC_MAINT_OFF;
    const size_t B = (size_t)L.buf_max;
    L.var = take(mt ? U * C * 8 : 0);
    L.lazy = take(mt ? U * C * 4 : 0);
    L.resident = take(mt ? U * C * 4 : 0);
    L.n_slots = take(mt ? U * 4 : 0);
    L.buf_frame = take(mt ? U * B * 4 : 0);
    L.buf_owner = take(mt ? U * B * 4 : 0);
    L.n_buf = take(mt ? U * 4 : 0);
    L.mt_cnt = take(mt ? U * 4 * 8 : 0);
    L.mt_mem = take(mt ? U * F * 4 : 0);
    L.mt_side = take(mt ? U * F * 4 : 0);
    L.mt_nrm = take(mt ? U * F * 8 : 0);
    L.vsumm = take(c.aug_global_reps ? U * F * D * 8 : 0);
    L.rvsum = take(c.aug_global_reps ? U * C * D * 8 : 0);
    L.rep_k = take(c.aug_global_reps ? U * C * D * 4 : 0);
    L.rep_v = take(c.aug_global_reps ? U * C * D * 4 : 0);
    L.aug_o = take(c.aug_global_reps ? U * (size_t)nt_max * kRowTile * D * 4 : 0);
    L.aug_ml = take(c.aug_global_reps ? U * (size_t)nt_max * 2 * kRowTile * 4 : 0);
    const size_t P = (size_t)c.n_partitions, Dv = (size_t)c.visual_dim, tp = (size_t)top_partitions_of(c);
    L.vemb = take(P ? F * Dv * 8 : 0);
    L.vr = take(P * Dv * 8);
    L.vrn = take(P * 8);
    L.vn = take(P * 4);
    L.part = take(P ? F * 4 : 0);
    L.pr = take(U * P * D * 8);
    L.prn = take(U * P * 8);
    L.pn = take(U * P * 4);
    L.pscores = take(U * P * 8);
    L.pids = take(U * tp * 4);
    L.n_pids = take(P ? U * 4 : 0);
    L.scores = take(U * (C + B) * 8);
    L.ids = take(U * k * 4);
    L.n_ids = take(U * 4);
    L.sel_pages = take(U * F * 4);
    L.n_sel = take(U * 4);
    L.tok_scratch = take((size_t)c.n_kv_heads * F * T * 4);
    L.part_o = take((size_t)L.part_entries * kRowTile * D * 4);
    L.part_ml = take((size_t)L.part_entries * kMlRows * kRowTile * 4);
    L.total = off;
    L.host_k = 0;
    L.host_v = host ? (size_t)L.SF * L.kpage : 0;     // inside the first slab: [SF K pages][SF V pages]
    if (host) {
        size_t ho = align_up(U * (size_t)L.HP * (L.kpage + L.vpage));
        auto htake = [&](size_t bytes) { size_t o = ho; ho = align_up(ho + bytes); return o; };
        L.host_sel = htake(U * F * 4);      // page lists on their way to the device
        L.host_nsel = htake(U * 4);
        L.host_ids = htake(U * k * 4);      // selections on their way back
        L.host_nids = htake(U * 4);
        L.host_moves = htake(U * F * 2 * 4);   // fetch work lists, read by the fetch kernel
        L.host_nmoves = htake(U * 4);
        L.host_assign = htake(U * (size_t)L.SN * 4);  // assignments of a staged batch on their way back
        L.host_dest = htake(2 * U * (size_t)L.SN * 4); // their slab positions on their way to the device (two tables)
        // maintainer on the host tier: what the host reads back to follow splits, and the residency flags it sends
        L.host_assign_full = htake(mt ? U * F * 4 : 0);
        L.host_cnt = htake(mt ? U * 4 * 8 : 0);
        L.host_nbuf = htake(mt ? U * 4 : 0);
        L.host_buf_frame = htake(mt ? U * B * 4 : 0);
        L.host_buf_owner = htake(mt ? U * B * 4 : 0);
        L.host_resident = htake(mt ? U * C * 4 : 0);
        L.host_total = ho;
    } else {
        L.host_total = 0;
    }
    return L;
}

// KV splits for one attend call, bounded by the partial-buffer capacity.
int choose_splits(const mosaic_ctx *ctx, int n_units, int Tq, long long part_entries) {
    const DeviceView &dv = ctx->dv;
    const long long NT = ((long long)Tq * dv.G + kRowTile - 1) / kRowTile;
    const bool mfma = ctx->impl == MOSAIC_ATTEND_MFMA;
    constexpr int pw = kPrefillWaves;
    const long long row_blocks = NT == 1 ? 1 : (mfma ? (NT + pw * kPrefillTiles - 1) / (pw * kPrefillTiles) : NT);
    const long long est_pages = std::max<long long>(1, (ctx->n_frames * dv.k + dv.C - 1) / dv.C);
    const long long est_chunks = est_pages * dv.chunks_per_page;
    long long s;
    if (NT > 1 && mfma) {
        // MFMA-bound multi-tile launches: every split writes 16 x D partial rows per
        // tile that the combine kernel reads back, so only as many splits as fill the
        // chip's two resident workgroups per CU once (more splits raise the attention
        // kernel's rate a little but cost more in the combine; measured on config 4),
        // each with at least 8 chunks; a multiple of 8 keeps the workgroups that share
        // a (unit, split) on one XCD (workgroup ids congruent mod 8)
        s = (2048 / pw + n_units * row_blocks - 1) / (n_units * row_blocks);
        s = std::min(s, std::max<long long>(1, est_chunks / 8));
        if (s >= 8) s = s / 8 * 8;
    } else {
        // bandwidth/latency-bound: cover the chip several times over (7 x 256 workgroups:
        // measured on the all-layers launch of config 2, 1568-1792 workgroups are 3 % faster
        // than 2128), at least 4 chunks (one per wavefront) per workgroup
        s = (1792 + n_units * row_blocks - 1) / (n_units * row_blocks);
        s = std::min(s, std::max<long long>(1, est_chunks / 4));
    }
    s = std::min<long long>(s, kMaxSplits);
    s = std::min(s, std::max<long long>(1, part_entries / (n_units * NT)));
    return (int)std::max<long long>(1, s);
}

__global__ __launch_bounds__(256) void k_calibration_copy(uint4 *dst, const uint4 *src, size_t n16) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16;
         i += (size_t)gridDim.x * blockDim.x)
        dst[i] = src[i];
}

} // namespace

extern "C" {

int32_t mosaic_calibration_copy(void *dst_dev, const void *src_dev, size_t bytes, void *stream) {
    if (!dst_dev || !src_dev || bytes % 16 || ((uintptr_t)dst_dev | (uintptr_t)src_dev) % 16)
        return fail(nullptr, MOSAIC_EINVAL, "calibration copy needs 16-byte aligned pointers and size");
    if (bytes == 0) return MOSAIC_OK;
    k_calibration_copy<<<2048, 256, 0, (hipStream_t)stream>>>((uint4 *)dst_dev, (const uint4 *)src_dev, bytes / 16);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail_hip(nullptr, e, "calibration copy launch");
    return MOSAIC_OK;
}

int32_t mosaic_host_alloc(size_t bytes, void **out) {
    if (!out || bytes == 0) return fail(nullptr, MOSAIC_EINVAL, "mosaic_host_alloc needs a size and an output pointer");
    void *p = nullptr;
    const hipError_t e = hipHostMalloc(&p, bytes, hipHostMallocDefault);
    if (e != hipSuccess || !p) {
        (void)hipGetLastError();             // the refusal must not surface in a later call
        *out = nullptr;
        return fail(nullptr, MOSAIC_ENOMEM, std::string("hipHostMalloc refused the pinned allocation: ") + hipGetErrorString(e));
    }
    *out = p;
    return MOSAIC_OK;
}

int32_t mosaic_host_free(void *p) {
    if (!p) return MOSAIC_OK;
    const hipError_t e = hipHostFree(p);
    return e == hipSuccess ? MOSAIC_OK : fail_hip(nullptr, e, "hipHostFree");
}

int32_t mosaic_workspace_size(const mosaic_config *cfg, size_t *dev_bytes, size_t *host_bytes) {
    std::string why;
    int rc = check_config(cfg, why);
    if (rc != MOSAIC_OK) return fail(nullptr, rc, why);
    if (!dev_bytes) return fail(nullptr, MOSAIC_EINVAL, "dev_bytes is NULL");
    const Layout L = make_layout(*cfg);
    *dev_bytes = L.total;
    if (host_bytes) *host_bytes = L.host_total;
    return MOSAIC_OK;
}

static hipError_t clear_maintainer(mosaic_ctx *ctx);

int32_t mosaic_create(const mosaic_config *cfg, mosaic_ctx **out) {
    std::string why;
    int rc = check_config(cfg, why);
    if (rc != MOSAIC_OK) return fail(nullptr, rc, why);
    if (!out) return fail(nullptr, MOSAIC_EINVAL, "out is NULL");
    const Layout L = make_layout(*cfg);
    if (!cfg->dev_arena) return fail(nullptr, MOSAIC_EINVAL, "dev_arena is NULL");
    if ((uintptr_t)cfg->dev_arena % 256) return fail(nullptr, MOSAIC_EINVAL, "dev_arena must be 256-byte aligned");
    if (cfg->dev_arena_bytes < L.total) {
        char b[128];
        snprintf(b, sizeof b, "dev_arena has %zu bytes, %zu needed", cfg->dev_arena_bytes, L.total);
        return fail(nullptr, MOSAIC_ENOMEM, b);
    }
    mosaic_ctx *ctx = new (std::nothrow) mosaic_ctx();
    if (!ctx) return fail(nullptr, MOSAIC_ENOMEM, "host allocation failed");
    ctx->cfg = *cfg;
    hipError_t e = hipGetDevice(&ctx->device);
    if (e != hipSuccess) { delete ctx; return fail_hip(nullptr, e, "hipGetDevice"); }
    ctx->static_scratch = nullptr;
    if ((e = static_scratch(ctx->device, &ctx->static_scratch)) != hipSuccess) {
        delete ctx;
        return fail_hip(nullptr, e, "hipGetSymbolAddress(static attention scratch)");
    }
    ctx->stream = (hipStream_t)cfg->stream;
    ctx->assign_stream = nullptr; ctx->stored = nullptr; ctx->assigned = nullptr; ctx->assign_pending = false;
    if (cfg->ingest_overlap == 1 && cfg->tier == MOSAIC_TIER_HBM && cfg->n_partitions == 0) {
        if ((e = hipStreamCreateWithFlags(&ctx->assign_stream, hipStreamNonBlocking)) != hipSuccess ||
            (e = hipEventCreateWithFlags(&ctx->stored, hipEventDisableTiming)) != hipSuccess ||
            (e = hipEventCreateWithFlags(&ctx->assigned, hipEventDisableTiming)) != hipSuccess) {
            if (ctx->assign_stream) (void)hipStreamDestroy(ctx->assign_stream);
            if (ctx->stored) (void)hipEventDestroy(ctx->stored);
            delete ctx;
            return fail_hip(nullptr, e, "stream / events of the overlapped ingest");
        }
    }
    ctx->W = L.W;
    ctx->iters = cfg->lloyd_iters > 0 ? cfg->lloyd_iters : 8;
    ctx->impl = L.impl;
    ctx->n_frames = 0;
    ctx->epoch = 1;
    ctx->sel_epoch.assign(cfg->n_layers, 0);
    ctx->sel_tq.assign(cfg->n_layers, 0);
    ctx->profile = false;
    ctx->ev_used = 0;
    ctx->prof_ms = 0.0; ctx->prof_n = 0;
    memset(&ctx->stats, 0, sizeof ctx->stats);
    ctx->stats.attend_impl = L.impl;
    DeviceView &dv = ctx->dv;
    dv.L = cfg->n_layers; dv.Hq = cfg->n_q_heads; dv.Hkv = cfg->n_kv_heads;
    dv.G = dv.Hq / dv.Hkv; dv.D = cfg->head_dim; dv.T = cfg->tokens_per_frame; dv.Tp = L.Tp;
    dv.F = cfg->max_frames; dv.C = cfg->n_clusters; dv.k = cfg->top_k; dv.U = dv.L * dv.Hkv;
    dv.esize = cfg->kv_dtype == MOSAIC_FP32 ? 4 : 2;
    dv.v_transposed = L.v_transposed;
    dv.chunks_per_page = (dv.T + kChunk - 1) / kChunk;
    char *base = (char *)cfg->dev_arena;
    dv.k_store = base + L.k_store; dv.v_store = base + L.v_store;
    dv.summ = (double *)(base + L.summ); dv.r = (double *)(base + L.r);
    dv.rnorm = (double *)(base + L.rnorm); dv.n = (int *)(base + L.n);
    dv.assign = (int *)(base + L.assign); dv.pos = (int *)(base + L.pos);
    dv.lloyd_moved = (int *)(base + L.lloyd_moved); dv.lloyd_changed = dv.lloyd_moved + (size_t)dv.U * 6;
    dv.lloyd_live = (int *)(base + L.lloyd_live);
    dv.lloyd_delta = (double *)(base + L.lloyd_delta);
    dv.lloyd_ub = (double *)(base + L.lloyd_ub); dv.lloyd_lb = (double *)(base + L.lloyd_lb);
    dv.sel_flag = (long long *)(base + L.sel_flag); dv.sync_err = (int *)(base + L.sync_err);
    ctx->launch_epoch = 0;
    dv.scores = (double *)(base + L.scores); dv.ids = (int *)(base + L.ids);
    dv.aug_reps = cfg->aug_global_reps; dv.aug_window = cfg->aug_window_frames; dv.nt_max = L.nt_max;
    dv.vsumm = cfg->aug_global_reps ? (double *)(base + L.vsumm) : nullptr;
    dv.rvsum = (double *)(base + L.rvsum);
    dv.rep_k = (float *)(base + L.rep_k); dv.rep_v = (float *)(base + L.rep_v);
    dv.aug_o = (float *)(base + L.aug_o); dv.aug_ml = (float *)(base + L.aug_ml);
    ctx->rv_epoch = -1;
    dv.maint_mode = cfg->maint_mode; dv.c_init = L.c_init; dv.split_iters = L.split_iters;
    dv.buf_max = L.buf_max; dv.SC = dv.C + L.buf_max;
    dv.tau_min = cfg->tau_min; dv.tau_max = cfg->tau_max; dv.tau_n0 = cfg->tau_n0;
    dv.var = (double *)(base + L.var); dv.lazy = (int *)(base + L.lazy);
    dv.resident = (int *)(base + L.resident); dv.n_slots = (int *)(base + L.n_slots);
    dv.buf_frame = (int *)(base + L.buf_frame); dv.buf_owner = (int *)(base + L.buf_owner);
    dv.n_buf = (int *)(base + L.n_buf); dv.mt_cnt = (long long *)(base + L.mt_cnt);
    dv.mt_mem = (int *)(base + L.mt_mem); dv.mt_side = (int *)(base + L.mt_side);
    dv.mt_nrm = (double *)(base + L.mt_nrm);
    dv.P = cfg->n_partitions; dv.Cs = dv.P > 0 ? dv.C / dv.P : 0; dv.Dv = cfg->visual_dim;
    dv.top_p = top_partitions_of(*cfg);
    dv.vemb = (double *)(base + L.vemb); dv.vr = (double *)(base + L.vr); dv.vrn = (double *)(base + L.vrn);
    dv.vn = (int *)(base + L.vn); dv.part = (int *)(base + L.part);
    dv.pr = (double *)(base + L.pr); dv.prn = (double *)(base + L.prn); dv.pn = (int *)(base + L.pn);
    dv.pscores = (double *)(base + L.pscores); dv.pids = (int *)(base + L.pids);
    dv.n_pids = (int *)(base + L.n_pids);
    dv.n_ids = (int *)(base + L.n_ids); dv.sel_pages = (int *)(base + L.sel_pages);
    dv.n_sel = (int *)(base + L.n_sel); dv.tok_scratch = (int *)(base + L.tok_scratch);
    dv.part_o = (float *)(base + L.part_o); dv.part_ml = (float *)(base + L.part_ml);
    dv.part_entries = L.part_entries;
    dv.tier = cfg->tier; dv.PU = L.PU; dv.SN = L.SN; dv.HP = L.HP;
    dv.kpage = L.kpage; dv.vpage = L.vpage;
    dv.k_ustride = (size_t)L.PU * L.kpage;
    dv.v_ustride = (size_t)L.PU * L.vpage;
    dv.SFh = 1; dv.h_bstride = dv.h_ustride = 0;
    if (cfg->tier == MOSAIC_TIER_HOST) {
        dv.SFh = L.SF;
        dv.h_bstride = (size_t)L.SF * (L.kpage + L.vpage);
        dv.h_ustride = (size_t)L.slabs_per_unit * dv.h_bstride;
    }
    dv.stage_k = base + L.stage_k; dv.stage_v = base + L.stage_v; dv.dest = (int *)(base + L.dest);
    dv.host_k = dv.host_v = nullptr;
    ctx->host = nullptr;
    if (cfg->tier == MOSAIC_TIER_HOST) {
        auto bail = [&](int code, const std::string &msg) {
            (void)mosaic_destroy(ctx);             // also ends the streams and events made so far
            return fail(nullptr, code, msg);
        };
        if (!cfg->host_arena) return bail(MOSAIC_EINVAL, "host_arena is NULL");
        if ((uintptr_t)cfg->host_arena % 256) return bail(MOSAIC_EINVAL, "host_arena must be 256-byte aligned");
        if (cfg->host_arena_bytes < L.host_total) {
            char b[128];
            snprintf(b, sizeof b, "host_arena has %zu bytes, %zu needed", cfg->host_arena_bytes, L.host_total);
            return bail(MOSAIC_ENOMEM, b);
        }
        void *dptr = nullptr;
        e = hipHostGetDevicePointer(&dptr, cfg->host_arena, 0);
        if (e != hipSuccess || !dptr)
            return bail(MOSAIC_EINVAL, "host_arena must be pinned, device-mapped host memory (hipHostMalloc)");
        dv.host_k = (char *)dptr + L.host_k;
        dv.host_v = (char *)dptr + L.host_v;
        ctx->h_sel = (int *)((char *)cfg->host_arena + L.host_sel);
        ctx->h_nsel = (int *)((char *)cfg->host_arena + L.host_nsel);
        ctx->h_ids = (int *)((char *)cfg->host_arena + L.host_ids);
        ctx->h_nids = (int *)((char *)cfg->host_arena + L.host_nids);
        ctx->h_k = (char *)cfg->host_arena + L.host_k;
        ctx->h_v = (char *)cfg->host_arena + L.host_v;
        ctx->h_moves = (int *)((char *)cfg->host_arena + L.host_moves);
        ctx->h_nmoves = (int *)((char *)cfg->host_arena + L.host_nmoves);
        ctx->h_assign = (int *)((char *)cfg->host_arena + L.host_assign);
        ctx->h_dest = (int *)((char *)cfg->host_arena + L.host_dest);
        ctx->h_assign_full = (int *)((char *)cfg->host_arena + L.host_assign_full);
        ctx->h_cnt = (long long *)((char *)cfg->host_arena + L.host_cnt);
        ctx->h_nbuf = (int *)((char *)cfg->host_arena + L.host_nbuf);
        ctx->h_buf_frame = (int *)((char *)cfg->host_arena + L.host_buf_frame);
        ctx->h_buf_owner = (int *)((char *)cfg->host_arena + L.host_buf_owner);
        ctx->h_resident = (int *)((char *)cfg->host_arena + L.host_resident);
        dv.moves = (const int *)((char *)dptr + L.host_moves);
        dv.n_moves = (const int *)((char *)dptr + L.host_nmoves);
        HostTier *ht = new (std::nothrow) HostTier();
        if (!ht) return bail(MOSAIC_ENOMEM, "host allocation failed");
        ctx->host = ht;
        ht->init(dv.U, dv.C, dv.C + L.buf_max, dv.F, L.SF, L.slabs_per_unit, L.PU, L.max_clusters, dv.k, L.kpage, L.vpage);
        // default-priority streams for selection and for the fetches
        // two internal streams only: selection (+ value fetches) and key fetches
        if ((e = hipStreamCreateWithFlags(&ht->sel_stream, hipStreamNonBlocking)) != hipSuccess ||
            (e = hipStreamCreateWithFlags(&ht->copy_stream, hipStreamNonBlocking)) != hipSuccess ||
            (e = hipEventCreateWithFlags(&ht->main_mark, hipEventDisableTiming)) != hipSuccess ||
            (e = hipEventCreateWithFlags(&ht->off_ready, hipEventDisableTiming)) != hipSuccess ||
            (e = hipEventCreateWithFlags(&ht->off_done[0], hipEventDisableTiming)) != hipSuccess ||
            (e = hipEventCreateWithFlags(&ht->off_done[1], hipEventDisableTiming)) != hipSuccess)
            return bail(MOSAIC_EHIP, std::string("host tier stream/event creation: ") + hipGetErrorString(e));
        ht->ready.resize(dv.L); ht->attend_done.resize(dv.L);
        ht->follow_dirty.assign(dv.L, 0);
        ht->attend_recorded.assign(dv.L, 0); ht->ready_recorded.assign(dv.L, 0);
        for (int l = 0; l < dv.L; ++l)
            if ((e = hipEventCreateWithFlags(&ht->ready[l], hipEventDisableTiming)) != hipSuccess ||
                (e = hipEventCreateWithFlags(&ht->attend_done[l], hipEventDisableTiming)) != hipSuccess)
                return bail(MOSAIC_EHIP, std::string("host tier event creation: ") + hipGetErrorString(e));
    }
    if (clear_maintainer(ctx) != hipSuccess) {     // (no context to keep a message in: the code says it)
        (void)mosaic_destroy(ctx);
        *out = nullptr;
        return MOSAIC_EHIP;
    }
    *out = ctx;
    return MOSAIC_OK;
}

int32_t mosaic_destroy(mosaic_ctx *ctx) {
    if (!ctx) return MOSAIC_EINVAL;
    (void)hipStreamSynchronize(ctx->stream);
    if (ctx->assign_stream) {
        (void)hipStreamSynchronize(ctx->assign_stream);
        (void)hipStreamDestroy(ctx->assign_stream);
        (void)hipEventDestroy(ctx->stored);
        (void)hipEventDestroy(ctx->assigned);
    }
    if (HostTier *ht = ctx->host) {
        if (ht->sel_stream) { (void)hipStreamSynchronize(ht->sel_stream); (void)hipStreamDestroy(ht->sel_stream); }
        if (ht->copy_stream) { (void)hipStreamSynchronize(ht->copy_stream); (void)hipStreamDestroy(ht->copy_stream); }
        if (ht->main_mark) (void)hipEventDestroy(ht->main_mark);
        if (ht->off_ready) (void)hipEventDestroy(ht->off_ready);
        for (hipEvent_t e : ht->off_done) if (e) (void)hipEventDestroy(e);
        for (hipEvent_t e : ht->ready) if (e) (void)hipEventDestroy(e);
        for (hipEvent_t e : ht->attend_done) if (e) (void)hipEventDestroy(e);
        for (hipEvent_t e : ht->busy_ev) (void)hipEventDestroy(e);
        delete ht;
    }
    for (hipEvent_t e : ctx->ev) (void)hipEventDestroy(e);
    delete ctx;
    return MOSAIC_OK;
}

// Overlapped ingest: the caller's stream waits for the order-dependent part that earlier ingest calls
// left on the context's own stream.  Called by everything that reads or changes the index.
static int join_ingest(mosaic_ctx *ctx) {
    if (!ctx->assign_pending) return MOSAIC_OK;
    const hipError_t e = hipStreamWaitEvent(ctx->stream, ctx->assigned, 0);
    if (e != hipSuccess) return fail_hip(ctx, e, "hipStreamWaitEvent(overlapped ingest)");
    ctx->assign_pending = false;
    return MOSAIC_OK;
}

int32_t mosaic_ingest_join(mosaic_ctx *ctx) {
    if (!ctx) return MOSAIC_EINVAL;
    return join_ingest(ctx);
}

// State that must read as empty before the initial clustering has run: the flags of the in-kernel
// selection exchange, and the maintainer's.
static hipError_t clear_maintainer(mosaic_ctx *ctx) {
    const DeviceView &dv = ctx->dv;
    hipError_t e;
    if ((e = hipMemsetAsync(dv.sel_flag, 0, (size_t)dv.U * 8, ctx->stream)) != hipSuccess) return e;
    if ((e = hipMemsetAsync(dv.sync_err, 0, 4, ctx->stream)) != hipSuccess) return e;
    ctx->launch_epoch = 0;
    if (!dv.maint_mode) return hipSuccess;
    if ((e = hipMemsetAsync(dv.n_buf, 0, (size_t)dv.U * 4, ctx->stream)) != hipSuccess) return e;
    if ((e = hipMemsetAsync(dv.n_slots, 0, (size_t)dv.U * 4, ctx->stream)) != hipSuccess) return e;
    if ((e = hipMemsetAsync(dv.mt_cnt, 0, (size_t)dv.U * 4 * 8, ctx->stream)) != hipSuccess) return e;
    if ((e = hipMemsetAsync(dv.var, 0, (size_t)dv.U * dv.C * 8, ctx->stream)) != hipSuccess) return e;
    if ((e = hipMemsetAsync(dv.lazy, 0, (size_t)dv.U * dv.C * 4, ctx->stream)) != hipSuccess) return e;
    return hipMemsetAsync(dv.resident, 0, (size_t)dv.U * dv.C * 4, ctx->stream);
}

int32_t mosaic_reset(mosaic_ctx *ctx) {
    if (!ctx) return MOSAIC_EINVAL;
    { const int rc = join_ingest(ctx); if (rc != MOSAIC_OK) return rc; }
    ctx->n_frames = 0;
    ctx->epoch += 1;
    if (HostTier *ht = ctx->host) {
        // nothing may still be reading the cache or the staging ring
        (void)hipStreamSynchronize(ctx->stream);
        (void)hipStreamSynchronize(ht->sel_stream);
        (void)hipStreamSynchronize(ht->copy_stream);
        ht->reset();
        ht->off_used[0] = ht->off_used[1] = false;
        ht->off_idx = 0;
        std::fill(ht->follow_dirty.begin(), ht->follow_dirty.end(), 0);
        ht->hits = ht->misses = ht->evictions = ht->h2d_bytes = ht->h2d_copies = 0;
        ht->pf_calls = ht->pf_fetched = ht->pf_useful = 0;
        ht->busy_ms = 0.0;
        ht->busy_used = 0;
        std::fill(ht->attend_recorded.begin(), ht->attend_recorded.end(), 0);
        std::fill(ht->ready_recorded.begin(), ht->ready_recorded.end(), 0);
    }
    const int attend_impl = ctx->stats.attend_impl;
    memset(&ctx->stats, 0, sizeof ctx->stats);
    ctx->stats.attend_impl = attend_impl;
    hipError_t e = clear_maintainer(ctx);
    if (e != hipSuccess) return fail_hip(ctx, e, "hipMemsetAsync");
    return MOSAIC_OK;
}

// Host tier + deferred-split maintainer: "C is in GPU memory" (Alg. 1 line 4) = the GPU cluster cache
// holds frames of C.  Send the flags of the units whose directory changed since the last time.
static int upload_residency(mosaic_ctx *ctx) {
    const DeviceView &dv = ctx->dv;
    HostTier *ht = ctx->host;
    if (!ht || dv.maint_mode != MOSAIC_MAINT_DEFERRED) return MOSAIC_OK;
    for (int u = 0; u < dv.U; ++u) {
        HostTier::Unit &un = ht->units[u];
        if (!un.resident_dirty) continue;
        int *fl = ctx->h_resident + (size_t)u * dv.C;
        for (int c = 0; c < dv.C; ++c) fl[c] = un.cached[c] > 0;
        const hipError_t e = hipMemcpyAsync(dv.resident + (size_t)u * dv.C, fl, (size_t)dv.C * 4, hipMemcpyHostToDevice, ctx->stream);
        if (e != hipSuccess) return fail_hip(ctx, e, "residency flags upload");
        un.resident_dirty = false;
    }
    return MOSAIC_OK;
}

// Host tier + maintainer: bring the host's frame lists of units [u0, u0 + nu) up to date after device
// work on `s` that may have changed membership (splits on insertion, deferred splits carried out,
// states buffered or released).  The counters and the buffer are small and always read; a unit's whole
// frame -> cluster map only when they say that something moved.  Waits for `s`.
static int follow_membership(mosaic_ctx *ctx, int u0, int nu, hipStream_t s) {
    const DeviceView &dv = ctx->dv;
    HostTier *ht = ctx->host;
    const size_t B = (size_t)dv.buf_max;
    hipError_t e;
    if ((e = hipMemcpyAsync(ctx->h_cnt + (size_t)u0 * 4, dv.mt_cnt + (size_t)u0 * 4, (size_t)nu * 4 * 8, hipMemcpyDeviceToHost, s)) != hipSuccess ||
        (e = hipMemcpyAsync(ctx->h_nbuf + u0, dv.n_buf + u0, (size_t)nu * 4, hipMemcpyDeviceToHost, s)) != hipSuccess)
        return fail_hip(ctx, e, "maintainer counters read-back");
    if (B && ((e = hipMemcpyAsync(ctx->h_buf_frame + (size_t)u0 * B, dv.buf_frame + (size_t)u0 * B, (size_t)nu * B * 4, hipMemcpyDeviceToHost, s)) != hipSuccess))
        return fail_hip(ctx, e, "singleton buffer read-back");
    if ((e = hipStreamSynchronize(s)) != hipSuccess) return fail_hip(ctx, e, "hipStreamSynchronize");
    const size_t nf = (size_t)ctx->n_frames;
    bool any = false;
    for (int u = u0; u < u0 + nu; ++u) {
        const bool moved = ctx->h_cnt[(size_t)u * 4] != ht->seen_splits[(size_t)u * 2] ||
                           ctx->h_cnt[(size_t)u * 4 + 1] != ht->seen_splits[(size_t)u * 2 + 1] ||
                           ctx->h_nbuf[u] != ht->seen_nbuf[u];
        if (!moved) continue;
        any = true;
        if ((e = hipMemcpyAsync(ctx->h_assign_full + (size_t)u * dv.F, dv.assign + (size_t)u * dv.F, nf * 4, hipMemcpyDeviceToHost, s)) != hipSuccess)
            return fail_hip(ctx, e, "frame map read-back");
    }
    if (!any) return MOSAIC_OK;
    if ((e = hipStreamSynchronize(s)) != hipSuccess) return fail_hip(ctx, e, "hipStreamSynchronize");
    for (int u = u0; u < u0 + nu; ++u) {
        const bool moved = ctx->h_cnt[(size_t)u * 4] != ht->seen_splits[(size_t)u * 2] ||
                           ctx->h_cnt[(size_t)u * 4 + 1] != ht->seen_splits[(size_t)u * 2 + 1] ||
                           ctx->h_nbuf[u] != ht->seen_nbuf[u];
        if (!moved) continue;
        const int nb = std::min<int>(ctx->h_nbuf[u], (int)B);
        ht->rebuild(u, ctx->h_assign_full + (size_t)u * dv.F, (int)nf, ctx->h_buf_frame + (size_t)u * B, nb);
        ht->seen_splits[(size_t)u * 2] = ctx->h_cnt[(size_t)u * 4];
        ht->seen_splits[(size_t)u * 2 + 1] = ctx->h_cnt[(size_t)u * 4 + 1];
        ht->seen_nbuf[u] = ctx->h_nbuf[u];
    }
    return MOSAIC_OK;
}

// Host tier: read back the assignments of staged frames f0..f1-1, give every
// page its slab position, and store the pages into pinned host memory.
// (ctx->n_frames must already count the frames up to f1.)
// The staging ring holds frame f in slot f % SN.  Before frames [g0, g1) are staged, the caller's stream waits for
// every offload still counted that read slots of theirs.
static int wait_for_ring(mosaic_ctx *ctx, long long g0, long long g1) {
    HostTier *ht = ctx->host;
    const long long SN = ctx->dv.SN;
    for (int p = 0; p < 2; ++p) {
        if (!ht->off_used[p]) continue;
        const long long a0 = ht->off_f0[p], a1 = ht->off_f1[p];
        bool overlap = (a1 - a0) >= SN || (g1 - g0) >= SN;
        for (long long f = g0; f < g1 && !overlap; ++f) {
            const long long d = ((f - a0) % SN + SN) % SN;       // slot distance from the offload's first frame
            overlap = d < a1 - a0;
        }
        if (!overlap) continue;
        const hipError_t e = hipStreamWaitEvent(ctx->stream, ht->off_done[p], 0);
        if (e != hipSuccess) return fail_hip(ctx, e, "hipStreamWaitEvent(offload)");
        ht->off_used[p] = false;
    }
    return MOSAIC_OK;
}

static int offload_range(mosaic_ctx *ctx, int f0, int f1) {
    const DeviceView &dv = ctx->dv;
    HostTier *ht = ctx->host;
    const int n = f1 - f0;
    const int p = (int)(ht->off_idx & 1);                 // slab table of this batch
    // both directions go through pinned memory of the host arena: an asynchronous copy to
    // or from pageable memory is only complete (or its source only free) when the runtime
    // says so, which a stream synchronisation does not promise
    int *a = ctx->h_assign, *dest = ctx->h_dest + (size_t)p * dv.U * dv.SN;
    hipError_t e = hipSuccess;
    // the batch's assignments are final (and the upload of this table's previous contents, two batches ago, is over)
    if ((e = hipStreamSynchronize(ctx->stream)) != hipSuccess) return fail_hip(ctx, e, "hipStreamSynchronize");
    for (int u = 0; u < dv.U && e == hipSuccess; ++u)
        e = hipMemcpyAsync(a + (size_t)u * n, dv.assign + (size_t)u * dv.F + f0, (size_t)n * 4,
                           hipMemcpyDeviceToHost, ctx->stream);
    if (e != hipSuccess) return fail_hip(ctx, e, "assignment read-back");
    if ((e = hipStreamSynchronize(ctx->stream)) != hipSuccess) return fail_hip(ctx, e, "hipStreamSynchronize");
    for (int fl = 0; fl < n; ++fl)
        for (int u = 0; u < dv.U; ++u) {
            // a state held in the singleton buffer (-2 - owner) is filed with its owner's pages
            const int c = a[(size_t)u * n + fl], filed = c >= 0 ? c : -2 - c;
            if (filed < 0 || filed >= dv.C) return fail(ctx, MOSAIC_EHIP, "assignment read-back returned an invalid cluster id");
            const int hp = ht->place(u, f0 + fl, filed);
            if (hp < 0) return fail(ctx, MOSAIC_ECAPACITY, "host slab pool exhausted");
            dest[(size_t)u * dv.SN + fl] = hp;
            if (c >= 0) ht->join(u, f0 + fl, c);     // (units whose membership moved are rebuilt below)
        }
    // The offload itself goes to the copy stream, behind the table's upload, so that the caller's stream can stage
    // and assign the next batch meanwhile; the device copy of this table was last read by the offload two batches ago.
    DeviceView d2 = dv;
    d2.dest = dv.dest + (size_t)p * dv.U * dv.SN;
    if (ht->off_used[p]) {
        if ((e = hipStreamWaitEvent(ctx->stream, ht->off_done[p], 0)) != hipSuccess) return fail_hip(ctx, e, "hipStreamWaitEvent(offload)");
        ht->off_used[p] = false;
    }
    e = hipMemcpyAsync(d2.dest, dest, (size_t)dv.U * dv.SN * 4, hipMemcpyHostToDevice, ctx->stream);
    if (e != hipSuccess) return fail_hip(ctx, e, "slab table upload");
    if ((e = hipEventRecord(ht->off_ready, ctx->stream)) != hipSuccess ||
        (e = hipStreamWaitEvent(ht->copy_stream, ht->off_ready, 0)) != hipSuccess)
        return fail_hip(ctx, e, "ordering the offload after its slab table");
    if ((e = launch_offload(d2, f0, n, ht->copy_stream)) != hipSuccess) return fail_hip(ctx, e, "offload launch");
    if ((e = hipEventRecord(ht->off_done[p], ht->copy_stream)) != hipSuccess) return fail_hip(ctx, e, "hipEventRecord(offload)");
    ht->off_used[p] = true; ht->off_f0[p] = f0; ht->off_f1[p] = f1;
    ht->off_idx += 1;
    // Membership after splits.  Deferred splits test "C is in GPU memory" against the cache directory at every
    // insertion batch, so the host follows at once; eager splits never ask, so the host follows when the layer is
    // next queried (reading every unit's frame map back after every batch was more than half of the ingest time).
    if (dv.maint_mode == MOSAIC_MAINT_DEFERRED) return follow_membership(ctx, 0, dv.U, ctx->stream);
    if (dv.maint_mode) std::fill(ht->follow_dirty.begin(), ht->follow_dirty.end(), 1);
    return MOSAIC_OK;
}

static int ingest_host(mosaic_ctx *ctx, const void *k_dev, const void *v_dev, int n_frames) {
    const DeviceView &dv = ctx->dv;
    HostTier *ht = ctx->host;
    const size_t frame_bytes = (size_t)dv.U * dv.T * dv.D * dv.esize;
    long long f = ctx->n_frames;
    const long long end = f + n_frames, W = ctx->W;
    size_t done = 0;
    hipError_t e;
    int rc;
    while (f < end) {
        if ((rc = upload_residency(ctx)) != MOSAIC_OK) return rc;
        // warm-up frames stay in the staging ring (SN >= W); afterwards batches of <= 64
        const int nb = (int)(f < W ? std::min(end, W) - f : std::min<long long>(end - f, 64));
        if ((rc = wait_for_ring(ctx, f, f + nb)) != MOSAIC_OK) return rc;
        e = launch_store_summary(dv, (const char *)k_dev + done * frame_bytes,
                                 (const char *)v_dev + done * frame_bytes, (int)f, nb, ctx->stream);
        if (e != hipSuccess) return fail_hip(ctx, e, "store_summary launch");
        if (f < W) {
            f += nb;
            if (f == W) {
                if ((e = launch_lloyd(dv, (int)W, ctx->iters, true, ctx->stream)) != hipSuccess)
                    return fail_hip(ctx, e, "initial clustering launch");
                ctx->stats.lloyd_runs += 1;
                ctx->n_frames = f;
                if ((rc = offload_range(ctx, 0, (int)W)) != MOSAIC_OK) return rc;
            }
        } else {
            if ((e = launch_assign_update(dv, (int)f, (int)f + nb, ctx->stream)) != hipSuccess)
                return fail_hip(ctx, e, "assign_update launch");
            ctx->n_frames = f + nb;
            if ((rc = offload_range(ctx, (int)f, (int)f + nb)) != MOSAIC_OK) return rc;
            f += nb;
        }
        done += nb;
        // a failure above leaves the frames before this batch ingested
        ctx->n_frames = f;
    }
    (void)ht;
    return MOSAIC_OK;
}

static int ingest_frames(mosaic_ctx *ctx, const void *k_dev, const void *v_dev, const float *e_dev,
                         int32_t n_frames);

int32_t mosaic_ingest_frame(mosaic_ctx *ctx, const void *k_dev, const void *v_dev, int32_t n_frames) {
    if (!ctx) return MOSAIC_EINVAL;
    if (ctx->dv.P > 0) return fail(ctx, MOSAIC_EINVAL, "n_partitions > 0: frames are ingested with mosaic_ingest_frame_visual");
    return ingest_frames(ctx, k_dev, v_dev, nullptr, n_frames);
}

int32_t mosaic_ingest_frame_visual(mosaic_ctx *ctx, const void *k_dev, const void *v_dev, const float *e_dev,
                                   int32_t n_frames) {
    if (!ctx) return MOSAIC_EINVAL;
    if (ctx->dv.P <= 0) return fail(ctx, MOSAIC_EINVAL, "n_partitions == 0: frames are ingested with mosaic_ingest_frame");
    if (!e_dev) return fail(ctx, MOSAIC_EINVAL, "e_dev is NULL");
    if ((uintptr_t)e_dev % 16) return fail(ctx, MOSAIC_EINVAL, "e_dev must be 16-byte aligned");
    return ingest_frames(ctx, k_dev, v_dev, e_dev, n_frames);
}

static int ingest_frames(mosaic_ctx *ctx, const void *k_dev, const void *v_dev, const float *e_dev,
                         int32_t n_frames) {
    if (!k_dev || !v_dev) return fail(ctx, MOSAIC_EINVAL, "k_dev / v_dev is NULL");
    if (((uintptr_t)k_dev | (uintptr_t)v_dev) % 16) return fail(ctx, MOSAIC_EINVAL, "k_dev / v_dev must be 16-byte aligned");
    if (n_frames < 1) return fail(ctx, MOSAIC_EINVAL, "n_frames must be >= 1");
    const DeviceView &dv = ctx->dv;
    if (ctx->n_frames + n_frames > dv.F) return fail(ctx, MOSAIC_ECAPACITY, "max_frames exceeded");
    if (ctx->host) {
        const long long before = ctx->n_frames;
        const int rc = ingest_host(ctx, k_dev, v_dev, n_frames);
        ctx->epoch += 1;
        ctx->stats.frames_ingested = ctx->n_frames;
        ctx->stats.kv_bytes_stored += (int64_t)(ctx->n_frames - before) * dv.U * dv.T * dv.D * dv.esize * 2;
        ctx->stats.ready = ctx->n_frames >= ctx->W;
        return rc;
    }
    hipError_t e;
    // A single frame of the online phase takes one launch where the assignment kernel that keeps
    // the table in registers applies: its workgroups store the pages and form the summary themselves.
    const bool one_launch = n_frames == 1 && ctx->n_frames >= ctx->W && !dv.maint_mode && dv.C <= 128;
    // Overlapped ingest: the order-dependent part of a batched call goes to the context's own stream
    // (it reads nothing of the caller's buffers), so that the next call's page stores run beside it.
    const bool overlap = ctx->assign_stream != nullptr && n_frames > 1;
    if (!overlap) { const int rc = join_ingest(ctx); if (rc != MOSAIC_OK) return rc; }
    const hipStream_t dep = overlap ? ctx->assign_stream : ctx->stream;
    // pages + summaries of the whole batch (independent across frames); the grid's
    // y dimension is limited to 65535 frames per launch
    for (int done = 0; done < n_frames && !one_launch;) {
        const int nb = std::min(n_frames - done, 32768);
        const size_t in_off = (size_t)done * dv.U * dv.T * dv.D * dv.esize;
        e = launch_store_summary(dv, (const char *)k_dev + in_off, (const char *)v_dev + in_off,
                                 (int)ctx->n_frames + done, nb, ctx->stream);
        if (e != hipSuccess) return fail_hip(ctx, e, "store_summary launch");
        // embeddings of warm-up frames are only filed; later ones are filed by the visual assignment
        const long long first = ctx->n_frames + done, n_warm = std::min<long long>(first + nb, ctx->W) - first;
        if (e_dev && n_warm > 0) {
            e = launch_visual_store(dv, e_dev + (size_t)done * dv.Dv, (int)first, (int)n_warm, ctx->stream);
            if (e != hipSuccess) return fail_hip(ctx, e, "visual_store launch");
        }
        done += nb;
    }
    if (overlap) {
        if ((e = hipEventRecord(ctx->stored, ctx->stream)) != hipSuccess ||
            (e = hipStreamWaitEvent(ctx->assign_stream, ctx->stored, 0)) != hipSuccess)
            return fail_hip(ctx, e, "ordering the assignment after the page stores");
    }
    // temporally dependent part, in stream order
    long long f = ctx->n_frames;
    const long long end = f + n_frames, W = ctx->W, every = ctx->cfg.recluster_every;
    while (f < end) {
        if (f < W) {
            f = std::min(end, W);
            if (f == W) {
                if (dv.P > 0) {      // the visual level first: the units' K-means runs inside its partitions
                    e = launch_visual_lloyd(dv, (int)W, ctx->iters, dep);
                    if (e != hipSuccess) return fail_hip(ctx, e, "visual clustering launch");
                }
                e = launch_lloyd(dv, (int)W, ctx->iters, true, dep);
                if (e != hipSuccess) return fail_hip(ctx, e, "initial clustering launch");
                if (dv.P > 0) {
                    e = launch_partition_reps(dv, (int)W, dep);
                    if (e != hipSuccess) return fail_hip(ctx, e, "partition representatives launch");
                }
                ctx->stats.lloyd_runs += 1;
            }
            continue;
        }
        long long seg_end = end;
        if (every > 0) seg_end = std::min(end, (f / every + 1) * every);
        if (dv.P > 0) {
            e = launch_visual_assign(dv, e_dev + (size_t)(f - ctx->n_frames) * dv.Dv, (int)f, (int)seg_end, dep);
            if (e != hipSuccess) return fail_hip(ctx, e, "visual assignment launch");
        }
        e = one_launch ? launch_ingest_one(dv, k_dev, v_dev, (int)f, dep)
                       : launch_assign_update(dv, (int)f, (int)seg_end, dep);
        if (e != hipSuccess) return fail_hip(ctx, e, "assign_update launch");
        f = seg_end;
        if (every > 0 && f % every == 0) {
            e = launch_lloyd(dv, (int)f, ctx->iters, false, dep);
            if (e != hipSuccess) return fail_hip(ctx, e, "re-clustering launch");
            ctx->stats.lloyd_runs += 1;
        }
    }
    if (overlap) {
        if ((e = hipEventRecord(ctx->assigned, ctx->assign_stream)) != hipSuccess)
            return fail_hip(ctx, e, "marking the end of the assignment");
        ctx->assign_pending = true;
    }
    ctx->n_frames = end;
    ctx->epoch += 1;
    ctx->stats.frames_ingested = end;
    ctx->stats.kv_bytes_stored += (int64_t)n_frames * dv.U * dv.T * dv.D * dv.esize * 2;
    ctx->stats.ready = end >= W;
    return MOSAIC_OK;
}

static int check_query_args(mosaic_ctx *ctx, int32_t layer, const void *q_dev, int32_t Tq, int *u0,
                            int *n_units) {
    if (!q_dev) return fail(ctx, MOSAIC_EINVAL, "q_dev is NULL");
    if ((uintptr_t)q_dev % 16) return fail(ctx, MOSAIC_EINVAL, "q_dev must be 16-byte aligned");
    if (layer < -1 || layer >= ctx->dv.L) return fail(ctx, MOSAIC_EINVAL, "layer out of range");
    { const int rc = join_ingest(ctx); if (rc != MOSAIC_OK) return rc; }       // every query call comes through here
    const int maxq = ctx->cfg.max_q_tokens > 0 ? ctx->cfg.max_q_tokens : 256;
    if (Tq < 1 || Tq > maxq) return fail(ctx, MOSAIC_EINVAL, "n_q_tokens must be in 1..max_q_tokens");
    *u0 = layer < 0 ? 0 : layer * ctx->dv.Hkv;
    *n_units = layer < 0 ? ctx->dv.U : ctx->dv.Hkv;
    return MOSAIC_OK;
}

// Host tier, profiling: add the elapsed times of the event pairs used so far to busy_ms (waits for
// the copy stream) and make the pool available again.
static hipError_t fold_busy_events(mosaic_ctx *ctx) {
    HostTier *ht = ctx->host;
    if (ht->busy_used == 0) return hipSuccess;
    hipError_t e = hipStreamSynchronize(ht->copy_stream);
    if (e != hipSuccess) return e;
    for (size_t i = 0; i + 1 < ht->busy_used; i += 2) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, ht->busy_ev[i], ht->busy_ev[i + 1]) == hipSuccess) ht->busy_ms += ms;
    }
    ht->busy_used = 0;
    return hipSuccess;
}

// Host tier: selection on the selection stream, LRU + fetches on the copy stream.
static int retrieve_host(mosaic_ctx *ctx, int layer, const void *q_dev, int Tq, bool prefetch) {
    const DeviceView &dv = ctx->dv;
    HostTier *ht = ctx->host;
    const int u0 = layer * dv.Hkv, nu = dv.Hkv, k = dv.k;
    hipError_t e;
    // the query was produced by work already enqueued on the caller's stream
    // (and the representatives by the last ingest): mark the stream, wait for the mark
    if ((e = hipEventRecord(ht->main_mark, ctx->stream)) != hipSuccess) return fail_hip(ctx, e, "hipEventRecord");
    if ((e = hipStreamWaitEvent(ht->sel_stream, ht->main_mark, 0)) != hipSuccess) return fail_hip(ctx, e, "hipStreamWaitEvent");
    // Alg. 1, retrieval procedure: with the deferred-split maintainer the buffered singletons take part
    // in the selection and the selected clusters' deferred splits are carried out by the same kernel
    // (a prefetch only predicts: clusters alone, nothing changes)
    const bool deferred = dv.maint_mode == MOSAIC_MAINT_DEFERRED && !prefetch;
    e = deferred ? launch_retrieve_deferred(dv, u0, nu, q_dev, Tq, (int)ctx->n_frames, ctx->cfg.score_mode, ht->sel_stream)
                 : launch_retrieve(dv, u0, nu, q_dev, Tq, (int)ctx->n_frames, ctx->cfg.score_mode, false, ht->sel_stream);
    if (e != hipSuccess) return fail_hip(ctx, e, "retrieve launch");
    int *ids = ctx->h_ids + (size_t)u0 * k, *nids = ctx->h_nids + u0;
    if ((e = hipMemcpyAsync(ids, dv.ids + (size_t)u0 * k, (size_t)nu * k * 4, hipMemcpyDeviceToHost, ht->sel_stream)) != hipSuccess ||
        (e = hipMemcpyAsync(nids, dv.n_ids + u0, (size_t)nu * 4, hipMemcpyDeviceToHost, ht->sel_stream)) != hipSuccess)
        return fail_hip(ctx, e, "selection read-back");
    if ((e = hipStreamSynchronize(ht->sel_stream)) != hipSuccess) return fail_hip(ctx, e, "hipStreamSynchronize");
    if (ht->follow_dirty[layer]) {           // eager splits since this layer was last queried (all ingest work is over: main_mark)
        const int rc2 = follow_membership(ctx, u0, nu, ht->sel_stream);
        if (rc2 != MOSAIC_OK) return rc2;
        ht->follow_dirty[layer] = 0;
    }
    // the pinned page-list staging of this layer must not be in flight any more
    if (ht->ready_recorded[layer] && (e = hipEventSynchronize(ht->ready[layer])) != hipSuccess)
        return fail_hip(ctx, e, "hipEventSynchronize");
    // cache blocks of this layer may still be read by its previous attend
    if (ht->attend_recorded[layer] &&
        (e = hipStreamWaitEvent(ht->copy_stream, ht->attend_done[layer], 0)) != hipSuccess)
        return fail_hip(ctx, e, "hipStreamWaitEvent");
    hipEvent_t b0 = nullptr, b1 = nullptr;
    if (ctx->profile && !ht->busy_ev.empty()) {   // time the copy stream's work for this retrieve (pooled events)
        if (ht->busy_used + 2 > ht->busy_ev.size() && (e = fold_busy_events(ctx)) != hipSuccess)
            return fail_hip(ctx, e, "fetch timing");
        b0 = ht->busy_ev[ht->busy_used]; b1 = ht->busy_ev[ht->busy_used + 1];
        ht->busy_used += 2;
    }
    // all or nothing: the cache directory is only touched once every unit's selection is known to fit
    const auto n_take_of = [&](int i) {
        return prefetch && ctx->cfg.prefetch_top_k > 0 ? std::min(nids[i], ctx->cfg.prefetch_top_k) : nids[i];
    };
    for (int i = 0; i < nu; ++i) {
        if (ht->fits(u0 + i, ids + (size_t)i * k, n_take_of(i))) continue;
        char b[256];
        snprintf(b, sizeof b, "the selected clusters do not fit the GPU cluster cache: unit %d selects %d pages in %d "
                 "clusters (cache: %d pages, at most %d clusters) (raise cache_pages_per_unit / cache_fraction)",
                 u0 + i, ht->fail_sel_pages, n_take_of(i), dv.PU, ht->max_clusters);
        if (b0) ht->busy_used -= 2;
        ctx->sel_epoch[layer] = -1;          // whatever selection the layer had is no longer current
        if (deferred) {                      // the kernel has carried out its deferred splits all the same
            const int rc2 = follow_membership(ctx, u0, nu, ht->sel_stream);
            if (rc2 != MOSAIC_OK) return rc2;
        }
        return fail(ctx, MOSAIC_ECAPACITY, b);
    }
    int max_moves = 0;
    for (int i = 0; i < nu; ++i) {
        const int u = u0 + i;
        int nm = 0, np = 0;
        int *hs = ctx->h_sel + (size_t)u * dv.F;
        const int rc = ht->fetch(u, ids + (size_t)i * k, n_take_of(i), ctx->h_moves + (size_t)u * dv.F * 2, &nm,
                                 hs, &np, prefetch);
        if (rc != MOSAIC_OK) {               // (fits() above rules this out)
            ctx->sel_epoch[layer] = -1;
            return fail(ctx, rc, "cluster cache bookkeeping failed after the capacity check");
        }
        if (!prefetch) {
            HostTier::Unit &un = ht->units[u];
            un.n_last = nids[i];
            std::copy(ids + (size_t)i * k, ids + (size_t)i * k + nids[i], un.last_ids.begin());
        }
        ctx->h_nmoves[u] = nm;
        max_moves = std::max(max_moves, nm);
        ctx->h_nsel[u] = np;
        if (np > 0 && (e = hipMemcpyAsync(dv.sel_pages + (size_t)u * dv.F, hs, (size_t)np * 4, hipMemcpyHostToDevice,
                                          ht->copy_stream)) != hipSuccess) {
            ctx->sel_epoch[layer] = -1;
            return fail_hip(ctx, e, "page list upload");
        }
    }
    if ((e = hipMemcpyAsync(dv.n_sel + u0, ctx->h_nsel + u0, (size_t)nu * 4, hipMemcpyHostToDevice,
                            ht->copy_stream)) != hipSuccess) {
        ctx->sel_epoch[layer] = -1;
        return fail_hip(ctx, e, "page count upload");
    }
    // one kernel moves every missing page of this layer (timed when profiling is on)
    if (b0) (void)hipEventRecord(b0, ht->copy_stream);
    if ((e = launch_fetch(dv, u0, nu, max_moves, ht->copy_stream)) != hipSuccess) return fail_hip(ctx, e, "fetch launch");
    if (max_moves > 0) ht->h2d_copies += 1;
    if (b1) (void)hipEventRecord(b1, ht->copy_stream);
    if ((e = hipEventRecord(ht->ready[layer], ht->copy_stream)) != hipSuccess) return fail_hip(ctx, e, "hipEventRecord");
    ht->ready_recorded[layer] = 1;
    // the query saw the clusters as they were; now follow what the kernel's deferred splits changed
    if (deferred) return follow_membership(ctx, u0, nu, ht->sel_stream);
    return MOSAIC_OK;
}

int32_t mosaic_retrieve(mosaic_ctx *ctx, int32_t layer, const void *q_dev, int32_t n_q_tokens) {
    if (!ctx) return MOSAIC_EINVAL;
    int u0, nu;
    int rc = check_query_args(ctx, layer, q_dev, n_q_tokens, &u0, &nu);
    if (rc != MOSAIC_OK) return rc;
    if (ctx->n_frames < ctx->W) return fail(ctx, MOSAIC_ENOTREADY, "initial clustering has not run yet (fewer than warmup_frames frames ingested)");
    if (ctx->host) {
        if (layer < 0) return fail(ctx, MOSAIC_EINVAL, "the host tier retrieves one layer per call");
        rc = retrieve_host(ctx, layer, q_dev, n_q_tokens, false);
        if (rc != MOSAIC_OK) return rc;
        ctx->sel_epoch[layer] = ctx->epoch; ctx->sel_tq[layer] = n_q_tokens;
        ctx->stats.retrieve_calls += 1;
        return MOSAIC_OK;
    }
    hipError_t e = ctx->dv.maint_mode == MOSAIC_MAINT_DEFERRED
        ? launch_retrieve_deferred(ctx->dv, u0, nu, q_dev, n_q_tokens, (int)ctx->n_frames,
                                   ctx->cfg.score_mode, ctx->stream)
        : launch_retrieve(ctx->dv, u0, nu, q_dev, n_q_tokens, (int)ctx->n_frames,
                          ctx->cfg.score_mode, true, ctx->stream);
    if (e != hipSuccess) return fail_hip(ctx, e, "retrieve launch");
    const int l0 = layer < 0 ? 0 : layer, l1 = layer < 0 ? ctx->dv.L : layer + 1;
    for (int l = l0; l < l1; ++l) { ctx->sel_epoch[l] = ctx->epoch; ctx->sel_tq[l] = n_q_tokens; }
    ctx->stats.retrieve_calls += 1;
    return MOSAIC_OK;
}

int32_t mosaic_prefetch(mosaic_ctx *ctx, int32_t layer, const void *q_proxy_dev, int32_t n_q_tokens) {
    if (!ctx) return MOSAIC_EINVAL;
    if (!ctx->host) return fail(ctx, MOSAIC_EINVAL, "mosaic_prefetch needs the host tier (MOSAIC_TIER_HOST)");
    if (layer < 0) return fail(ctx, MOSAIC_EINVAL, "mosaic_prefetch takes one layer per call");
    int u0, nu;
    int rc = check_query_args(ctx, layer, q_proxy_dev, n_q_tokens, &u0, &nu);
    if (rc != MOSAIC_OK) return rc;
    if (ctx->n_frames < ctx->W) return fail(ctx, MOSAIC_ENOTREADY, "initial clustering has not run yet (fewer than warmup_frames frames ingested)");
    rc = retrieve_host(ctx, layer, q_proxy_dev, n_q_tokens, true);
    if (rc != MOSAIC_OK) return rc;
    ctx->sel_epoch[layer] = -1;          // a prediction is not a selection: attend needs mosaic_retrieve
    ctx->host->pf_calls += 1;
    return MOSAIC_OK;
}

// The decode kernels read K/V with the non-temporal hint once the stored KV is well beyond the 256 MB
// memory-side cache (measured: 15 GB store, 3.3 GB per launch 562 -> 519 us; 134 MB store, 26 MB per
// launch 18.1 -> 19.5 us with the hint; at 268 MB 22.5 -> 24.5 us, at 537 MB equal, at 1074 MB 48.5 -> 45.9 us:
// stores beyond 768 MiB get it).
static bool kv_beyond_caches(const mosaic_ctx *ctx) {
    const DeviceView &dv = ctx->dv;
    // (host tier: what the kernels read is the GPU cluster cache, PU pages per unit)
    const long long pages = ctx->host ? (long long)dv.PU : ctx->n_frames;
    const long long stored = pages * (long long)dv.U * (long long)(dv.kpage + dv.vpage);
    return stored > (768ll << 20);
}

// Profiling: sum the kernel times of the event pairs used so far into prof_ms (waits for the
// stream) and make the pool available again.
static hipError_t fold_profile_events(mosaic_ctx *ctx) {
    if (ctx->ev_used == 0) return hipSuccess;
    hipError_t e = hipStreamSynchronize(ctx->stream);
    if (e != hipSuccess) return e;
    for (size_t i = 0; i + 1 < ctx->ev_used; i += 2) {
        float ms = 0.f;
        if ((e = hipEventElapsedTime(&ms, ctx->ev[i], ctx->ev[i + 1])) != hipSuccess) return e;
        ctx->prof_ms += ms;
    }
    ctx->prof_n += (long long)(ctx->ev_used / 2);
    ctx->ev_used = 0;
    return hipSuccess;
}

// An event pair from the pool for one attention launch while profiling is on (else both null).
static hipError_t take_profile_events(mosaic_ctx *ctx, hipEvent_t *ev0, hipEvent_t *ev1) {
    *ev0 = *ev1 = nullptr;
    if (!ctx->profile || ctx->ev.empty()) return hipSuccess;
    if (ctx->ev_used + 2 > ctx->ev.size()) {
        const hipError_t e = fold_profile_events(ctx);
        if (e != hipSuccess) return e;
    }
    *ev0 = ctx->ev[ctx->ev_used]; *ev1 = ctx->ev[ctx->ev_used + 1];
    ctx->ev_used += 2;
    return hipSuccess;
}

// Body of mosaic_attend and mosaic_attend_static: `dv` is the context's view with the partial
// buffers the kernels are to use (the arena's, or the static scratch); `timed`: attach the
// profiling events when profiling is on.
static int attend_with(mosaic_ctx *ctx, const DeviceView &dv, int32_t layer, const void *q_dev, int32_t n_q_tokens,
                       void *out_dev, float *lse_dev, bool timed) {
    int u0, nu;
    int rc = check_query_args(ctx, layer, q_dev, n_q_tokens, &u0, &nu);
    if (rc != MOSAIC_OK) return rc;
    if (!out_dev) return fail(ctx, MOSAIC_EINVAL, "out_dev is NULL");
    const int l0 = layer < 0 ? 0 : layer, l1 = layer < 0 ? dv.L : layer + 1;
    for (int l = l0; l < l1; ++l)
        if (ctx->sel_epoch[l] != ctx->epoch)
            return fail(ctx, MOSAIC_ENOTREADY, "no current selection for this layer: call mosaic_retrieve after the last ingest");
    const long long NT = ((long long)n_q_tokens * dv.G + kRowTile - 1) / kRowTile;
    if ((long long)nu * NT > dv.part_entries) {
        char b[200];
        snprintf(b, sizeof b, "attention partials of this call need %lld entries (units x row tiles), the buffer holds %lld",
                 (long long)nu * NT, dv.part_entries);
        return fail(ctx, MOSAIC_ECAPACITY, b);
    }
    const int S = choose_splits(ctx, nu, n_q_tokens, dv.part_entries);
    hipError_t e;
    if (ctx->host) {
        if (layer < 0) return fail(ctx, MOSAIC_EINVAL, "the host tier attends one layer per call");
        if ((e = hipStreamWaitEvent(ctx->stream, ctx->host->ready[layer], 0)) != hipSuccess)
            return fail_hip(ctx, e, "hipStreamWaitEvent");
    }
    hipEvent_t ev0 = nullptr, ev1 = nullptr;
    if (timed && (e = take_profile_events(ctx, &ev0, &ev1)) != hipSuccess) return fail_hip(ctx, e, "kernel timing");
    if (dv.aug_reps && ctx->rv_epoch != ctx->epoch) {
        // global representatives (Sec. V-C): the clustering changed since the value sums were formed.
        // Their attention partial is computed by extra workgroups of the attention launch below.
        // (Its own kernel cost ~8 us per decode step; its own stream, with fork/join events, more.)
        if ((e = launch_value_reps(dv, (int)ctx->n_frames, ctx->stream)) != hipSuccess)
            return fail_hip(ctx, e, "value representatives launch");
        ctx->rv_epoch = ctx->epoch;
    }
    e = ctx->impl == MOSAIC_ATTEND_MFMA
            ? launch_attend_mfma(dv, u0, nu, q_dev, n_q_tokens, S, kv_beyond_caches(ctx), ctx->stream, ev0, ev1)
            : launch_attend_valu(dv, u0, nu, q_dev, n_q_tokens, S, ctx->stream, ev0, ev1);
    if (e != hipSuccess) return fail_hip(ctx, e, "attend launch");
    e = launch_attend_combine(dv, u0, nu, n_q_tokens, S, out_dev, lse_dev, ctx->stream);
    if (e != hipSuccess) return fail_hip(ctx, e, "combine launch");
    if (ctx->host) {
        if ((e = hipEventRecord(ctx->host->attend_done[layer], ctx->stream)) != hipSuccess)
            return fail_hip(ctx, e, "hipEventRecord");
        ctx->host->attend_recorded[layer] = 1;
    }
    ctx->stats.attend_calls += 1;
    ctx->stats.last_n_splits = S;
    return MOSAIC_OK;
}

int32_t mosaic_attend(mosaic_ctx *ctx, int32_t layer, const void *q_dev, int32_t n_q_tokens,
                      void *out_dev, float *lse_dev) {
    if (!ctx) return MOSAIC_EINVAL;
    return attend_with(ctx, ctx->dv, layer, q_dev, n_q_tokens, out_dev, lse_dev, true);
}

int32_t mosaic_attend_static(mosaic_ctx *ctx, int32_t layer, const void *q_dev, int32_t n_q_tokens,
                             void *out_dev, float *lse_dev) {
    if (!ctx) return MOSAIC_EINVAL;
    if (!ctx->static_scratch) return fail(ctx, MOSAIC_EHIP, "the static scratch buffer has no device address");
    // the same kernels, with their split partials in the library's static buffer instead of the arena:
    // [entries][16][D] outputs, then [entries][3][16] statistics; every entry a launch reads was written
    // by that launch, so nothing has to be cleared between calls
    DeviceView dv = ctx->dv;
    const size_t per_entry = (size_t)kRowTile * dv.D * 4 + (size_t)kMlRows * kRowTile * 4;
    dv.part_entries = (long long)(kStaticScratchBytes / per_entry);
    dv.part_o = (float *)ctx->static_scratch;
    dv.part_ml = dv.part_o + (size_t)dv.part_entries * kRowTile * dv.D;
    return attend_with(ctx, dv, layer, q_dev, n_q_tokens, out_dev, lse_dev, false);
}

int32_t mosaic_decode_step(mosaic_ctx *ctx, int32_t layer, const void *q_dev, int32_t n_q_tokens,
                           void *out_dev, float *lse_dev) {
    if (!ctx) return MOSAIC_EINVAL;
    const DeviceView &dv = ctx->dv;
    const long long NT = ((long long)n_q_tokens * dv.G + kRowTile - 1) / kRowTile;
    // The fused kernel pays for a shorter launch chain with equal (not size-proportional) splits and a
    // selection repeated by every workgroup: it wins while the step is latency-bound, i.e. while the
    // expected K/V volume of the launch is small (measured: 26 MB -15 %, 118 MB +7 %).
    const long long est_pages = std::max<long long>(1, (ctx->n_frames * dv.k + dv.C - 1) / dv.C);
    const long long est_bytes = (long long)dv.Hkv * est_pages * (long long)(dv.kpage + dv.vpage);
    const bool fused = !ctx->host && ctx->impl == MOSAIC_ATTEND_MFMA && layer >= 0 && NT == 1 &&
                       dv.maint_mode == MOSAIC_MAINT_OFF && !dv.aug_reps && !dv.aug_window && dv.P == 0 &&
                       dv.C <= 256 && ctx->cfg.decode_fused_max_mib >= 0 &&
                       est_bytes <= ((long long)(ctx->cfg.decode_fused_max_mib > 0 ? ctx->cfg.decode_fused_max_mib : 48) << 20);
    int S = 0;
    if (fused) {
        S = choose_splits(ctx, dv.Hkv, n_q_tokens, dv.part_entries);
        // a workgroup lists the pages of its chunk range in LDS (2048 entries)
        while (S < kMaxSplits && ctx->n_frames / S + 2 > 2048) ++S;
    }
    if (!fused || ctx->n_frames / std::max(S, 1) + 2 > 2048 ||
        (long long)dv.Hkv * S > dv.part_entries) {
        // On request (decode_fused_max_mib = -1) the selection moves into the attention launch, whose first
        // workgroups select and publish, with splits proportional to the retrieved sizes.  Not the
        // default: what the waiting workgroups read must cross the chip's L2s, and those round trips
        // cost more than the selection launch they replace (28 launches of ~118 MB: 47 us against 39 us).
        const bool layer_fused = !ctx->host && ctx->impl == MOSAIC_ATTEND_MFMA && layer >= 0 && NT == 1 &&
                                 dv.maint_mode == MOSAIC_MAINT_OFF && !dv.aug_reps && !dv.aug_window && dv.P == 0 &&
                                 dv.C <= 256 && dv.Hkv <= 64 && ctx->cfg.decode_fused_max_mib == -1;
        if (!layer_fused) {
            ctx->stats.last_decode_fused = 0;
            const int rc = mosaic_retrieve(ctx, layer, q_dev, n_q_tokens);
            return rc != MOSAIC_OK ? rc : mosaic_attend(ctx, layer, q_dev, n_q_tokens, out_dev, lse_dev);
        }
        int u0, nu;
        int rc = check_query_args(ctx, layer, q_dev, n_q_tokens, &u0, &nu);
        if (rc != MOSAIC_OK) return rc;
        if (!out_dev) return fail(ctx, MOSAIC_EINVAL, "out_dev is NULL");
        if (ctx->n_frames < ctx->W) return fail(ctx, MOSAIC_ENOTREADY, "initial clustering has not run yet (fewer than warmup_frames frames ingested)");
        const int S2 = choose_splits(ctx, nu, n_q_tokens, dv.part_entries);
        const int B = std::max(nu * S2, nu);
        hipError_t e;
        hipEvent_t ev0 = nullptr, ev1 = nullptr;
        if ((e = take_profile_events(ctx, &ev0, &ev1)) != hipSuccess) return fail_hip(ctx, e, "kernel timing");
        if (++ctx->launch_epoch == 0x7fffffff) ctx->launch_epoch = 1;      // (flags hold the last ~2^31 launches apart)
        e = launch_decode_layer(dv, u0, nu, q_dev, n_q_tokens, B, (int)ctx->n_frames, ctx->cfg.score_mode,
                                ctx->launch_epoch, kv_beyond_caches(ctx), ctx->stream, ev0, ev1);
        if (e != hipSuccess) return fail_hip(ctx, e, "layer decode launch");
        e = launch_attend_combine(dv, u0, nu, n_q_tokens, S2, out_dev, lse_dev, ctx->stream);
        if (e != hipSuccess) return fail_hip(ctx, e, "combine launch");
        ctx->sel_epoch[layer] = ctx->epoch; ctx->sel_tq[layer] = n_q_tokens;
        ctx->stats.retrieve_calls += 1;
        ctx->stats.attend_calls += 1;
        ctx->stats.last_n_splits = S2;
        ctx->stats.last_decode_fused = 2;
        return MOSAIC_OK;
    }
    int u0, nu;
    int rc = check_query_args(ctx, layer, q_dev, n_q_tokens, &u0, &nu);
    if (rc != MOSAIC_OK) return rc;
    if (!out_dev) return fail(ctx, MOSAIC_EINVAL, "out_dev is NULL");
    if (ctx->n_frames < ctx->W) return fail(ctx, MOSAIC_ENOTREADY, "initial clustering has not run yet (fewer than warmup_frames frames ingested)");
    hipError_t e;
    hipEvent_t ev0 = nullptr, ev1 = nullptr;
    if ((e = take_profile_events(ctx, &ev0, &ev1)) != hipSuccess) return fail_hip(ctx, e, "kernel timing");
    e = launch_decode_fused(dv, u0, nu, q_dev, n_q_tokens, S, (int)ctx->n_frames, ctx->cfg.score_mode,
                            kv_beyond_caches(ctx), ctx->stream, ev0, ev1);
    if (e != hipSuccess) return fail_hip(ctx, e, "fused decode launch");
    e = launch_attend_combine(dv, u0, nu, n_q_tokens, S, out_dev, lse_dev, ctx->stream, true);
    if (e != hipSuccess) return fail_hip(ctx, e, "combine launch");
    ctx->sel_epoch[layer] = ctx->epoch; ctx->sel_tq[layer] = n_q_tokens;
    ctx->stats.retrieve_calls += 1;
    ctx->stats.attend_calls += 1;
    ctx->stats.last_n_splits = S;
    ctx->stats.last_decode_fused = 1;
    return MOSAIC_OK;
}

static int d2h(mosaic_ctx *ctx, void *dst, const void *src, size_t bytes) {     // (observers: after any overlapped ingest)
    { const int rc = join_ingest(ctx); if (rc != MOSAIC_OK) return rc; }
    hipError_t e = hipMemcpyAsync(dst, src, bytes, hipMemcpyDeviceToHost, ctx->stream);
    if (e != hipSuccess) return fail_hip(ctx, e, "hipMemcpyAsync D2H");
    return MOSAIC_OK;
}
static int sync(mosaic_ctx *ctx) {
    { const int rc = join_ingest(ctx); if (rc != MOSAIC_OK) return rc; }
    hipError_t e = hipStreamSynchronize(ctx->stream);
    if (e != hipSuccess) return fail_hip(ctx, e, "hipStreamSynchronize");
    return MOSAIC_OK;
}

int32_t mosaic_get_assignments(mosaic_ctx *ctx, int32_t *frame_to_cluster) {
    if (!ctx) return MOSAIC_EINVAL;
    if (!frame_to_cluster) return fail(ctx, MOSAIC_EINVAL, "frame_to_cluster is NULL");
    const DeviceView &dv = ctx->dv;
    const size_t nf = (size_t)ctx->n_frames;
    if (ctx->n_frames < ctx->W) {
        for (size_t i = 0; i < nf * dv.U; ++i) frame_to_cluster[i] = -1;
        return MOSAIC_OK;
    }
    for (int u = 0; u < dv.U; ++u) {
        int rc = d2h(ctx, frame_to_cluster + (size_t)u * nf, dv.assign + (size_t)u * dv.F, nf * 4);
        if (rc != MOSAIC_OK) return rc;
    }
    return sync(ctx);
}

int32_t mosaic_get_centroids(mosaic_ctx *ctx, double *r, int32_t *n) {
    if (!ctx) return MOSAIC_EINVAL;
    const DeviceView &dv = ctx->dv;
    const size_t UC = (size_t)dv.U * dv.C;
    if (ctx->n_frames < ctx->W) {
        if (r) memset(r, 0, UC * dv.D * 8);
        if (n) memset(n, 0, UC * 4);
        return MOSAIC_OK;
    }
    int rc;
    if (r && (rc = d2h(ctx, r, dv.r, UC * dv.D * 8)) != MOSAIC_OK) return rc;
    if (n && (rc = d2h(ctx, n, dv.n, UC * 4)) != MOSAIC_OK) return rc;
    return sync(ctx);
}

int32_t mosaic_get_summaries(mosaic_ctx *ctx, double *summaries) {
    if (!ctx) return MOSAIC_EINVAL;
    if (!summaries) return fail(ctx, MOSAIC_EINVAL, "summaries is NULL");
    const DeviceView &dv = ctx->dv;
    const size_t nf = (size_t)ctx->n_frames;
    for (int u = 0; u < dv.U; ++u) {
        int rc = d2h(ctx, summaries + (size_t)u * nf * dv.D, dv.summ + (size_t)u * dv.F * dv.D, nf * dv.D * 8);
        if (rc != MOSAIC_OK) return rc;
    }
    return sync(ctx);
}

int32_t mosaic_get_maintainer(mosaic_ctx *ctx, double *var, int32_t *lazy, int32_t *resident,
                              int32_t *n_slots, int32_t *n_buf, int32_t *buf_frame, int32_t *buf_owner) {
    if (!ctx) return MOSAIC_EINVAL;
    const DeviceView &dv = ctx->dv;
    if (!dv.maint_mode) return fail(ctx, MOSAIC_EINVAL, "the maintainer is off (maint_mode = MOSAIC_MAINT_OFF)");
    {   // (host tier: the residency flags follow the cache directory; send what is pending)
        const int rc0 = upload_residency(ctx);
        if (rc0 != MOSAIC_OK) return rc0;
    }
    const size_t UC = (size_t)dv.U * dv.C, UB = (size_t)dv.U * dv.buf_max;
    int rc;
    if (var && (rc = d2h(ctx, var, dv.var, UC * 8)) != MOSAIC_OK) return rc;
    if (lazy && (rc = d2h(ctx, lazy, dv.lazy, UC * 4)) != MOSAIC_OK) return rc;
    if (resident && (rc = d2h(ctx, resident, dv.resident, UC * 4)) != MOSAIC_OK) return rc;
    if (n_slots && (rc = d2h(ctx, n_slots, dv.n_slots, (size_t)dv.U * 4)) != MOSAIC_OK) return rc;
    if (n_buf && (rc = d2h(ctx, n_buf, dv.n_buf, (size_t)dv.U * 4)) != MOSAIC_OK) return rc;
    if (buf_frame && UB && (rc = d2h(ctx, buf_frame, dv.buf_frame, UB * 4)) != MOSAIC_OK) return rc;
    if (buf_owner && UB && (rc = d2h(ctx, buf_owner, dv.buf_owner, UB * 4)) != MOSAIC_OK) return rc;
    return sync(ctx);
}

int32_t mosaic_get_partitions(mosaic_ctx *ctx, int32_t *frame_to_partition, double *visual_r,
                              int32_t *visual_n, double *part_r, int32_t *part_n) {
    if (!ctx) return MOSAIC_EINVAL;
    const DeviceView &dv = ctx->dv;
    if (dv.P <= 0) return fail(ctx, MOSAIC_EINVAL, "n_partitions == 0: there is no visual level");
    int rc = sync(ctx);
    if (rc != MOSAIC_OK) return rc;
    const bool ready = ctx->n_frames >= ctx->W;
    if (frame_to_partition) {
        if (!ready) {
            for (long long f = 0; f < ctx->n_frames; ++f) frame_to_partition[f] = -1;
        } else if ((rc = d2h(ctx, frame_to_partition, dv.part, (size_t)ctx->n_frames * 4)) != MOSAIC_OK) {
            return rc;
        }
    }
    if (!ready) {       // nothing has been built yet
        if (visual_r) memset(visual_r, 0, (size_t)dv.P * dv.Dv * 8);
        if (visual_n) memset(visual_n, 0, (size_t)dv.P * 4);
        if (part_r) memset(part_r, 0, (size_t)dv.U * dv.P * dv.D * 8);
        if (part_n) memset(part_n, 0, (size_t)dv.U * dv.P * 4);
        return MOSAIC_OK;
    }
    if (visual_r && (rc = d2h(ctx, visual_r, dv.vr, (size_t)dv.P * dv.Dv * 8)) != MOSAIC_OK) return rc;
    if (visual_n && (rc = d2h(ctx, visual_n, dv.vn, (size_t)dv.P * 4)) != MOSAIC_OK) return rc;
    if (part_r && (rc = d2h(ctx, part_r, dv.pr, (size_t)dv.U * dv.P * dv.D * 8)) != MOSAIC_OK) return rc;
    if (part_n && (rc = d2h(ctx, part_n, dv.pn, (size_t)dv.U * dv.P * 4)) != MOSAIC_OK) return rc;
    return MOSAIC_OK;
}

int32_t mosaic_get_partition_selection(mosaic_ctx *ctx, int32_t layer, int32_t *part_ids,
                                       int32_t *n_part_ids, double *part_scores) {
    if (!ctx) return MOSAIC_EINVAL;
    const DeviceView &dv = ctx->dv;
    if (dv.P <= 0) return fail(ctx, MOSAIC_EINVAL, "n_partitions == 0: there is no visual level");
    if (layer < 0 || layer >= dv.L) return fail(ctx, MOSAIC_EINVAL, "layer out of range");
    if (ctx->sel_epoch[layer] != ctx->epoch) return fail(ctx, MOSAIC_ENOTREADY, "no current selection for this layer");
    int rc = sync(ctx);
    if (rc != MOSAIC_OK) return rc;
    const size_t u0 = (size_t)layer * dv.Hkv;
    if (part_ids && (rc = d2h(ctx, part_ids, dv.pids + u0 * dv.top_p, (size_t)dv.Hkv * dv.top_p * 4)) != MOSAIC_OK) return rc;
    if (n_part_ids && (rc = d2h(ctx, n_part_ids, dv.n_pids + u0, (size_t)dv.Hkv * 4)) != MOSAIC_OK) return rc;
    if (part_scores && (rc = d2h(ctx, part_scores, dv.pscores + u0 * dv.P, (size_t)dv.Hkv * dv.P * 8)) != MOSAIC_OK) return rc;
    return MOSAIC_OK;
}

int32_t mosaic_get_selection(mosaic_ctx *ctx, int32_t layer, int32_t *ids, int32_t *n_ids,
                             double *scores, int32_t *tok_idx, int64_t tok_cap, int32_t *n_tok) {
    if (!ctx) return MOSAIC_EINVAL;
    const DeviceView &dv = ctx->dv;
    if (layer < 0 || layer >= dv.L) return fail(ctx, MOSAIC_EINVAL, "layer out of range");
    if (ctx->sel_epoch[layer] != ctx->epoch) return fail(ctx, MOSAIC_ENOTREADY, "no current selection for this layer");
    const int u0 = layer * dv.Hkv, H = dv.Hkv;
    int rc;
    if (HostTier *ht = ctx->host) {
        // ids and scores were produced on the selection stream; the token list comes from
        // the host-side cluster membership (frames of each selected cluster, ascending)
        hipError_t he = hipStreamSynchronize(ht->sel_stream);
        if (he != hipSuccess) return fail_hip(ctx, he, "hipStreamSynchronize");
        if (ids && (rc = d2h(ctx, ids, dv.ids + (size_t)u0 * dv.k, (size_t)H * dv.k * 4)) != MOSAIC_OK) return rc;
        if (n_ids && (rc = d2h(ctx, n_ids, dv.n_ids + u0, (size_t)H * 4)) != MOSAIC_OK) return rc;
        if (scores && (rc = d2h(ctx, scores, dv.scores + (size_t)u0 * dv.SC, (size_t)H * dv.SC * 8)) != MOSAIC_OK) return rc;
        if ((rc = sync(ctx)) != MOSAIC_OK) return rc;
        for (int h = 0; h < H; ++h) {
            const HostTier::Unit &un = ht->units[u0 + h];
            const int64_t m = (int64_t)un.n_last_frames * dv.T;     // the frames the query was given, in gather order
            if (n_tok) n_tok[h] = (int32_t)m;
            if (!tok_idx) continue;
            if (m > tok_cap) return fail(ctx, MOSAIC_ECAPACITY, "tok_cap too small for the retrieved token list");
            int32_t *o = tok_idx + (size_t)h * tok_cap;
            for (int i = 0; i < un.n_last_frames; ++i)
                for (int t = 0; t < dv.T; ++t) *o++ = un.last_frames[i] * dv.T + t;
        }
        return MOSAIC_OK;
    }
    if (ids && (rc = d2h(ctx, ids, dv.ids + (size_t)u0 * dv.k, (size_t)H * dv.k * 4)) != MOSAIC_OK) return rc;
    if (n_ids && (rc = d2h(ctx, n_ids, dv.n_ids + u0, (size_t)H * 4)) != MOSAIC_OK) return rc;
    if (scores && (rc = d2h(ctx, scores, dv.scores + (size_t)u0 * dv.SC, (size_t)H * dv.SC * 8)) != MOSAIC_OK) return rc;
    std::vector<int32_t> nsel(H);
    if ((rc = d2h(ctx, nsel.data(), dv.n_sel + u0, (size_t)H * 4)) != MOSAIC_OK) return rc;
    if ((rc = sync(ctx)) != MOSAIC_OK) return rc;
    if (n_tok) for (int h = 0; h < H; ++h) n_tok[h] = nsel[h] * dv.T;
    if (tok_idx) {
        for (int h = 0; h < H; ++h)
            if ((int64_t)nsel[h] * dv.T > tok_cap) return fail(ctx, MOSAIC_ECAPACITY, "tok_cap too small for the retrieved token list");
        hipError_t e = launch_expand_tok_idx(dv, u0, H, ctx->stream);
        if (e != hipSuccess) return fail_hip(ctx, e, "expand_tok_idx launch");
        for (int h = 0; h < H; ++h)
            if (nsel[h] > 0 && (rc = d2h(ctx, tok_idx + (size_t)h * tok_cap, dv.tok_scratch + (size_t)h * dv.F * dv.T,
                                         (size_t)nsel[h] * dv.T * 4)) != MOSAIC_OK) return rc;
        if ((rc = sync(ctx)) != MOSAIC_OK) return rc;
    }
    return MOSAIC_OK;
}

int32_t mosaic_get_cache_directory(mosaic_ctx *ctx, int32_t *cached_pages) {
    if (!ctx) return MOSAIC_EINVAL;
    if (!ctx->host) return fail(ctx, MOSAIC_EINVAL, "the cluster cache exists in the host tier only");
    if (!cached_pages) return fail(ctx, MOSAIC_EINVAL, "cached_pages is NULL");
    const DeviceView &dv = ctx->dv;
    for (int l = 0; l < dv.L; ++l) {         // eager splits the host has not followed yet
        if (!ctx->host->follow_dirty[l]) continue;
        const int rc = follow_membership(ctx, l * dv.Hkv, dv.Hkv, ctx->stream);
        if (rc != MOSAIC_OK) return rc;
        ctx->host->follow_dirty[l] = 0;
    }
    for (int u = 0; u < dv.U; ++u) {
        const HostTier::Unit &un = ctx->host->units[u];
        for (int c = 0; c < dv.C; ++c) cached_pages[(size_t)u * dv.C + c] = un.cached[c] > 0 ? un.cached[c] : -1;
    }
    return MOSAIC_OK;
}

int32_t mosaic_get_stats(mosaic_ctx *ctx, mosaic_stats *stats) {
    if (!ctx || !stats) return MOSAIC_EINVAL;
    if (HostTier *ht = ctx->host) {
        hipError_t e = fold_busy_events(ctx);
        if (e != hipSuccess) return fail_hip(ctx, e, "fetch timing");
        ctx->stats.cache_hits = ht->hits; ctx->stats.cache_misses = ht->misses;
        ctx->stats.h2d_bytes = ht->h2d_bytes; ctx->stats.h2d_copies = ht->h2d_copies;
        ctx->stats.h2d_busy_ms = ht->busy_ms;
        ctx->stats.prefetch_calls = ht->pf_calls; ctx->stats.prefetch_fetched = ht->pf_fetched;
        ctx->stats.prefetch_useful = ht->pf_useful;
    }
    {   // bounded in-kernel waits that ran out (never, unless the GPU was shared with other waiting kernels)
        int err = 0;
        int rc = d2h(ctx, &err, ctx->dv.sync_err, 4);
        if (rc != MOSAIC_OK || (rc = sync(ctx)) != MOSAIC_OK) return rc;
        ctx->stats.sync_timeouts = err;
    }
    if (ctx->dv.maint_mode) {
        const DeviceView &dv = ctx->dv;
        std::vector<long long> cnt((size_t)dv.U * 4);
        int rc = d2h(ctx, cnt.data(), dv.mt_cnt, cnt.size() * 8);
        if (rc != MOSAIC_OK || (rc = sync(ctx)) != MOSAIC_OK) return rc;
        long long tot[4] = {0, 0, 0, 0};
        for (int u = 0; u < dv.U; ++u)
            for (int i = 0; i < 4; ++i) tot[i] += cnt[(size_t)u * 4 + i];
        ctx->stats.splits_immediate = tot[0]; ctx->stats.splits_deferred = tot[1];
        ctx->stats.deferred_inserts = tot[2]; ctx->stats.forced_absorbs = tot[3];
    }
    *stats = ctx->stats;
    return MOSAIC_OK;
}

// Event pools of the profiling mode: created here, never on the query path.
constexpr size_t kProfileEvents = 2 * 2048;

int32_t mosaic_profile_enable(mosaic_ctx *ctx, int32_t on) {
    if (!ctx) return MOSAIC_EINVAL;
    if (on) {
        hipError_t e;
        while (ctx->ev.size() < kProfileEvents) {
            hipEvent_t x;
            if ((e = hipEventCreate(&x)) != hipSuccess) return fail_hip(ctx, e, "hipEventCreate");
            ctx->ev.push_back(x);
        }
        if (HostTier *ht = ctx->host)
            while (ht->busy_ev.size() < kProfileEvents) {
                hipEvent_t x;
                if ((e = hipEventCreate(&x)) != hipSuccess) return fail_hip(ctx, e, "hipEventCreate");
                ht->busy_ev.push_back(x);
            }
    }
    ctx->profile = on != 0;
    return MOSAIC_OK;
}

int32_t mosaic_profile_read(mosaic_ctx *ctx, double *attend_kernel_ms, int64_t *launches) {
    if (!ctx) return MOSAIC_EINVAL;
    int rc = sync(ctx);
    if (rc != MOSAIC_OK) return rc;
    const hipError_t e = fold_profile_events(ctx);
    if (e != hipSuccess) return fail_hip(ctx, e, "hipEventElapsedTime");
    if (attend_kernel_ms) *attend_kernel_ms = ctx->prof_ms;
    if (launches) *launches = (int64_t)ctx->prof_n;
    ctx->prof_ms = 0.0; ctx->prof_n = 0;
    return MOSAIC_OK;
}

const char *mosaic_last_error(const mosaic_ctx *ctx) {
    return ctx ? ctx->err.c_str() : g_create_err.c_str();
}

} // extern "C"
