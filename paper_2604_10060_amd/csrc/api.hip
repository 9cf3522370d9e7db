// C ABI of libmosaic: configuration checks, arena carving, host-side sequencing
// of the kernels.  All frame counting is done on the host from call arguments,
// so no call on the hot path waits for the device.
#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>

#include "mosaic_internal.h"

using namespace mosaic;

struct mosaic_ctx : public Ctx {};

namespace {

thread_local std::string g_create_err = "";

size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

int fail(mosaic_ctx *ctx, int code, const std::string &msg) {
    if (ctx) ctx->err = msg; else g_create_err = msg;
    return code;
}
int fail_hip(mosaic_ctx *ctx, hipError_t e, const char *what) {
    return fail(ctx, MOSAIC_EHIP, std::string(what) + ": " + hipGetErrorString(e));
}

struct Layout {
    size_t k_store, v_store, summ, r, rnorm, n, assign, pos, scores, ids, n_ids, sel_pages, n_sel,
        tok_scratch, part_o, part_ml, total;
    long long part_entries;
    int Tp, impl, v_transposed;
};

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
    const int W = c->warmup_frames > 0 ? c->warmup_frames : 2 * c->n_clusters;
    if (W < c->n_clusters) { why = "warmup_frames must be at least n_clusters (one seed per cluster)"; return MOSAIC_EINVAL; }
    if (c->score_mode != 0 && c->score_mode != 1) { why = "score_mode must be 0 or 1"; return MOSAIC_EINVAL; }
    if (c->attend_impl < MOSAIC_ATTEND_AUTO || c->attend_impl > MOSAIC_ATTEND_MFMA) { why = "attend_impl out of range"; return MOSAIC_EINVAL; }
    if (c->attend_impl == MOSAIC_ATTEND_MFMA && c->kv_dtype != MOSAIC_BF16) { why = "the MFMA attention kernel needs bf16 KV"; return MOSAIC_EINVAL; }
    if ((long long)c->max_frames * c->tokens_per_frame > 0x7fffffffLL) { why = "max_frames * tokens_per_frame must fit in int32"; return MOSAIC_EINVAL; }
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
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
    L.k_store = take(U * F * T * D * e);
    L.v_store = take(U * F * D * (L.v_transposed ? (size_t)L.Tp : T) * e);
    L.summ = take(U * F * D * 8);
    L.r = take(U * C * D * 8);
    L.rnorm = take(U * C * 8);
    L.n = take(U * C * 4);
    L.assign = take(U * F * 4);
    L.pos = take(U * F * 4);
    L.scores = take(U * C * 8);
    L.ids = take(U * k * 4);
    L.n_ids = take(U * 4);
    L.sel_pages = take(U * F * 4);
    L.n_sel = take(U * 4);
    L.tok_scratch = take((size_t)c.n_kv_heads * F * T * 4);
    L.part_o = take((size_t)L.part_entries * kRowTile * D * 4);
    L.part_ml = take((size_t)L.part_entries * 2 * kRowTile * 4);
    L.total = off;
    return L;
}

// KV splits for one attend call, bounded by the partial-buffer capacity.
int choose_splits(const mosaic_ctx *ctx, int n_units, int Tq) {
    const DeviceView &dv = ctx->dv;
    const long long NT = ((long long)Tq * dv.G + kRowTile - 1) / kRowTile;
    const bool mfma = ctx->impl == MOSAIC_ATTEND_MFMA;
    const long long row_blocks = NT == 1 ? 1 : (mfma ? (NT + 15) / 16 : NT);
    const long long est_pages = std::max<long long>(1, (ctx->n_frames * dv.k + dv.C - 1) / dv.C);
    const long long est_chunks = est_pages * dv.chunks_per_page;
    long long s;
    if (NT > 1 && mfma) {
        // MFMA-bound multi-tile launches: every split re-writes 16 x D partial rows per
        // tile, so only as many splits as needed to cover the chip once, each with at
        // least 8 chunks; a multiple of 8 keeps the workgroups that share a
        // (unit, split) on one XCD (workgroup ids congruent mod 8)
        s = (256 + n_units * row_blocks - 1) / (n_units * row_blocks);
        s = std::min(s, std::max<long long>(1, est_chunks / 8));
        if (s >= 8) s = s / 8 * 8;
    } else {
        // bandwidth/latency-bound: cover the chip several times over, at least 4
        // chunks (one per wavefront) per workgroup
        s = (2048 + n_units * row_blocks - 1) / (n_units * row_blocks);
        s = std::min(s, std::max<long long>(1, est_chunks / 4));
    }
    s = std::min<long long>(s, kMaxSplits);
    s = std::min(s, std::max<long long>(1, dv.part_entries / (n_units * NT)));
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

int32_t mosaic_workspace_size(const mosaic_config *cfg, size_t *dev_bytes) {
    std::string why;
    int rc = check_config(cfg, why);
    if (rc != MOSAIC_OK) return fail(nullptr, rc, why);
    if (!dev_bytes) return fail(nullptr, MOSAIC_EINVAL, "dev_bytes is NULL");
    *dev_bytes = make_layout(*cfg).total;
    return MOSAIC_OK;
}

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
    ctx->stream = (hipStream_t)cfg->stream;
    ctx->W = cfg->warmup_frames > 0 ? cfg->warmup_frames : 2 * cfg->n_clusters;
    ctx->iters = cfg->lloyd_iters > 0 ? cfg->lloyd_iters : 8;
    ctx->impl = L.impl;
    ctx->n_frames = 0;
    ctx->epoch = 1;
    ctx->sel_epoch.assign(cfg->n_layers, 0);
    ctx->sel_tq.assign(cfg->n_layers, 0);
    ctx->profile = false;
    ctx->ev_used = 0;
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
    dv.scores = (double *)(base + L.scores); dv.ids = (int *)(base + L.ids);
    dv.n_ids = (int *)(base + L.n_ids); dv.sel_pages = (int *)(base + L.sel_pages);
    dv.n_sel = (int *)(base + L.n_sel); dv.tok_scratch = (int *)(base + L.tok_scratch);
    dv.part_o = (float *)(base + L.part_o); dv.part_ml = (float *)(base + L.part_ml);
    dv.part_entries = L.part_entries;
    *out = ctx;
    return MOSAIC_OK;
}

int32_t mosaic_destroy(mosaic_ctx *ctx) {
    if (!ctx) return MOSAIC_EINVAL;
    (void)hipStreamSynchronize(ctx->stream);
    for (hipEvent_t e : ctx->ev) (void)hipEventDestroy(e);
    delete ctx;
    return MOSAIC_OK;
}

int32_t mosaic_reset(mosaic_ctx *ctx) {
    if (!ctx) return MOSAIC_EINVAL;
    ctx->n_frames = 0;
    ctx->epoch += 1;
    const int attend_impl = ctx->stats.attend_impl;
    memset(&ctx->stats, 0, sizeof ctx->stats);
    ctx->stats.attend_impl = attend_impl;
    return MOSAIC_OK;
}

int32_t mosaic_ingest_frame(mosaic_ctx *ctx, const void *k_dev, const void *v_dev, int32_t n_frames) {
    if (!ctx) return MOSAIC_EINVAL;
    if (!k_dev || !v_dev) return fail(ctx, MOSAIC_EINVAL, "k_dev / v_dev is NULL");
    if (((uintptr_t)k_dev | (uintptr_t)v_dev) % 16) return fail(ctx, MOSAIC_EINVAL, "k_dev / v_dev must be 16-byte aligned");
    if (n_frames < 1) return fail(ctx, MOSAIC_EINVAL, "n_frames must be >= 1");
    const DeviceView &dv = ctx->dv;
    if (ctx->n_frames + n_frames > dv.F) return fail(ctx, MOSAIC_ECAPACITY, "max_frames exceeded");
    hipError_t e;
    // pages + summaries of the whole batch (independent across frames); the grid's
    // y dimension is limited to 65535 frames per launch
    for (int done = 0; done < n_frames;) {
        const int nb = std::min(n_frames - done, 32768);
        const size_t in_off = (size_t)done * dv.U * dv.T * dv.D * dv.esize;
        e = launch_store_summary(dv, (const char *)k_dev + in_off, (const char *)v_dev + in_off,
                                 (int)ctx->n_frames + done, nb, ctx->stream);
        if (e != hipSuccess) return fail_hip(ctx, e, "store_summary launch");
        done += nb;
    }
    // temporally dependent part, in stream order
    long long f = ctx->n_frames;
    const long long end = f + n_frames, W = ctx->W, every = ctx->cfg.recluster_every;
    while (f < end) {
        if (f < W) {
            f = std::min(end, W);
            if (f == W) {
                e = launch_lloyd(dv, (int)W, ctx->iters, true, ctx->stream);
                if (e != hipSuccess) return fail_hip(ctx, e, "initial clustering launch");
                ctx->stats.lloyd_runs += 1;
            }
            continue;
        }
        long long seg_end = end;
        if (every > 0) seg_end = std::min(end, (f / every + 1) * every);
        e = launch_assign_update(dv, (int)f, (int)seg_end, ctx->stream);
        if (e != hipSuccess) return fail_hip(ctx, e, "assign_update launch");
        f = seg_end;
        if (every > 0 && f % every == 0) {
            e = launch_lloyd(dv, (int)f, ctx->iters, false, ctx->stream);
            if (e != hipSuccess) return fail_hip(ctx, e, "re-clustering launch");
            ctx->stats.lloyd_runs += 1;
        }
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
    const int maxq = ctx->cfg.max_q_tokens > 0 ? ctx->cfg.max_q_tokens : 256;
    if (Tq < 1 || Tq > maxq) return fail(ctx, MOSAIC_EINVAL, "n_q_tokens must be in 1..max_q_tokens");
    *u0 = layer < 0 ? 0 : layer * ctx->dv.Hkv;
    *n_units = layer < 0 ? ctx->dv.U : ctx->dv.Hkv;
    return MOSAIC_OK;
}

int32_t mosaic_retrieve(mosaic_ctx *ctx, int32_t layer, const void *q_dev, int32_t n_q_tokens) {
    if (!ctx) return MOSAIC_EINVAL;
    int u0, nu;
    int rc = check_query_args(ctx, layer, q_dev, n_q_tokens, &u0, &nu);
    if (rc != MOSAIC_OK) return rc;
    if (ctx->n_frames < ctx->W) return fail(ctx, MOSAIC_ENOTREADY, "initial clustering has not run yet (fewer than warmup_frames frames ingested)");
    hipError_t e = launch_retrieve(ctx->dv, u0, nu, q_dev, n_q_tokens, (int)ctx->n_frames,
                                   ctx->cfg.score_mode, ctx->stream);
    if (e != hipSuccess) return fail_hip(ctx, e, "retrieve launch");
    const int l0 = layer < 0 ? 0 : layer, l1 = layer < 0 ? ctx->dv.L : layer + 1;
    for (int l = l0; l < l1; ++l) { ctx->sel_epoch[l] = ctx->epoch; ctx->sel_tq[l] = n_q_tokens; }
    ctx->stats.retrieve_calls += 1;
    return MOSAIC_OK;
}

int32_t mosaic_attend(mosaic_ctx *ctx, int32_t layer, const void *q_dev, int32_t n_q_tokens,
                      void *out_dev, float *lse_dev) {
    if (!ctx) return MOSAIC_EINVAL;
    int u0, nu;
    int rc = check_query_args(ctx, layer, q_dev, n_q_tokens, &u0, &nu);
    if (rc != MOSAIC_OK) return rc;
    if (!out_dev) return fail(ctx, MOSAIC_EINVAL, "out_dev is NULL");
    const int l0 = layer < 0 ? 0 : layer, l1 = layer < 0 ? ctx->dv.L : layer + 1;
    for (int l = l0; l < l1; ++l)
        if (ctx->sel_epoch[l] != ctx->epoch)
            return fail(ctx, MOSAIC_ENOTREADY, "no current selection for this layer: call mosaic_retrieve after the last ingest");
    const int S = choose_splits(ctx, nu, n_q_tokens);
    hipError_t e;
    hipEvent_t ev0 = nullptr, ev1 = nullptr;
    if (ctx->profile) {
        if (ctx->ev_used + 2 > ctx->ev.size()) {
            for (int i = 0; i < 2; ++i) {
                hipEvent_t x;
                e = hipEventCreate(&x);
                if (e != hipSuccess) return fail_hip(ctx, e, "hipEventCreate");
                ctx->ev.push_back(x);
            }
        }
        ev0 = ctx->ev[ctx->ev_used]; ev1 = ctx->ev[ctx->ev_used + 1];
        ctx->ev_used += 2;
    }
    e = ctx->impl == MOSAIC_ATTEND_MFMA
            ? launch_attend_mfma(ctx->dv, u0, nu, q_dev, n_q_tokens, S, ctx->stream, ev0, ev1)
            : launch_attend_valu(ctx->dv, u0, nu, q_dev, n_q_tokens, S, ctx->stream, ev0, ev1);
    if (e != hipSuccess) return fail_hip(ctx, e, "attend launch");
    e = launch_attend_combine(ctx->dv, u0, nu, n_q_tokens, S, out_dev, lse_dev, ctx->stream);
    if (e != hipSuccess) return fail_hip(ctx, e, "combine launch");
    ctx->stats.attend_calls += 1;
    ctx->stats.last_n_splits = S;
    return MOSAIC_OK;
}

static int d2h(mosaic_ctx *ctx, void *dst, const void *src, size_t bytes) {
    hipError_t e = hipMemcpyAsync(dst, src, bytes, hipMemcpyDeviceToHost, ctx->stream);
    if (e != hipSuccess) return fail_hip(ctx, e, "hipMemcpyAsync D2H");
    return MOSAIC_OK;
}
static int sync(mosaic_ctx *ctx) {
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

int32_t mosaic_get_selection(mosaic_ctx *ctx, int32_t layer, int32_t *ids, int32_t *n_ids,
                             double *scores, int32_t *tok_idx, int64_t tok_cap, int32_t *n_tok) {
    if (!ctx) return MOSAIC_EINVAL;
    const DeviceView &dv = ctx->dv;
    if (layer < 0 || layer >= dv.L) return fail(ctx, MOSAIC_EINVAL, "layer out of range");
    if (ctx->sel_epoch[layer] != ctx->epoch) return fail(ctx, MOSAIC_ENOTREADY, "no current selection for this layer");
    const int u0 = layer * dv.Hkv, H = dv.Hkv;
    int rc;
    if (ids && (rc = d2h(ctx, ids, dv.ids + (size_t)u0 * dv.k, (size_t)H * dv.k * 4)) != MOSAIC_OK) return rc;
    if (n_ids && (rc = d2h(ctx, n_ids, dv.n_ids + u0, (size_t)H * 4)) != MOSAIC_OK) return rc;
    if (scores && (rc = d2h(ctx, scores, dv.scores + (size_t)u0 * dv.C, (size_t)H * dv.C * 8)) != MOSAIC_OK) return rc;
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

int32_t mosaic_get_stats(mosaic_ctx *ctx, mosaic_stats *stats) {
    if (!ctx || !stats) return MOSAIC_EINVAL;
    *stats = ctx->stats;
    return MOSAIC_OK;
}

int32_t mosaic_profile_enable(mosaic_ctx *ctx, int32_t on) {
    if (!ctx) return MOSAIC_EINVAL;
    ctx->profile = on != 0;
    return MOSAIC_OK;
}

int32_t mosaic_profile_read(mosaic_ctx *ctx, double *attend_kernel_ms, int64_t *launches) {
    if (!ctx) return MOSAIC_EINVAL;
    int rc = sync(ctx);
    if (rc != MOSAIC_OK) return rc;
    double total = 0.0;
    for (size_t i = 0; i + 1 < ctx->ev_used; i += 2) {
        float ms = 0.f;
        hipError_t e = hipEventElapsedTime(&ms, ctx->ev[i], ctx->ev[i + 1]);
        if (e != hipSuccess) return fail_hip(ctx, e, "hipEventElapsedTime");
        total += ms;
    }
    if (attend_kernel_ms) *attend_kernel_ms = total;
    if (launches) *launches = (int64_t)(ctx->ev_used / 2);
    ctx->ev_used = 0;
    return MOSAIC_OK;
}

const char *mosaic_last_error(const mosaic_ctx *ctx) {
    return ctx ? ctx->err.c_str() : g_create_err.c_str();
}

} // extern "C"
