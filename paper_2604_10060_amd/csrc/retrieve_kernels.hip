// Query Retrieval, selection part (paper Sec. V-C; top-K of Sec. VII-B):
// one workgroup per unit computes the mean query, scores every representative
// of the GPU-resident index, ranks them, and lists the pages of the chosen
// clusters.  Nothing is copied: attention later reads the pages in place.
#include "mosaic_internal.h"
#include "maintain_device.h"
#include "topk_device.h"

namespace mosaic {

namespace {

// (every call site has all 16 lanes of the group active; k_decode_fused uses the same sum)
__device__ __forceinline__ double group16_sum(double x) { return row16_sum(x); }

template <typename E> __device__ __forceinline__ double to_f64(E v);
template <> __device__ __forceinline__ double to_f64<float>(float v) { return (double)v; }
template <> __device__ __forceinline__ double to_f64<unsigned short>(unsigned short v) {
    return (double)bf16_to_f32(v);
}

// grid (n_units), kRetrBlock threads.  u0 is a multiple of Hkv.
// A single workgroup per unit is latency-bound, so it is wide (1024 threads) and
// every global load whose address does not depend on an earlier result (query
// rows, sizes, norms, the representative rows, and the first frames'
// assignment/position entries) is issued up front, unconditionally; what
// follows runs out of LDS and registers.
constexpr int kRetrBlock = 1024;

// ---------------------------------------------------------------------------
// Mean query of a unit, first half: per-wavefront partial sums of the Tq * G
// query rows of KV head h (fp64), written to wpart[wave][channel].  A thread
// owns 8 consecutive channels (one 16-byte load per row for bf16, two for
// fp32) of every (BLK / (D/8))-th row, with eight rows' loads in flight (row
// index clamped, loads unconditional), so a 256-token question costs a handful
// of memory round trips and a decode query exactly one.  The caller adds the 16
// wavefront partials after a barrier.
// ---------------------------------------------------------------------------
template <typename E> __device__ __forceinline__ void load8_f64(const E *p, double (&out)[8]);
template <> __device__ __forceinline__ void load8_f64<float>(const float *p, double (&out)[8]) {
    const float4 a = *reinterpret_cast<const float4 *>(p), b = *reinterpret_cast<const float4 *>(p + 4);
    out[0] = a.x; out[1] = a.y; out[2] = a.z; out[3] = a.w; out[4] = b.x; out[5] = b.y; out[6] = b.z; out[7] = b.w;
}
template <> __device__ __forceinline__ void load8_f64<unsigned short>(const unsigned short *p, double (&out)[8]) {
    const uint4 a = *reinterpret_cast<const uint4 *>(p);
    const unsigned int w[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        out[2 * i] = (double)__uint_as_float(w[i] << 16);
        out[2 * i + 1] = (double)__uint_as_float(w[i] & 0xffff0000u);
    }
}

template <typename E, int D>
__device__ __forceinline__ void mean_query_partials(const E *q, int lc, int h, int Tq, int G, int Hq,
                                                    double (*wpart)[D]) {
    constexpr int BLK = kRetrBlock, LPR = D / 8, NPART = BLK / LPR, UN = 8;
    const int tid = threadIdx.x, lane = tid % 64, wave = tid / 64;
    const int c8 = tid % LPR, part = tid / LPR, R = Tq * G;
    const E *qb = q + (size_t)lc * Tq * Hq * D + (size_t)h * G * D + 8 * c8;
    double a[8] = {0.0, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0};
    for (int r0 = part; r0 < R; r0 += UN * NPART) {
        double v[UN][8];
#pragma unroll
        for (int x = 0; x < UN; ++x) {
            const int rr = min(r0 + x * NPART, R - 1), t = rr / G, g = rr - t * G;
            load8_f64<E>(qb + ((size_t)t * Hq + g) * D, v[x]);
        }
#pragma unroll
        for (int x = 0; x < UN; ++x)
            if (r0 + x * NPART < R) {
#pragma unroll
                for (int e = 0; e < 8; ++e) a[e] += v[x][e];
            }
    }
    // the 64 / LPR parts inside a wavefront
#pragma unroll
    for (int e = 0; e < 8; ++e) {
#pragma unroll
        for (int o = LPR; o < 64; o <<= 1) a[e] += __shfl_xor(a[e], o, 64);
    }
    if (lane < LPR) {
#pragma unroll
        for (int e = 0; e < 8; ++e) wpart[wave][8 * c8 + e] = a[e];
    }
}

// NESTED (paper Sec. V-C "Two-Stage Retrieval"): the mean query is first scored against the
// unit's P partition representatives; only the clusters of the top_p best partitions are then
// scored (the rest count as empty: their rows are never read) and ranked.
template <typename E, int D, bool NESTED>
__global__ __launch_bounds__(kRetrBlock) void k_retrieve(DeviceView dv, int u0, const E *q, int Tq,
                                                         int n_frames, int score_mode, bool write_pages) {
    constexpr int BLK = kRetrBlock;
    constexpr int EPL = D / 16;        // doubles per lane in a 16-lane row group
    constexpr int RPP = BLK / 16;      // representative rows per pass
    constexpr int FPT = 4;             // frames per thread prefetched for the page-list scatter
    constexpr int RPF = 2;             // passes of representative rows prefetched into registers
    const int uc = blockIdx.x, u = u0 + uc, tid = threadIdx.x;
    const int C = dv.C, G = dv.G, Hq = dv.Hq, k = dv.k;
    const int lc = uc / dv.Hkv, h = u % dv.Hkv;
    const int lr = tid % 16, row0 = tid / 16;
    __shared__ double qbar[D];
    __shared__ double qpart[BLK / 64][D];   // per-wavefront partial sums of the query rows
    __shared__ double sc_sh[1024];
    __shared__ double rn_sh[1024];
    __shared__ int n_sh[1024];
    __shared__ int rank_sh[1024];   // selection rank of cluster j, or -1
    __shared__ int cnt_sh[1024];
    __shared__ int wcnt_sh[1024];   // members inside the local window
    __shared__ int ids_sh[1024];
    __shared__ int off_sh[1025];
    __shared__ TopkShared tk_sh;
    __shared__ double ps_sh[64];    // first-stage scores
    __shared__ int psel_sh[64];     // partition kept by the first stage
    __shared__ int p_live_sh;
    const double *r = dv.r + (size_t)u * C * D;
    const double *rn = dv.rnorm + (size_t)u * C;
    const int *n = dv.n + (size_t)u * C;
    const int *assign = dv.assign + (size_t)u * dv.F;
    const int *pos = dv.pos + (size_t)u * dv.F;

    // ---- independent loads ----
    int fa[FPT], fp[FPT];
#pragma unroll
    for (int i = 0; i < FPT; ++i) {
        const int f = tid + BLK * i;
        const bool in = write_pages && f < n_frames;
        fa[i] = in ? assign[f] : -1;
        fp[i] = in ? pos[f] : 0;
    }
    // (C <= 1024 = BLK: one table entry per thread, loaded into registers now and stored to LDS only after every
    // other load has been issued: a loop here would be a basic block of its own, and its LDS stores would wait for
    // its loads before the loads below could start)
    int n_reg = 0;
    double rn_reg = 0.0;
    if (tid < C) { n_reg = n[tid]; rn_reg = rn[tid]; }
    if (tid == 0) tk_sh.n_live = 0;
    // local-window augmentation (Sec. V-C): the w most recent frames are listed once, after the
    // clusters; they are the last members of their clusters (ranks ascend with the frame id), so
    // a cluster's list is simply cut short by its number of window members
    const int w0 = write_pages && dv.aug_window > 0 ? max(0, n_frames - dv.aug_window) : n_frames;
    int wa = -1;
    if (w0 + tid < n_frames) wa = assign[w0 + tid];          // aug_window <= 1024 (checked at create)
    // representative rows of the first RPF passes (row index clamped, loads unconditional)
    double rpre[RPF][EPL];
    if constexpr (!NESTED) {
#pragma unroll
        for (int i = 0; i < RPF; ++i) {
            if (RPP * i < C) {              // workgroup-uniform: passes beyond the table are not loaded
                const double *rj = r + (size_t)min(row0 + RPP * i, C - 1) * D + lr * EPL;
#pragma unroll
                for (int e = 0; e < EPL; ++e) rpre[i][e] = rj[e];
            }
        }
    }
    // first stage: the partition rows (P <= 64: one 16-lane group each), loaded up front as well
    double ppre[EPL];
    int pn_pre = 0;
    double prn_pre = 0.0;
    if constexpr (NESTED) {
        const int pj = min(row0, dv.P - 1);
        const double *prow = dv.pr + ((size_t)u * dv.P + pj) * D + lr * EPL;
#pragma unroll
        for (int e = 0; e < EPL; ++e) ppre[e] = prow[e];
        pn_pre = dv.pn[(size_t)u * dv.P + pj];
        prn_pre = dv.prn[(size_t)u * dv.P + pj];
        if (tid == 0) p_live_sh = 0;
    }
    // mean query over the Tq tokens and the G query heads of this KV head
    const int R = Tq * G;
    if (R <= 16) {
        // A decode step or a short question: a thread per channel adds the rows in order, every row's load in flight
        // at once, beside the loads above: the prologue is one trip to memory.  (The general path below costs a
        // decode step two trips and a reduction through LDS permutes for seven rows.)
        if (tid < D) {
            const E *qb = q + (size_t)lc * Tq * Hq * D + (size_t)h * G * D + tid;
            E v[16];
#pragma unroll
            for (int x = 0; x < 16; ++x) {
                const int rr = min(x, R - 1), t = rr / G, g = rr - t * G;
                v[x] = qb[((size_t)t * Hq + g) * D];
            }
            double acc = 0.0;
#pragma unroll
            for (int x = 0; x < 16; ++x)
                if (x < R) acc += to_f64<E>(v[x]);
            qbar[tid] = acc / (double)R;
        }
        if (tid < C) { n_sh[tid] = n_reg; rn_sh[tid] = rn_reg; cnt_sh[tid] = 0; wcnt_sh[tid] = 0; }
        __syncthreads();
        if (wa >= 0) atomicAdd(&wcnt_sh[wa], 1);         // (read after the scores' barrier at the earliest)
    } else {
        if (tid < C) { n_sh[tid] = n_reg; rn_sh[tid] = rn_reg; cnt_sh[tid] = 0; wcnt_sh[tid] = 0; }
        mean_query_partials<E, D>(q, lc, h, Tq, G, Hq, qpart);
        __syncthreads();
        if (wa >= 0) atomicAdd(&wcnt_sh[wa], 1);
        if (tid < D) {
            double acc = 0.0;
#pragma unroll
            for (int p = 0; p < BLK / 64; ++p) acc += qpart[p][tid];
            qbar[tid] = acc / (double)R;
        }
        __syncthreads();
    }
    if constexpr (NESTED) {
        const int P = dv.P, top_p = dv.top_p;
        if (row0 < P) {
            double p = 0.0;
#pragma unroll
            for (int e = 0; e < EPL; ++e) p += qbar[lr * EPL + e] * ppre[e];
            p = group16_sum(p);
            if (lr == 0) {
                double sc = -INFINITY;
                if (pn_pre > 0) {
                    sc = score_mode == 1 ? p : (prn_pre == 0.0 ? 0.0 : p / prn_pre);
                    atomicAdd(&p_live_sh, 1);
                }
                ps_sh[row0] = sc;
                dv.pscores[(size_t)u * P + row0] = sc;
            }
        }
        __syncthreads();
        if (tid < P) {      // rank by (score descending, id ascending); empty partitions carry -inf
            const double sj = ps_sh[tid];
            int c = 0;
            for (int i = 0; i < P; ++i) {
                const double si = ps_sh[i];
                c += (si > sj) || (si == sj && i < tid);
            }
            const bool keep = sj != -INFINITY && c < top_p;
            psel_sh[tid] = keep;
            if (keep) dv.pids[(size_t)u * top_p + c] = tid;
        }
        const int n_pk = min(top_p, p_live_sh);
        for (int i = n_pk + tid; i < top_p; i += BLK) dv.pids[(size_t)u * top_p + i] = -1;
        if (tid == 0) dv.n_pids[u] = n_pk;
        __syncthreads();
        for (int j = tid; j < C; j += BLK)
            if (!psel_sh[j / dv.Cs]) n_sh[j] = 0;        // pruned: treated as empty from here on
        __syncthreads();
    }
    // score_j = (qbar . r_j) / |r_j|   (plain dot product in score_mode 1)
    auto finish_row = [&](int j, double p, bool reduced = false) {
        if (!reduced) p = group16_sum(p);
        if (lr == 0) {
            double sc = -INFINITY;
            if (n_sh[j] > 0) {
                const double nr = rn_sh[j];
                sc = score_mode == 1 ? p : (nr == 0.0 ? 0.0 : p / nr);
            }
            sc_sh[j] = sc;        // (goes to dv.scores at the end: a store here would be waited for at the next barrier)
        }
    };
    if constexpr (NESTED) {
        for (int j = row0; j < C; j += RPP) {
            double p = 0.0;
            if (n_sh[j] > 0) {                           // uniform within the 16-lane group
                const double *rj = r + (size_t)j * D + lr * EPL;
#pragma unroll
                for (int e = 0; e < EPL; ++e) p += qbar[lr * EPL + e] * rj[e];
            }
            finish_row(j, p);
        }
    } else {
        // the prefetched rows: all reductions first, without lane-dependent branches, so that the
        // rows' chains interleave (a row beyond the table repeats the last one and is not stored)
        double pv[RPF];
#pragma unroll
        for (int i = 0; i < RPF; ++i) {
            pv[i] = 0.0;
            if (RPP * i < C) {                                // workgroup-uniform
#pragma unroll
                for (int e = 0; e < EPL; ++e) pv[i] += qbar[lr * EPL + e] * rpre[i][e];
                pv[i] = group16_sum(pv[i]);
            }
        }
        {   // lane i of the group finishes prefetched row i: one pass through the division instead of RPF (the
            // workgroup's sixteen wavefronts share four SIMDs, so every instruction of a phase counts four times)
            static_assert(RPF == 2, "the select below is written for two prefetched passes");
            const int j = row0 + RPP * lr;
            if (lr < RPF && j < C) {
                const double p = lr == 0 ? pv[0] : pv[1];
                double sc = -INFINITY;
                if (n_sh[j] > 0) {
                    const double nr = rn_sh[j];
                    sc = score_mode == 1 ? p : (nr == 0.0 ? 0.0 : p / nr);
                }
                sc_sh[j] = sc;
            }
        }
        for (int j = row0 + RPP * RPF; j < C; j += RPP) {
            const double *rj = r + (size_t)j * D + lr * EPL;
            double p = 0.0;
#pragma unroll
            for (int e = 0; e < EPL; ++e) p += qbar[lr * EPL + e] * rj[e];
            finish_row(j, p);
        }
    }
    __syncthreads();
    // ranks of the k best non-empty clusters by (score descending, id ascending); empty and
    // pruned clusters have n_sh = 0 and take no part
    const int n_live = topk_rank(sc_sh, n_sh, C, k, rank_sh, ids_sh, cnt_sh, off_sh, tk_sh);
    const int n_ids = min(k, n_live);
    int run = 0;
    if (tid < 64) {      // page offsets of the selected clusters: running sums of their sizes, 64 at a time
        for (int i0 = 0; i0 < n_ids; i0 += 64) {
            const int i = i0 + tid;
            const int sz = i < n_ids ? n_sh[ids_sh[i]] - wcnt_sh[ids_sh[i]] : 0;
            int incl = sz;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const int t = __shfl_up(incl, o, 64);
                if (tid >= o) incl += t;
            }
            if (i < n_ids) off_sh[i + 1] = run + incl;
            run += __shfl(incl, 63, 64);
        }
        if (tid == 0) off_sh[0] = 0;
    }
    __syncthreads();
    // Everything this launch leaves in global memory is stored from here on, after the last barrier: a barrier
    // waits for the acknowledgement of the wavefront's outstanding stores (1-2 us for lines that are not in L2).
    if (tid == 0) {
        dv.n_ids[u] = n_ids;
        if (write_pages) dv.n_sel[u] = run + (n_frames - w0);
    }
    for (int i = tid; i < k; i += BLK) dv.ids[(size_t)u * k + i] = i < n_ids ? ids_sh[i] : -1;
    if (tid < C) dv.scores[(size_t)u * C + tid] = sc_sh[tid];
    if (!write_pages) return;     // host tier: the host maps clusters to cache slots
    // page list: clusters in selection order, member frames ascending
    int *sel = dv.sel_pages + (size_t)u * dv.F;
#pragma unroll
    for (int i = 0; i < FPT; ++i) {   // (no early exits: the LDS look-ups of the batch overlap)
        const int rk = rank_sh[max(fa[i], 0)];
        const int p = off_sh[max(rk, 0)] + fp[i];
        if (fa[i] >= 0 && tid + BLK * i < w0 && rk >= 0) sel[p] = tid + BLK * i;
    }
    for (int f = tid + BLK * FPT; f < w0; f += BLK) {
        const int c = assign[f];
        if (c < 0) continue;
        const int rk = rank_sh[c];
        if (rk >= 0) sel[off_sh[rk] + pos[f]] = f;
    }
    if (w0 + tid < n_frames) sel[off_sh[n_ids] + tid] = w0 + tid;      // the local window, ascending
}

// ---------------------------------------------------------------------------
// Query Retrieval with the deferred-split maintainer (paper Sec. VI-B, Alg. 1):
// the representative set is the non-empty clusters plus the buffered singletons
// (a singleton's representative is its own frame summary; id = C + buffer slot);
// after the page list of this query has been written, the selected clusters
// become the resident set and every selected cluster that carries a lazy-split
// flag has its buffered entries merged and its split carried out (lines 12-17),
// in selection order.  grid (n_units), kRetrBlock threads; C + buf_max <= 1024.
// ---------------------------------------------------------------------------
template <typename E, int D>
__global__ __launch_bounds__(kRetrBlock) void k_retrieve_deferred(DeviceView dv, int u0, const E *q, int Tq,
                                                                  int n_frames, int score_mode) {
    constexpr int BLK = kRetrBlock;
    constexpr int EPL = D / 16, RPP = BLK / 16;
    const int uc = blockIdx.x, u = u0 + uc, tid = threadIdx.x;
    const int C = dv.C, G = dv.G, Hq = dv.Hq, k = dv.k, SC = dv.SC;
    const int lc = uc / dv.Hkv, h = u % dv.Hkv;
    const int lr = tid % 16, row0 = tid / 16;
    __shared__ double qbar[D];
    __shared__ double qpart[BLK / 64][D];   // per-wavefront partial sums of the query rows
    __shared__ double sc_sh[1024];
    __shared__ int n_sh[1024];      // size in frames of a representative's cluster (0 = not live)
    __shared__ int rank_sh[1024];
    __shared__ int cnt_sh[1024];
    __shared__ int ids_sh[1024];
    __shared__ int off_sh[1025];
    __shared__ TopkShared tk_sh;
    __shared__ SplitShared<D> split_sh;
    const double *r = dv.r + (size_t)u * C * D;
    const double *rn = dv.rnorm + (size_t)u * C;
    const int *n = dv.n + (size_t)u * C;
    int *assign = dv.assign + (size_t)u * dv.F;
    const int *pos = dv.pos + (size_t)u * dv.F;
    int *buf_frame = dv.buf_frame + (size_t)u * dv.buf_max;
    int *buf_owner = dv.buf_owner + (size_t)u * dv.buf_max;
    const int nb = dv.n_buf[u], R = C + nb;

    for (int j = tid; j < 1024; j += BLK) { n_sh[j] = j < C ? n[j] : (j < R ? 1 : 0); cnt_sh[j] = 0; }
    if (tid == 0) tk_sh.n_live = 0;
    mean_query_partials<E, D>(q, lc, h, Tq, G, Hq, qpart);
    __syncthreads();
    if (tid < D) {
        double acc = 0.0;
#pragma unroll
        for (int p = 0; p < BLK / 64; ++p) acc += qpart[p][tid];
        qbar[tid] = acc / (double)(Tq * G);
    }
    __syncthreads();
    // scores of clusters and singletons
    for (int j = row0; j < SC; j += RPP) {
        double sc = -INFINITY;
        if (j < R && n_sh[j] > 0) {
            const double *rj = (j < C ? r + (size_t)j * D
                                      : dv.summ + ((size_t)u * dv.F + buf_frame[j - C]) * D) + lr * EPL;
            double p = 0.0, sq = 0.0;
#pragma unroll
            for (int e = 0; e < EPL; ++e) { p += qbar[lr * EPL + e] * rj[e]; sq += rj[e] * rj[e]; }
            p = group16_sum(p);
            sq = group16_sum(sq);
            const double nr = j < C ? rn[j] : sqrt(sq);
            sc = score_mode == 1 ? p : (nr == 0.0 ? 0.0 : p / nr);
        }
        if (lr == 0) {
            if (j < 1024) sc_sh[j] = sc;
            dv.scores[(size_t)u * SC + j] = sc;
        }
    }
    __syncthreads();
    // ranks of the k best live representatives by (score descending, id ascending)
    const int n_live = topk_rank(sc_sh, n_sh, R, k, rank_sh, ids_sh, cnt_sh, off_sh, tk_sh);
    const int n_ids = min(k, n_live);
    if (tid == 0) {
        int o = 0;
        off_sh[0] = 0;
        for (int i = 0; i < n_ids; ++i) { o += n_sh[ids_sh[i]]; off_sh[i + 1] = o; }
        dv.n_ids[u] = n_ids;
        dv.n_sel[u] = o;
    }
    for (int i = tid; i < k; i += BLK) dv.ids[(size_t)u * k + i] = i < n_ids ? ids_sh[i] : -1;
    __syncthreads();
    // page list: representatives in selection order, member frames ascending
    int *sel = dv.sel_pages + (size_t)u * dv.F;
    for (int f = tid; f < n_frames; f += BLK) {
        const int c = assign[f];
        if (c < 0) continue;
        const int rk = rank_sh[c];
        if (rk >= 0) sel[off_sh[rk] + pos[f]] = f;
    }
    for (int b = tid; b < nb; b += BLK) {
        const int rk = rank_sh[C + b];
        if (rk >= 0) sel[off_sh[rk]] = buf_frame[b];
    }
    // the selection is what is on the GPU from now on (host tier: the host sends the flags of its
    // cluster cache's directory instead)
    if (dv.tier == MOSAIC_TIER_HBM)
        for (int j = tid; j < C; j += BLK) dv.resident[(size_t)u * C + j] = rank_sh[j] >= 0;
    __syncthreads();
    // deferred splits of the selected clusters
    for (int i = 0; i < n_ids; ++i) {
        const int j = ids_sh[i];
        if (j >= C || !dv.lazy[(size_t)u * C + j]) continue;      // workgroup-uniform
        __syncthreads();
        {   // the cluster's buffered entries join it, the others close ranks in order: one entry per
            // thread (C + buf_max <= 1024), kept entries placed by an exclusive scan over the workgroup
            const int cur = dv.n_buf[u];
            const bool have = tid < cur;
            int fr = 0, ow = -1;
            if (have) { fr = buf_frame[tid]; ow = buf_owner[tid]; }
            const bool mine = have && ow == j;
            if (mine) assign[fr] = j;
            const int keep = have && !mine;
            int total;
            const int w = mt_block_excl_scan<D>(keep, split_sh, &total);   // (its barriers come after every load above)
            if (keep) { buf_frame[w] = fr; buf_owner[w] = ow; }
            if (tid == 0) {
                dv.n_buf[u] = total;
                dv.lazy[(size_t)u * C + j] = 0;
            }
        }
        __syncthreads();
        const int fresh = mt_split_cluster<D>(dv, u, j, n_frames, true, split_sh);
        if (tid == 0 && fresh >= 0) dv.mt_cnt[(size_t)u * 4 + 1] += 1;
        __syncthreads();
    }
}

// Token-index expansion of the page lists (observer only).  grid (n_units).
__global__ __launch_bounds__(kBlock) void k_expand_tok_idx(DeviceView dv, int u0) {
    const int uc = blockIdx.x, u = u0 + uc, T = dv.T;
    const long long total = (long long)dv.n_sel[u] * T;
    const int *sel = dv.sel_pages + (size_t)u * dv.F;
    int *out = dv.tok_scratch + (size_t)uc * dv.F * T;
    for (long long i = threadIdx.x; i < total; i += kBlock)
        out[i] = sel[i / T] * T + (int)(i % T);
}

} // namespace

template <bool NESTED>
static void launch_retrieve_t(const DeviceView &dv, int u0, int n_units, const void *q, int Tq,
                              int n_frames, int score_mode, bool write_pages, hipStream_t s) {
    if (dv.esize == 4) {
        if (dv.D == 64) k_retrieve<float, 64, NESTED><<<n_units, kRetrBlock, 0, s>>>(dv, u0, (const float *)q, Tq, n_frames, score_mode, write_pages);
        else k_retrieve<float, 128, NESTED><<<n_units, kRetrBlock, 0, s>>>(dv, u0, (const float *)q, Tq, n_frames, score_mode, write_pages);
    } else {
        if (dv.D == 64) k_retrieve<unsigned short, 64, NESTED><<<n_units, kRetrBlock, 0, s>>>(dv, u0, (const unsigned short *)q, Tq, n_frames, score_mode, write_pages);
        else k_retrieve<unsigned short, 128, NESTED><<<n_units, kRetrBlock, 0, s>>>(dv, u0, (const unsigned short *)q, Tq, n_frames, score_mode, write_pages);
    }
}

hipError_t launch_retrieve(const DeviceView &dv, int u0, int n_units, const void *q, int Tq,
                           int n_frames, int score_mode, bool write_pages, hipStream_t s) {
    if (dv.P > 0) launch_retrieve_t<true>(dv, u0, n_units, q, Tq, n_frames, score_mode, write_pages, s);
    else launch_retrieve_t<false>(dv, u0, n_units, q, Tq, n_frames, score_mode, write_pages, s);
    return hipGetLastError();
}

hipError_t launch_retrieve_deferred(const DeviceView &dv, int u0, int n_units, const void *q, int Tq,
                                    int n_frames, int score_mode, hipStream_t s) {
    if (dv.esize == 4) {
        if (dv.D == 64) k_retrieve_deferred<float, 64><<<n_units, kRetrBlock, 0, s>>>(dv, u0, (const float *)q, Tq, n_frames, score_mode);
        else k_retrieve_deferred<float, 128><<<n_units, kRetrBlock, 0, s>>>(dv, u0, (const float *)q, Tq, n_frames, score_mode);
    } else {
        if (dv.D == 64) k_retrieve_deferred<unsigned short, 64><<<n_units, kRetrBlock, 0, s>>>(dv, u0, (const unsigned short *)q, Tq, n_frames, score_mode);
        else k_retrieve_deferred<unsigned short, 128><<<n_units, kRetrBlock, 0, s>>>(dv, u0, (const unsigned short *)q, Tq, n_frames, score_mode);
    }
    return hipGetLastError();
}

hipError_t launch_expand_tok_idx(const DeviceView &dv, int u0, int n_units, hipStream_t s) {
    k_expand_tok_idx<<<n_units, kBlock, 0, s>>>(dv, u0);
    return hipGetLastError();
}

} // namespace mosaic

