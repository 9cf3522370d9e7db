// One decode step of one layer (paper Sec. V-C selection + Sec. V-A (2) attention) in ONE
// launch with size-proportional KV splits: the separate selection launch (one workgroup per
// unit) is folded into the attention launch.  An option, not the default path: measured on 28
// per-layer launches of ~118 MB each, this kernel takes 39.7 us where the selection and the
// attention launches take 9.3 + 22.5 us, because everything a waiting workgroup reads -- flag,
// page ids -- was written on another XCD in the same launch and has to bypass the L2s, and
// those round trips (store acknowledged, flag seen, page id read) are serial and cost more than
// the launch they replace.  It stays selectable so that the measurement can be repeated.
//
// grid B >= n_units workgroups of 256 threads.  Workgroup w < n_units is the LEADER of unit
// u0 + w: it computes that unit's selection (mean query, scores, ranking, page list: the
// arithmetic of k_retrieve / k_decode_fused, lane for lane) and publishes the page list with
// agent-scope (write-through) stores, then raises the unit's flag.
// The flag is one 64-bit word (launch number << 32 | retrieved pages), so a waiter that sees
// the flag has the size as well.  Every workgroup -- the leaders too, afterwards -- waits
// until all units of the launch are published (lane i of its first wavefront polls unit i:
// one memory round trip when everything is ready), shares the B workgroups out over the units
// in proportion to the sizes (split_slot, as k_attend_decode_mfma does after a separate
// selection launch) and reduces its share of the pages exactly like k_attend_decode_mfma; the
// combine kernel follows.
//
// The wait cannot deadlock: leaders wait for nobody before they publish, and they are the
// first workgroups of the grid, which the dispatcher starts first, so whenever a waiter
// occupies a compute unit the leaders have been started as well.  The wait is bounded all the
// same (kSpinLimit polls, tens of milliseconds): a workgroup that gives up sets sync_err and
// leaves, and the next reading of the statistics reports it.
#include "mosaic_internal.h"
#include "attend_mfma_device.h"

namespace mosaic {

namespace {

constexpr int kLayerMaxC = 256;
constexpr int kSpinLimit = 1 << 18;      // polls of ~1 us: a few tenths of a second

// Selection of unit u by one 256-thread workgroup; everything other workgroups of this launch
// read (retrieved size, page list) goes out with agent-scope stores.
template <int D>
__device__ __forceinline__ void leader_select(const DeviceView &dv, int u, int lc, int h, const unsigned short *q,
                                              int Tq, int n_frames, int score_mode, int *n_sel_out) {
    constexpr int EPL = D / 16, NG = kBlock / 16, RPF = 8, FPT = 8;
    const int tid = threadIdx.x, wave = tid / 64, lane = tid % 64;
    const int lr = tid % 16, grp = tid / 16;
    const int C = dv.C, k = dv.k, G = dv.G, Hq = dv.Hq, F = dv.F, R = Tq * G;
    __shared__ double qbar[D];
    __shared__ double sc_sh[kLayerMaxC], rn_sh[kLayerMaxC];
    __shared__ int n_sh[kLayerMaxC], rank_sh[kLayerMaxC], cnt_sh[kLayerMaxC], ids_sh[kLayerMaxC], off_sh[kLayerMaxC + 1];
    __shared__ int n_live_sh;
    const double *r = dv.r + (size_t)u * C * D;
    const int *assign = dv.assign + (size_t)u * F;
    const int *pos = dv.pos + (size_t)u * F;

    // ---- independent loads, all issued up front ----
    int fa[FPT], fp[FPT];
#pragma unroll
    for (int i = 0; i < FPT; ++i) {
        const int f = tid + kBlock * i;
        fa[i] = f < n_frames ? assign[f] : -1;
        fp[i] = f < n_frames ? pos[f] : 0;
    }
    for (int j = tid; j < C; j += kBlock) {
        n_sh[j] = dv.n[(size_t)u * C + j];
        rn_sh[j] = dv.rnorm[(size_t)u * C + j];
        cnt_sh[j] = 0;
    }
    if (tid == 0) n_live_sh = 0;
    double rpre[RPF][EPL];
#pragma unroll
    for (int i = 0; i < RPF; ++i) {
        if (NG * i < C) {               // workgroup-uniform: passes beyond the table are not loaded
            const double *rj = r + (size_t)min(grp + NG * i, C - 1) * D + lr * EPL;
#pragma unroll
            for (int e = 0; e < EPL; ++e) rpre[i][e] = rj[e];
        }
    }
    if (tid < D) {      // mean query over the Tq tokens and the G query heads of this KV head (R <= 16)
        const unsigned short *qb = q + (size_t)lc * Tq * Hq * D + (size_t)h * G * D + tid;
        double a = 0.0;
        for (int r0 = 0; r0 < R; r0 += 8) {
            unsigned short v[8];
#pragma unroll
            for (int x = 0; x < 8; ++x) {
                const int rr = min(r0 + x, R - 1), t = rr / G, gg = rr - t * G;
                v[x] = qb[((size_t)t * Hq + gg) * D];
            }
#pragma unroll
            for (int x = 0; x < 8; ++x)
                if (r0 + x < R) a += (double)bf16_to_f32(v[x]);
        }
        qbar[tid] = a / (double)R;
    }
    __syncthreads();
    // ---- scores: score_j = (qbar . r_j) / |r_j|   (plain dot product in score_mode 1) ----
#pragma unroll
    for (int i = 0; i < RPF; ++i) {
        const int j = grp + NG * i;
        if (NG * i < C) {                                     // workgroup-uniform
            double p = 0.0;
#pragma unroll
            for (int e = 0; e < EPL; ++e) p += qbar[lr * EPL + e] * rpre[i][e];
            p = row16_sum(p);
            if (lr == 0 && j < C) sc_sh[j] = p;
        }
    }
    for (int j = grp + NG * RPF; j < C; j += NG) {
        const double *rj = r + (size_t)j * D + lr * EPL;
        double p = 0.0;
#pragma unroll
        for (int e = 0; e < EPL; ++e) p += qbar[lr * EPL + e] * rj[e];
        p = row16_sum(p);
        if (lr == 0) sc_sh[j] = p;
    }
    __syncthreads();
    float *key_sh = reinterpret_cast<float *>(off_sh);     // (the page offsets are formed after the ranking)
    if (tid < C) {
        double sc = -INFINITY;
        if (n_sh[tid] > 0) {
            const double p = sc_sh[tid], nr = rn_sh[tid];
            sc = score_mode == 1 ? p : (nr == 0.0 ? 0.0 : p / nr);
        }
        sc_sh[tid] = sc;
        key_sh[tid] = (float)sc;          // fp32 rounding for the pair count below
        dv.scores[(size_t)u * dv.SC + tid] = sc;
    }
    __syncthreads();
    // ---- ranks by (score descending, id ascending) among the non-empty clusters: pairs compared on
    //      the fp32 roundings (monotone), collisions settled exactly in fp64 ----
    {
        const int pl = 31 - __clz(kBlock / C);
        const int j = tid >> pl, part = tid & ((1 << pl) - 1);
        if (j < C && n_sh[j] > 0) {
            const float fj = key_sh[j];
            const int i0 = (C * part) >> pl, i1 = (C * (part + 1)) >> pl;
            int c = 0, ceq = 0;
#pragma unroll 8
            for (int i = i0; i < i1; ++i) {
                const float fi = key_sh[i];
                c += fi > fj;
                ceq += fi == fj;
            }
            atomicAdd(&cnt_sh[j], c + (ceq << 16));     // c <= 256, ceq <= 256
        }
    }
    __syncthreads();
    {
        const bool live = tid < C && n_sh[tid] > 0;
        int rk = -1;
        if (live) {
            const int v = cnt_sh[tid];
            rk = v & 0xffff;
            if ((v >> 16) > 1) {                        // collisions (the entry itself counts once)
                const float fj = key_sh[tid];
                const double sj = sc_sh[tid];
                for (int i = 0; i < C; ++i) {
                    if (i == tid || key_sh[i] != fj) continue;
                    const double si = sc_sh[i];
                    rk += (si > sj) || (si == sj && i < tid);
                }
            }
            if (rk < k) ids_sh[rk] = tid; else rk = -1;
        }
        if (tid < C) rank_sh[tid] = rk;
        const unsigned long long lb = __ballot(live);
        if (lane == 0 && lb) atomicAdd(&n_live_sh, __popcll(lb));
    }
    __syncthreads();
    const int n_ids = min(k, n_live_sh);
    if (wave == 0) {     // page offsets of the selected clusters: running sums of their sizes, 64 at a time
        int run = 0;
        for (int i0 = 0; i0 < n_ids; i0 += 64) {
            const int i = i0 + lane;
            const int sz = i < n_ids ? n_sh[ids_sh[i]] : 0;
            int incl = sz;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const int t = __shfl_up(incl, o, 64);
                if (lane >= o) incl += t;
            }
            if (i < n_ids) off_sh[i + 1] = run + incl;
            run += __shfl(incl, 63, 64);
        }
        if (lane == 0) {
            off_sh[0] = 0;
            dv.n_ids[u] = n_ids;
            dv.n_sel[u] = run;               // (for the combine launch and the observers)
            *n_sel_out = run;
        }
    }
    for (int i = tid; i < k; i += kBlock) dv.ids[(size_t)u * k + i] = i < n_ids ? ids_sh[i] : -1;
    __syncthreads();
    // ---- page list: clusters in selection order, member frames ascending ----
    int *sel = dv.sel_pages + (size_t)u * F;
    auto place = [&](int f, int a, int ps) {
        const int rk = rank_sh[max(a, 0)];
        if (a >= 0 && rk >= 0) st_agent(sel + off_sh[rk] + ps, f);
    };
#pragma unroll
    for (int i = 0; i < FPT; ++i) place(tid + kBlock * i, fa[i], fp[i]);
    for (int f0 = tid + kBlock * FPT; f0 < n_frames; f0 += kBlock * FPT) {      // further batches of FPT loads
#pragma unroll
        for (int i = 0; i < FPT; ++i) {
            const int f = f0 + kBlock * i;
            fa[i] = f < n_frames ? assign[f] : -1;
            fp[i] = f < n_frames ? pos[f] : 0;
        }
#pragma unroll
        for (int i = 0; i < FPT; ++i) place(f0 + kBlock * i, fa[i], fp[i]);
    }
}

template <int D, bool STREAM>
__global__ __launch_bounds__(kBlock, 2) void k_decode_layer(DeviceView dv, int u0, int n_units, const unsigned short *q,
                                                            int Tq, int B, int n_frames, int score_mode, int epoch) {
    constexpr int KK = D / 32, DB = D / 16;
    const int tid = threadIdx.x, wave = tid / 64, lane = tid % 64, g = lane / 16, n = lane % 16;
    __shared__ int ok_sh, pub_sh, nsel_sh[64];
    // ---- phase 1: the leaders select and publish ----
    if ((int)blockIdx.x < n_units) {
        const int u = u0 + (int)blockIdx.x;
        leader_select<D>(dv, u, (int)blockIdx.x / dv.Hkv, u % dv.Hkv, q, Tq, n_frames, score_mode, &pub_sh);
        // every published value has left this workgroup before the flag goes up
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        if (tid == 0) st_agent(dv.sel_flag + u, ((long long)epoch << 32) | (long long)pub_sh);
    }
    // ---- everybody waits for all units of the launch (bounded; n_units <= 64) ----
    if (wave == 0) {
        int spins = 0;
        long long v = 0;
        bool mine = lane < n_units;              // still waiting for unit `lane`
        while (true) {
            if (mine) {
                v = ld_agent(dv.sel_flag + u0 + lane);
                mine = (int)(v >> 32) != epoch;
            }
            if (!__ballot(mine)) break;
            __builtin_amdgcn_s_sleep(8);
            if (++spins > kSpinLimit) break;     // (wavefront-uniform)
        }
        const bool ok = !__ballot(mine);
        nsel_sh[lane] = lane < n_units ? (int)(v & 0xffffffffll) : 0;
        if (lane == 0) {
            if (!ok) st_agent(dv.sync_err, 1);
            ok_sh = ok;
        }
    }
    __syncthreads();
    if (!ok_sh) return;
    // ---- phase 2: this workgroup's share of the retrieved pages (as k_attend_decode_mfma) ----
    const SplitSlot slot = split_slot<false>(nsel_sh, n_units, B, blockIdx.x);
    if (slot.uc < 0) return;                       // block-uniform
    const int uc = slot.uc, u = u0 + uc, split = slot.split, S = slot.S;
    const int T = dv.T, F = dv.F, cpp = dv.chunks_per_page;
    const int lc = uc / dv.Hkv, h = u % dv.Hkv, R = Tq * dv.G;
    const int *sel = dv.sel_pages + (size_t)u * F;
    const int stride = __builtin_amdgcn_readfirstlane(4 * S);
    const int first = __builtin_amdgcn_readfirstlane(split + S * wave);

    bf16x8 qf[KK];
    load_q<D>(dv, q, lc, h, Tq, n, g, qf);
    const float sl2 = 1.4426950408889634f / sqrtf((float)D);
    f32x4 acc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db) acc[db] = f32x4{0.f, 0.f, 0.f, 0.f};
    float m = -INFINITY, l = 0.f, lx = 0.f;

    const int NC = __builtin_amdgcn_readfirstlane(nsel_sh[uc]) * cpp;
    const int n_my = __builtin_amdgcn_readfirstlane(first < NC ? (NC - first + stride - 1) / stride : 0);

    bf16x8 kA[2 * KK], vA[DB], kB[2 * KK], vB[DB];
    int ccA = 0, ccB = 0;
    const int sq = __builtin_amdgcn_readfirstlane(stride / cpp), sr = __builtin_amdgcn_readfirstlane(stride % cpp);
    int lq = __builtin_amdgcn_readfirstlane(first / cpp), lr = __builtin_amdgcn_readfirstlane(first % cpp), lj = 0;
    auto lookup = [&](int &page, int &cc) {           // page and in-page chunk of the cursor's chunk
        page = __builtin_amdgcn_readfirstlane(ld_agent(sel + lq)); cc = lr;      // (published in this launch)
        if (lj + 1 < n_my) {
            ++lj; lq += sq; lr += sr;
            if (lr >= cpp) { lr -= cpp; ++lq; }
        }
    };
    auto issue = [&](int page, int cc_in, bf16x8 (&kf)[2 * KK], bf16x8 (&vf)[DB], int &cc) {
        cc = cc_in;
        issue_chunk<D, STREAM>(reinterpret_cast<const unsigned short *>(k_page(dv, u, page)),
                               reinterpret_cast<const unsigned short *>(v_page(dv, u, page)) + (size_t)cc * D * 32,
                               cc * kChunk, T, g, n, kf, vf);
    };
    auto step = [&](const bf16x8 (&kf)[2 * KK], const bf16x8 (&vf)[DB], int cc) {
        chunk_step<D>(kf, vf, qf, min(kChunk, T - cc * kChunk), g, sl2, acc, m, l, lx);
    };
    if (n_my > 0) {
        int pg, cc, pg_n, cc_n;
        lookup(pg, cc);
        lookup(pg_n, cc_n);
        issue(pg, cc, kA, vA, ccA);
        int i = 0;
        for (; i + 2 < n_my; i += 2) {
            issue(pg_n, cc_n, kB, vB, ccB);
            lookup(pg_n, cc_n);
            __builtin_amdgcn_sched_barrier(0);
            step(kA, vA, ccA);
            issue(pg_n, cc_n, kA, vA, ccA);
            lookup(pg_n, cc_n);
            __builtin_amdgcn_sched_barrier(0);
            step(kB, vB, ccB);
        }
        if (i + 2 == n_my) {
            issue(pg_n, cc_n, kB, vB, ccB);
            __builtin_amdgcn_sched_barrier(0);
            step(kA, vA, ccA);
            step(kB, vB, ccB);
        } else {
            step(kA, vA, ccA);
        }
    }
    merge_waves_store<D>(dv, acc, m, l, lx, R, (size_t)slot.base + split);
}

} // namespace

hipError_t launch_decode_layer(const DeviceView &dv, int u0, int n_units, const void *q, int Tq, int B, int n_frames,
                               int score_mode, int epoch, bool stream_kv, hipStream_t s, hipEvent_t ev0, hipEvent_t ev1) {
    const dim3 grid(B), block(kBlock);
    const unsigned short *qq = (const unsigned short *)q;
    if (stream_kv) {
        if (dv.D == 64) launch_timed(k_decode_layer<64, true>, grid, block, 0, s, ev0, ev1, dv, u0, n_units, qq, Tq, B, n_frames, score_mode, epoch);
        else launch_timed(k_decode_layer<128, true>, grid, block, 0, s, ev0, ev1, dv, u0, n_units, qq, Tq, B, n_frames, score_mode, epoch);
    } else {
        if (dv.D == 64) launch_timed(k_decode_layer<64, false>, grid, block, 0, s, ev0, ev1, dv, u0, n_units, qq, Tq, B, n_frames, score_mode, epoch);
        else launch_timed(k_decode_layer<128, false>, grid, block, 0, s, ev0, ev1, dv, u0, n_units, qq, Tq, B, n_frames, score_mode, epoch);
    }
    return hipGetLastError();
}

} // namespace mosaic
