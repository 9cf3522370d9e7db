// Attention over the retrieved KV on the matrix cores (bf16 pages); paper
// Sec. V-A (2).  The G*Tq query rows of a unit form the small dense operand, so
// both the logits (K Q^T) and the output (V^T P^T) are 16x16x32 bf16 MFMA
// contractions fed straight from global memory with 16-byte loads: no LDS
// staging and no register transposes.
//
// Value pages are stored chunk-blocked and transposed, [chunk][D][32 tokens], so
// that every operand load of a wavefront covers one contiguous KiB.
//
// Operand layout of v_mfma_f32_16x16x32_bf16 (lane = 16*g + n):
//   A (16 x 32): lane holds A[n][8g .. 8g+7]
//   B (32 x 16): lane holds B[8g .. 8g+7][n]
//   D (16 x 16): lane holds D[4g + i][n], i = 0..3
// Logits:  A = keys (row slot n of tile tau holds token t0 + 8*(n/4) + 4*tau + n%4),
//          B = Q^T; lane (g, n) then owns, for query row n, the logits of tokens
//          t0 + 8g + j, j = 0..7 -- exactly the B operand P^T[8g+j][n] of
// Output:  A = V^T (row slot n = channel 16*db + n, k-slots = tokens t0 + 8g + j),
//          D = O^T[16*db + 4g + i][n].

#include "mosaic_internal.h"
#include "attend_mfma_device.h"
#include "attend_reps_device.h"

namespace mosaic {

namespace {

// ---------------------------------------------------------------------------
// Decode shape: at most 16 query rows per unit (one row tile).
// grid (n_units * n_splits), 4 waves; split_slot() shares the workgroups out
// over the units by retrieved size.  Inside a unit chunks are dealt round-robin:
// wave w of split s takes chunks s + S*(w + 4*i); the next chunk's operands are
// in flight while the current one is reduced.
// ---------------------------------------------------------------------------
template <int D, bool AUG, bool STREAM>
__global__ __launch_bounds__(kBlock, 2) void k_attend_decode_mfma(DeviceView dv, int u0, int n_units,
                                                                  const unsigned short *q, int Tq, int B) {
    constexpr int KK = D / 32, DB = D / 16;
    if constexpr (AUG) {
        if ((int)blockIdx.x >= B) {   // extra workgroups: the global representatives' part (augmentation)
            attend_reps_partial<unsigned short, D>(dv, u0, (int)blockIdx.x - B, 0, q, Tq);
            return;
        }
    }
    const int tid = threadIdx.x, wave = tid / 64, lane = tid % 64, g = lane / 16, n = lane % 16;
    const SplitSlot slot = split_slot<false>(dv.n_sel + u0, n_units, B, blockIdx.x);
    if (slot.uc < 0) return;                       // block-uniform: no barrier reached yet
    const int uc = slot.uc, u = u0 + uc, split = slot.split, S = slot.S;
    const int T = dv.T, F = dv.F, cpp = dv.chunks_per_page;
    const int lc = uc / dv.Hkv, h = u % dv.Hkv, R = Tq * dv.G;
    const int *sel = dv.sel_pages + (size_t)u * F;
    // wave-uniform chunk walk: wave w of split s takes chunks first + stride * i
    const int stride = __builtin_amdgcn_readfirstlane(4 * S);
    const int first = __builtin_amdgcn_readfirstlane(split + S * wave);

    bf16x8 qf[KK];
    load_q<D>(dv, q, lc, h, Tq, n, g, qf);

    const float sl2 = 1.4426950408889634f / sqrtf((float)D);

    f32x4 acc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db) acc[db] = f32x4{0.f, 0.f, 0.f, 0.f};
    float m = -INFINITY, l = 0.f, lx = 0.f;

    const int NC = __builtin_amdgcn_readfirstlane(slot.n) * cpp;
    const int n_my = __builtin_amdgcn_readfirstlane(first < NC ? (NC - first + stride - 1) / stride : 0);

    // The page id of a chunk is read (a wave-uniform scalar load) one step before the
    // chunk's operand loads are issued, the cursor that walks the selection advances by
    // increments (no division in the loop), and inside the steady-state loop every load
    // is issued unconditionally, so the operand loads of chunk i+1 stay in flight across
    // the whole reduction of chunk i.
    bf16x8 kA[2 * KK], vA[DB], kB[2 * KK], vB[DB];
    int ccA = 0, ccB = 0;                             // chunk index inside its page
    const int sq = __builtin_amdgcn_readfirstlane(stride / cpp), sr = __builtin_amdgcn_readfirstlane(stride % cpp);
    int lq = __builtin_amdgcn_readfirstlane(first / cpp), lr = __builtin_amdgcn_readfirstlane(first % cpp), lj = 0;
    auto lookup = [&](int &page, int &cc) {           // page and in-page chunk of the cursor's chunk
        page = sel[lq]; cc = lr;
        if (lj + 1 < n_my) {                          // advance, stopping at the wave's last chunk
            ++lj; lq += sq; lr += sr;
            if (lr >= cpp) { lr -= cpp; ++lq; }
        }
    };
    auto issue = [&](int page, int cc_in, bf16x8 (&kf)[2 * KK], bf16x8 (&vf)[DB], int &cc) {
        cc = cc_in;
        const char *kp = k_page(dv, u, page);
        const char *vp = v_page(dv, u, page);
        issue_chunk<D, STREAM>(reinterpret_cast<const unsigned short *>(kp),
                               reinterpret_cast<const unsigned short *>(vp) + (size_t)cc * D * 32,
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
        for (; i + 2 < n_my; i += 2) {                // A holds chunk i; (pg_n, cc_n) is chunk i+1
            issue(pg_n, cc_n, kB, vB, ccB);
            lookup(pg_n, cc_n);
            __builtin_amdgcn_sched_barrier(0);        // keep the loads ahead of the arithmetic
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
    // merge the four waves, write one partial per workgroup
    merge_waves_store<D>(dv, acc, m, l, lx, R, (size_t)slot.base + split);        // one row tile
}

// ---------------------------------------------------------------------------
// Fused decode step (one row tile, per-layer call): selection and attention in one
// launch.  grid (n_units * S), 4 waves; workgroup = (unit, split), S uniform.
// Every workgroup of a unit first repeats the unit's selection for itself -- mean
// query, scores of the C <= 256 representatives, ranks of the k best, page offsets --
// which costs it the table's C x D x 8 bytes through L2 (the longest part of its life: the query is
// back after ~2 k cycles, the table after 6-7 k) and ~4 k cycles of arithmetic, but
// removes the separate selection launch and the two dependent round trips (sizes,
// page ids) at the start of the attention kernel; it then lists the pages of its own
// contiguous chunk range in LDS and reduces them like k_attend_decode_mfma.  Split 0
// of each unit also writes the selection (scores, ids, page list, counts) to memory,
// so the observers and a later mosaic_attend see what mosaic_retrieve would have left.
// Same arithmetic, lane for lane, as k_retrieve (scores, ranking) and as the decode
// kernel (chunk steps), hence the same ids, token lists and -- up to the order in
// which partials are merged -- outputs.
// ---------------------------------------------------------------------------
constexpr int kFusedMaxC = 256, kFusedList = 2048;

__device__ __forceinline__ double group16_sum_f64(double x) { return row16_sum(x); }   // as in k_retrieve

template <int D, bool STREAM>
__global__ __launch_bounds__(kBlock) void k_decode_fused(DeviceView dv, int u0, const unsigned short *q, int Tq,
                                                         int S, int n_frames, int score_mode) {
    constexpr int KK = D / 32, DB = D / 16, EPL = D / 16, NG = kBlock / 16, RPF = 8, FPT = 8;
    const int tid = threadIdx.x, wave = tid / 64, lane = tid % 64, g = lane / 16, n = lane % 16;
    const int lr = tid % 16, grp = tid / 16;
    const int uc = (int)blockIdx.x / S, split = (int)blockIdx.x % S, u = u0 + uc;
    const int C = dv.C, k = dv.k, G = dv.G, Hq = dv.Hq, T = dv.T, F = dv.F, cpp = dv.chunks_per_page;
    const int lc = uc / dv.Hkv, h = u % dv.Hkv, R = Tq * G;
    __shared__ double qbar[D];
    __shared__ double sc_sh[kFusedMaxC], rn_sh[kFusedMaxC];
    __shared__ int n_sh[kFusedMaxC], rank_sh[kFusedMaxC], cnt_sh[kFusedMaxC], ids_sh[kFusedMaxC], off_sh[kFusedMaxC + 1];
    __shared__ int list_sh[kFusedList];
    __shared__ int n_live_sh;
    const double *r = dv.r + (size_t)u * C * D;
    const int *assign = dv.assign + (size_t)u * F;
    const int *pos = dv.pos + (size_t)u * F;

    // ---- independent loads, all issued up front ----
    bf16x8 qf[KK];
    load_q<D>(dv, q, lc, h, Tq, n, g, qf);
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
    if (tid < D) {      // mean query over the Tq tokens and the G query heads of this KV head
        // (R <= 16: two batches of eight loads, row index clamped, loads unconditional)
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
    // the 16-lane groups leave the raw dot products in LDS; thread j then finishes entry j
    // (one fp64 division per thread instead of one per row on a single lane)
    // (no lane-dependent branch around a row: the rows' reduction chains interleave; a row
    // beyond the table repeats the last one and is not stored)
#pragma unroll
    for (int i = 0; i < RPF; ++i) {
        const int j = grp + NG * i;
        if (NG * i < C) {                                     // workgroup-uniform
            double p = 0.0;
#pragma unroll
            for (int e = 0; e < EPL; ++e) p += qbar[lr * EPL + e] * rpre[i][e];
            p = group16_sum_f64(p);
            if (lr == 0 && j < C) sc_sh[j] = p;
        }
    }
    for (int j = grp + NG * RPF; j < C; j += NG) {
        const double *rj = r + (size_t)j * D + lr * EPL;
        double p = 0.0;
#pragma unroll
        for (int e = 0; e < EPL; ++e) p += qbar[lr * EPL + e] * rj[e];
        p = group16_sum_f64(p);
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
        if (split == 0) dv.scores[(size_t)u * dv.SC + tid] = sc;
    }
    __syncthreads();
    // ---- ranks by (score descending, id ascending) among the non-empty clusters ----
    {   // 2^pl threads per entry (the largest power of two that fits the workgroup: shifts, no divisions);
        // pairs compared on the fp32 roundings (monotone, so a strict fp32 order is the fp64 order; fp64
        // compares run at a quarter of the rate), collisions settled exactly below
        const int pl = 31 - __clz(kBlock / C);
        const int j = tid >> pl, part = tid & ((1 << pl) - 1);
        if (j < C && n_sh[j] > 0) {
            const float fj = key_sh[j];
            const int i0 = (C * part) >> pl, i1 = (C * (part + 1)) >> pl;
            int c = 0, ceq = 0;  // (an empty cluster carries -inf and neither outranks nor equals a live one)
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
    {   // C <= 256 = kBlock: thread j owns entry j; live entries counted with one atomic per wavefront
        const bool live = tid < C && n_sh[tid] > 0;
        int rk = -1;
        if (live) {
            const int v = cnt_sh[tid];
            rk = v & 0xffff;
            if ((v >> 16) > 1) {                        // collisions (the entry itself counts once): exact order among them
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
            if (split == 0) { dv.n_ids[u] = n_ids; dv.n_sel[u] = run; }
        }
    }
    if (split == 0)
        for (int i = tid; i < k; i += kBlock) dv.ids[(size_t)u * k + i] = i < n_ids ? ids_sh[i] : -1;
    __syncthreads();
    // ---- this workgroup's chunk range and its pages ----
    const int NC = off_sh[n_ids] * cpp;
    const int cps = (NC + S - 1) / S;
    const int c0 = split * cps, c1 = min(NC, c0 + cps);
    const int p_lo = c0 / cpp, p_hi = c1 > c0 ? (c1 - 1) / cpp : p_lo - 1;
    int *sel = dv.sel_pages + (size_t)u * F;
    auto place = [&](int f, int a, int ps) {   // (no early exits: the LDS look-ups of a batch overlap)
        const int rk = rank_sh[max(a, 0)];
        const bool sel_f = a >= 0 && rk >= 0;
        const int p = off_sh[max(rk, 0)] + ps;
        if (sel_f && p >= p_lo && p <= p_hi) list_sh[p - p_lo] = f;
        if (sel_f && split == 0) sel[p] = f;
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
    __syncthreads();

    // ---- attention over chunks c0 + wave, + 4, ... of the range ----
    const float sl2 = 1.4426950408889634f / sqrtf((float)D);
    f32x4 acc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db) acc[db] = f32x4{0.f, 0.f, 0.f, 0.f};
    float m = -INFINITY, l = 0.f, lx = 0.f;
    const int first = c0 + wave;
    const int n_my = first < c1 ? (c1 - first + 3) / 4 : 0;
    bf16x8 kA[2 * KK], vA[DB], kB[2 * KK], vB[DB];
    int ccA = 0, ccB = 0;
    auto issue = [&](int c, bf16x8 (&kf)[2 * KK], bf16x8 (&vf)[DB], int &cc) {
        const int pi = c / cpp;
        cc = c - pi * cpp;
        const int page = list_sh[pi - p_lo];
        const char *kp = k_page(dv, u, page);
        const char *vp = v_page(dv, u, page);
        issue_chunk<D, STREAM>(reinterpret_cast<const unsigned short *>(kp),
                               reinterpret_cast<const unsigned short *>(vp) + (size_t)cc * D * 32,
                               cc * kChunk, T, g, n, kf, vf);
    };
    auto step = [&](const bf16x8 (&kf)[2 * KK], const bf16x8 (&vf)[DB], int cc) {
        chunk_step<D>(kf, vf, qf, min(kChunk, T - cc * kChunk), g, sl2, acc, m, l, lx);
    };
    if (n_my > 0) {
        issue(first, kA, vA, ccA);
        int i = 0;
        for (; i + 2 < n_my; i += 2) {
            issue(first + 4 * (i + 1), kB, vB, ccB);
            __builtin_amdgcn_sched_barrier(0);
            step(kA, vA, ccA);
            issue(first + 4 * (i + 2), kA, vA, ccA);
            __builtin_amdgcn_sched_barrier(0);
            step(kB, vB, ccB);
        }
        if (i + 2 == n_my) {
            issue(first + 4 * (i + 1), kB, vB, ccB);
            __builtin_amdgcn_sched_barrier(0);
            step(kA, vA, ccA);
            step(kB, vB, ccB);
        } else {
            step(kA, vA, ccA);
        }
    }
    merge_waves_store<D>(dv, acc, m, l, lx, R, (size_t)uc * S + split);
}

} // namespace

hipError_t launch_decode_fused(const DeviceView &dv, int u0, int n_units, const void *q, int Tq, int n_splits,
                               int n_frames, int score_mode, bool stream_kv, hipStream_t s, hipEvent_t ev0,
                               hipEvent_t ev1) {
    const dim3 grid(n_units * n_splits), block(kBlock);
    const unsigned short *qq = (const unsigned short *)q;
    if (stream_kv) {
        if (dv.D == 64) launch_timed((k_decode_fused<64, true>), grid, block, 0, s, ev0, ev1, dv, u0, qq, Tq, n_splits, n_frames, score_mode);
        else launch_timed((k_decode_fused<128, true>), grid, block, 0, s, ev0, ev1, dv, u0, qq, Tq, n_splits, n_frames, score_mode);
    } else {
        if (dv.D == 64) launch_timed((k_decode_fused<64, false>), grid, block, 0, s, ev0, ev1, dv, u0, qq, Tq, n_splits, n_frames, score_mode);
        else launch_timed((k_decode_fused<128, false>), grid, block, 0, s, ev0, ev1, dv, u0, qq, Tq, n_splits, n_frames, score_mode);
    }
    return hipGetLastError();
}

hipError_t launch_attend_mfma(const DeviceView &dv, int u0, int n_units, const void *q, int Tq,
                              int n_splits, bool stream_kv, hipStream_t s, hipEvent_t ev0, hipEvent_t ev1) {
    const int NT = (Tq * dv.G + kRowTile - 1) / kRowTile;
    const unsigned short *qq = (const unsigned short *)q;
    const dim3 block(kBlock);
    if (NT == 1) {
        const int B = n_units * n_splits;
        const dim3 grid(B + (dv.aug_reps ? n_units : 0));
        auto go = [&](auto kern) { launch_timed(kern, grid, block, 0, s, ev0, ev1, dv, u0, n_units, qq, Tq, B); };
        if (dv.aug_reps) {
            if (dv.D == 64) stream_kv ? go(k_attend_decode_mfma<64, true, true>) : go(k_attend_decode_mfma<64, true, false>);
            else stream_kv ? go(k_attend_decode_mfma<128, true, true>) : go(k_attend_decode_mfma<128, true, false>);
        } else {
            if (dv.D == 64) stream_kv ? go(k_attend_decode_mfma<64, false, true>) : go(k_attend_decode_mfma<64, false, false>);
            else stream_kv ? go(k_attend_decode_mfma<128, false, true>) : go(k_attend_decode_mfma<128, false, false>);
        }
    } else {
        return launch_attend_prefill(dv, u0, n_units, qq, Tq, n_splits, s, ev0, ev1);
    }
    return hipGetLastError();
}

} // namespace mosaic
