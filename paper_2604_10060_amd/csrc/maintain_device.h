// Self-Adaptive Maintainer, device side (paper Sec. VI): cluster refinement by
// Split, shared by the ingest kernel (Alg. 1 insertion procedure, lines 4-6) and
// the retrieve kernel (retrieval procedure, lines 12-17).
//
// Everything here is executed cooperatively by ONE workgroup (any size that is a
// multiple of 64, at most 1024 threads) working on one unit; every thread of the
// workgroup must make the call.  Arithmetic is fp64 like the rest of the
// clustering state.  Means are accumulated in ascending frame order (the same
// sequence of additions a sequential loop performs), so representatives do not
// depend on the workgroup size.
//
// Split itself is not defined by the paper.  Reading: two-means under the
// clustering criterion of Sec. V-B; seeds are the two members with the lowest
// mutual cosine (first such pair in (i, i') order); `split_iters` rounds of
// (every member to the more similar of the two representatives, equal goes to
// the first; representatives = means of their sides, an empty side keeps its
// representative).  The side of the first seed keeps the cluster id.
#pragma once
#include "mosaic_internal.h"

namespace mosaic {

template <int D> struct SplitShared {
    double ca[D], cb[D];     // the two representatives
    double na, nb;           // their norms
    double red_v[16];        // per-wavefront reduction slots
    int red_i[16], red_k[16];
    int wtot[16];
    int m, cnt1, fresh;
};

// (every call site has all 16 lanes of the group active)
__device__ __forceinline__ double mt_g16sum(double x) { return row16_sum(x); }
// (every call site has the whole wavefront active)
__device__ __forceinline__ double mt_wave_sum(double x) { return wave64_sum(x); }

// Exclusive prefix of one count per thread over the workgroup, in thread order;
// *total receives the sum.  Uses sh.wtot; ends with a barrier.
template <int D>
__device__ __forceinline__ int mt_block_excl_scan(int c, SplitShared<D> &sh, int *total) {
    const int tid = threadIdx.x, lane = tid % 64, wave = tid / 64, nw = blockDim.x / 64;
    int x = c;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int y = __shfl_up(x, o, 64);
        if (lane >= o) x += y;
    }
    __syncthreads();                      // wtot may still be read from an earlier scan
    if (lane == 63) sh.wtot[wave] = x;
    __syncthreads();
    int base = 0, tot = 0;
    for (int w = 0; w < nw; ++w) {
        if (w < wave) base += sh.wtot[w];
        tot += sh.wtot[w];
    }
    *total = tot;
    return base + x - c;
}

// |v|^2 of a D-vector held one element per thread (tid < D); result in every thread.
// Uses sh.red_v[0..1]; ends with a barrier.
template <int D>
__device__ __forceinline__ double mt_block_sq(double v_tid, SplitShared<D> &sh) {
    const int tid = threadIdx.x, lane = tid % 64, wave = tid / 64;
    double sq = tid < D ? v_tid * v_tid : 0.0;
    __syncthreads();
    if (wave < 2) {
        sq = mt_wave_sum(sq);
        if (lane == 0) sh.red_v[wave] = sq;
    }
    __syncthreads();
    const double r = D > 64 ? sh.red_v[0] + sh.red_v[1] : sh.red_v[0];
    __syncthreads();
    return r;
}

// Split cluster `a` of unit `u` (members = frames f < n_frames with assign[f] == a).
// Returns the new cluster's id, or -1 if nothing was split (no free id, fewer than
// two members, or one side empty).  With `refresh`, the size, representative,
// variance and member ranks of `a` are recomputed from its members also when
// nothing was split (used after buffered entries were merged into it).
// Scratch (global, per unit): mem [F] int, side [F] int, nrm [F] double.
template <int D>
__device__ int mt_split_cluster(const DeviceView &dv, int u, int a, int n_frames, bool refresh,
                                SplitShared<D> &sh) {
    constexpr int EPL = D / 16;
    const int tid = threadIdx.x, NTH = blockDim.x, lane = tid % 64, wave = tid / 64;
    const int lr = tid % 16, grp = tid / 16, NG = NTH / 16, nw = NTH / 64;
    const int C = dv.C;
    int *assign = dv.assign + (size_t)u * dv.F;
    int *pos = dv.pos + (size_t)u * dv.F;
    int *mem = dv.mt_mem + (size_t)u * dv.F;
    int *side = dv.mt_side + (size_t)u * dv.F;
    double *nrm = dv.mt_nrm + (size_t)u * dv.F;
    const double *summ = dv.summ + (size_t)u * dv.F * D;
    double *r = dv.r + (size_t)u * C * D;

    // ---- member list, ascending frames ----
    const int per = (n_frames + NTH - 1) / NTH;
    const int b0 = min(tid * per, n_frames), b1 = min(b0 + per, n_frames);
    int c = 0;
    for (int f = b0; f < b1; ++f) c += assign[f] == a;
    int m;
    int w = mt_block_excl_scan<D>(c, sh, &m);
    for (int f = b0; f < b1; ++f)
        if (assign[f] == a) mem[w++] = f;
    __syncthreads();

    const int slots = dv.n_slots[u];
    bool can_split = m >= 2 && slots < C;
    int n1 = 0;
    if (can_split) {
        // ---- norms of the members' summaries ----
        for (int i = grp; i < m; i += NG) {
            const double *s = summ + (size_t)mem[i] * D + lr * EPL;
            double p = 0.0;
#pragma unroll
            for (int e = 0; e < EPL; ++e) p += s[e] * s[e];
            p = mt_g16sum(p);
            if (lr == 0) nrm[i] = sqrt(p);
        }
        __syncthreads();
        // ---- seeds: the pair with the lowest mutual cosine, first in (i, k) order ----
        double bv = INFINITY;
        int bi = 0x7fffffff, bk = 0x7fffffff;
        for (int i = grp; i + 1 < m; i += NG) {
            double si[EPL];
            const double *s = summ + (size_t)mem[i] * D + lr * EPL;
#pragma unroll
            for (int e = 0; e < EPL; ++e) si[e] = s[e];
            const double ni = nrm[i];
            // four partners at a time: their indices, then their rows, are fetched together (one chain of
            // two round trips per batch instead of per pair); compared in k order
            for (int k0 = i + 1; k0 < m; k0 += 4) {
                int row[4];
                double nk[4], t[4][EPL];
#pragma unroll
                for (int x = 0; x < 4; ++x) {
                    const int kk = min(k0 + x, m - 1);
                    row[x] = mem[kk];
                    nk[x] = nrm[kk];
                }
#pragma unroll
                for (int x = 0; x < 4; ++x) {
                    const double *tp = summ + (size_t)row[x] * D + lr * EPL;
#pragma unroll
                    for (int e = 0; e < EPL; ++e) t[x][e] = tp[e];
                }
#pragma unroll
                for (int x = 0; x < 4; ++x) {
                    const int k = k0 + x;
                    double p = 0.0;
#pragma unroll
                    for (int e = 0; e < EPL; ++e) p += si[e] * t[x][e];
                    p = mt_g16sum(p);
                    const double cs = (ni == 0.0 || nk[x] == 0.0) ? 0.0 : p / (ni * nk[x]);
                    if (k < m && (cs < bv || (cs == bv && (i < bi || (i == bi && k < bk))))) { bv = cs; bi = i; bk = k; }
                }
            }
        }
#pragma unroll
        for (int o = 16; o <= 32; o <<= 1) {
            const double ov = __shfl_xor(bv, o, 64);
            const int oi = __shfl_xor(bi, o, 64), ok = __shfl_xor(bk, o, 64);
            if (ov < bv || (ov == bv && (oi < bi || (oi == bi && ok < bk)))) { bv = ov; bi = oi; bk = ok; }
        }
        if (lane == 0) { sh.red_v[wave] = bv; sh.red_i[wave] = bi; sh.red_k[wave] = bk; }
        __syncthreads();
        if (tid == 0) {
            for (int x = 1; x < nw; ++x) {
                const double ov = sh.red_v[x];
                const int oi = sh.red_i[x], ok = sh.red_k[x];
                if (ov < bv || (ov == bv && (oi < bi || (oi == bi && ok < bk)))) { bv = ov; bi = oi; bk = ok; }
            }
            sh.red_i[0] = bi; sh.red_k[0] = bk;
        }
        __syncthreads();
        bi = sh.red_i[0]; bk = sh.red_k[0];
        __syncthreads();
        double va = 0.0, vb = 0.0;
        if (tid < D) {
            va = summ[(size_t)mem[bi] * D + tid];
            vb = summ[(size_t)mem[bk] * D + tid];
            sh.ca[tid] = va; sh.cb[tid] = vb;
        }
        double qa = mt_block_sq<D>(va, sh), qb = mt_block_sq<D>(vb, sh);
        double na = sqrt(qa), nb = sqrt(qb);
        // ---- two-means rounds ----
        for (int it = 0; it < dv.split_iters; ++it) {
            if (tid == 0) sh.cnt1 = 0;
            __syncthreads();
            for (int i = grp; i < m; i += NG) {
                const double *s = summ + (size_t)mem[i] * D + lr * EPL;
                double pa = 0.0, pb = 0.0;
#pragma unroll
                for (int e = 0; e < EPL; ++e) {
                    pa += s[e] * sh.ca[lr * EPL + e];
                    pb += s[e] * sh.cb[lr * EPL + e];
                }
                pa = mt_g16sum(pa); pb = mt_g16sum(pb);
                if (lr == 0) {
                    const double ni = nrm[i];
                    const double ka = (ni == 0.0 || na == 0.0) ? 0.0 : pa / (ni * na);
                    const double kb = (ni == 0.0 || nb == 0.0) ? 0.0 : pb / (ni * nb);
                    const int sd = kb > ka;
                    side[i] = sd;
                    if (sd) atomicAdd(&sh.cnt1, 1);
                }
            }
            __syncthreads();
            n1 = sh.cnt1;
            const int n0 = m - n1;
            va = 0.0; vb = 0.0;
            if (tid < D) {
                double acc0 = 0.0, acc1 = 0.0;
                // eight members' indices, sides and rows in flight at a time (clamped, unconditional), added in member order
                for (int i0 = 0; i0 < m; i0 += 8) {
                    int row[8], sd[8];
                    double v[8];
#pragma unroll
                    for (int x = 0; x < 8; ++x) { const int i = min(i0 + x, m - 1); row[x] = mem[i]; sd[x] = side[i]; }
#pragma unroll
                    for (int x = 0; x < 8; ++x) v[x] = summ[(size_t)row[x] * D + tid];
#pragma unroll
                    for (int x = 0; x < 8; ++x)
                        if (i0 + x < m) { if (sd[x]) acc1 += v[x]; else acc0 += v[x]; }
                }
                if (n0 > 0) sh.ca[tid] = acc0 / (double)n0;
                if (n1 > 0) sh.cb[tid] = acc1 / (double)n1;
                va = sh.ca[tid]; vb = sh.cb[tid];
            }
            qa = mt_block_sq<D>(va, sh); qb = mt_block_sq<D>(vb, sh);
            na = sqrt(qa); nb = sqrt(qb);
        }
        can_split = n1 > 0 && n1 < m;
        if (can_split) {
            const int fresh = slots;
            // squared distances to the own side's representative (Eq. 2), one per member
            for (int i = grp; i < m; i += NG) {
                const double *s = summ + (size_t)mem[i] * D + lr * EPL;
                const double *cc = side[i] ? sh.cb : sh.ca;
                double p = 0.0;
#pragma unroll
                for (int e = 0; e < EPL; ++e) { const double t = s[e] - cc[lr * EPL + e]; p += t * t; }
                p = mt_g16sum(p);
                if (lr == 0) nrm[i] = p;
            }
            // ranks inside the two sides, ascending frames
            const int pm = (m + NTH - 1) / NTH;
            const int i0 = min(tid * pm, m), i1 = min(i0 + pm, m);
            int c1 = 0;
            for (int i = i0; i < i1; ++i) c1 += side[i];
            int tot1;
            int r1 = mt_block_excl_scan<D>(c1, sh, &tot1);
            int r0 = i0 - r1;
            for (int i = i0; i < i1; ++i) {
                const int f = mem[i];
                if (side[i]) { assign[f] = fresh; pos[f] = r1++; }
                else pos[f] = r0++;
            }
            if (tid < D) {
                r[(size_t)a * D + tid] = sh.ca[tid];
                r[(size_t)fresh * D + tid] = sh.cb[tid];
            }
            __syncthreads();
            if (tid < 2) {                        // thread 0: cluster a, thread 1: the new cluster
                double acc = 0.0;
                for (int i0 = 0; i0 < m; i0 += 8) {      // eight entries in flight, added in member order
                    int sd[8];
                    double v[8];
#pragma unroll
                    for (int x = 0; x < 8; ++x) { const int i = min(i0 + x, m - 1); sd[x] = side[i]; v[x] = nrm[i]; }
#pragma unroll
                    for (int x = 0; x < 8; ++x)
                        if (i0 + x < m && sd[x] == tid) acc += v[x];
                }
                const int j = tid ? fresh : a, cnt = tid ? n1 : m - n1;
                dv.var[(size_t)u * C + j] = acc / (double)cnt;
                dv.n[(size_t)u * C + j] = cnt;
                dv.rnorm[(size_t)u * C + j] = tid ? nb : na;
                dv.lazy[(size_t)u * C + j] = 0;
                if (tid) {
                    dv.resident[(size_t)u * C + fresh] = dv.resident[(size_t)u * C + a];
                    dv.n_slots[u] = slots + 1;
                }
            }
            __syncthreads();
            return fresh;
        }
    }
    if (refresh) {
        // exact statistics of the (merged) cluster: Eq. 1, Eq. 2, ranks
        double v = 0.0;
        if (tid < D && m > 0) {
            double acc = 0.0;
            for (int i0 = 0; i0 < m; i0 += 8) {          // eight members in flight, added in member order
                int row[8];
                double w[8];
#pragma unroll
                for (int x = 0; x < 8; ++x) row[x] = mem[min(i0 + x, m - 1)];
#pragma unroll
                for (int x = 0; x < 8; ++x) w[x] = summ[(size_t)row[x] * D + tid];
#pragma unroll
                for (int x = 0; x < 8; ++x)
                    if (i0 + x < m) acc += w[x];
            }
            v = acc / (double)m;
            sh.ca[tid] = v;
            r[(size_t)a * D + tid] = v;
        }
        const double q = mt_block_sq<D>(v, sh);
        for (int i = grp; i < m; i += NG) {
            const double *s = summ + (size_t)mem[i] * D + lr * EPL;
            double p = 0.0;
#pragma unroll
            for (int e = 0; e < EPL; ++e) { const double t = s[e] - sh.ca[lr * EPL + e]; p += t * t; }
            p = mt_g16sum(p);
            if (lr == 0) nrm[i] = p;
        }
        for (int i = tid; i < m; i += NTH) pos[mem[i]] = i;
        __syncthreads();
        if (tid == 0) {
            double acc = 0.0;
            for (int i0 = 0; i0 < m; i0 += 8) {
                double w[8];
#pragma unroll
                for (int x = 0; x < 8; ++x) w[x] = nrm[min(i0 + x, m - 1)];
#pragma unroll
                for (int x = 0; x < 8; ++x)
                    if (i0 + x < m) acc += w[x];
            }
            dv.var[(size_t)u * C + a] = m > 0 ? acc / (double)m : 0.0;
            dv.n[(size_t)u * C + a] = m;
            if (m > 0) dv.rnorm[(size_t)u * C + a] = sqrt(q);
        }
        __syncthreads();
    }
    return -1;
}

} // namespace mosaic
