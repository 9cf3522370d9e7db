// Frame Encoding kernels (paper Sec. V-A (1), Sec. VI-A, Sec. V-B):
//   k_store_summary  copy a frame's K/V pages into the arena and form the
//                    frame's key summary (mean of its T keys) in fp64
//   k_assign_update  greedy cosine assignment + running-mean update (Eq. 3),
//                    sequential over the frames of a batch, one workgroup per unit
//   k_lloyd_*        cosine K-means rounds for the initial clustering and the
//                    periodic warm-started re-clustering
// All decision arithmetic is fp64: on CDNA4 the fp64 vector rate equals the
// non-packed fp32 rate, so exact-to-rounding decisions cost only table bytes.
#include <type_traits>

#include <algorithm>
#include "mosaic_internal.h"
#include "maintain_device.h"

namespace mosaic {

namespace {

template <typename E> struct Elem;
template <> struct Elem<float> {
    static __device__ __forceinline__ void load8(const float *p, float (&v)[8]) {
        const float4 a = *reinterpret_cast<const float4 *>(p);
        const float4 b = *reinterpret_cast<const float4 *>(p + 4);
        v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
        v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
    }
    static __device__ __forceinline__ void copy8(const float *src, float *dst) {
        *reinterpret_cast<float4 *>(dst) = *reinterpret_cast<const float4 *>(src);
        *reinterpret_cast<float4 *>(dst + 4) = *reinterpret_cast<const float4 *>(src + 4);
    }
};
template <> struct Elem<unsigned short> {
    static __device__ __forceinline__ void load8(const unsigned short *p, float (&v)[8]) {
        const uint4 a = *reinterpret_cast<const uint4 *>(p);
        const unsigned int w[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[2 * i] = __uint_as_float(w[i] << 16);
            v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
    static __device__ __forceinline__ void copy8(const unsigned short *src, unsigned short *dst) {
        *reinterpret_cast<uint4 *>(dst) = *reinterpret_cast<const uint4 *>(src);
    }
};

// (every call site has all 16 lanes of the group active)
__device__ __forceinline__ double group16_sum(double x) { return row16_sum(x); }
// (every call site has the whole wavefront active)
__device__ __forceinline__ double wave_sum(double x) { return wave64_sum(x); }
// (value, id) ordered by value descending then id ascending
__device__ __forceinline__ bool better(double v, int i, double bv, int bi) {
    return v > bv || (v == bv && i < bi);
}
// fp64 max / min as single instructions (the builtins add an instruction per operand that quiets signalling NaNs);
// only used on values that are never NaN
__device__ __forceinline__ double max_f64(double a, double b) {
    double r;
    asm("v_max_f64 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}
__device__ __forceinline__ double min_f64(double a, double b) {
    double r;
    asm("v_min_f64 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}

// Best (value, id) of a wavefront when the ids ascend with the lane (at most one candidate per lane, -inf and
// 0x7fffffff in lanes without one; no NaN): the largest value by a max butterfly (three instructions per step
// against a dozen for the (value, id) pair), then the first lane that holds it, which is the lowest id.  Left in
// every lane.
__device__ __forceinline__ void wave_best_ascending(double &bv, int &bi) {
    double m = bv;
    m = max_f64(m, dpp_f64<kDppXor8>(m));
    m = max_f64(m, dpp_f64<kDppXor7>(m));
    m = max_f64(m, dpp_f64<kDppXor3>(m));
    m = max_f64(m, dpp_f64<kDppXor1>(m));
    const long long b = __double_as_longlong(m);
    const int lo = (int)b, hi = (int)(b >> 32);
    double wm = -INFINITY;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int l = __builtin_amdgcn_readlane(lo, 16 * r), h = __builtin_amdgcn_readlane(hi, 16 * r);
        wm = fmax(wm, __longlong_as_double(((long long)h << 32) | (long long)(unsigned int)l));
    }
    const unsigned long long at = __ballot(bv == wm);
    const int first = __ffsll((long long)at) - 1;                       // some lane holds the maximum
    const int id = __builtin_amdgcn_readlane(bi, first);
    bv = wm;
    bi = wm == -INFINITY ? 0x7fffffff : id;
}

// Best (value, id) of a wavefront, left in every lane: a butterfly inside each row of 16
// lanes with data-parallel primitives (the order is total, so every lane of a row ends
// with the same pair), then the four rows' pairs are read from their first lanes.
template <int CTRL> __device__ __forceinline__ void best_step(double &bv, int &bi) {
    const double ov = dpp_f64<CTRL>(bv);
    const int oi = dpp_i32<CTRL>(bi);
    if (better(ov, oi, bv, bi)) { bv = ov; bi = oi; }
}
__device__ __forceinline__ void wave_best(double &bv, int &bi) {
    best_step<kDppXor8>(bv, bi);
    best_step<kDppXor7>(bv, bi);
    best_step<kDppXor3>(bv, bi);
    best_step<kDppXor1>(bv, bi);
    const long long b = __double_as_longlong(bv);
    const int lo = (int)b, hi = (int)(b >> 32);
    double rv[4];
    int ri[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int l = __builtin_amdgcn_readlane(lo, 16 * r), h = __builtin_amdgcn_readlane(hi, 16 * r);
        rv[r] = __longlong_as_double(((long long)h << 32) | (long long)(unsigned int)l);
        ri[r] = __builtin_amdgcn_readlane(bi, 16 * r);
    }
    bv = rv[0]; bi = ri[0];
#pragma unroll
    for (int r = 1; r < 4; ++r)
        if (better(rv[r], ri[r], bv, bi)) { bv = rv[r]; bi = ri[r]; }
}

// ---------------------------------------------------------------------------
// Page store + summaries.  store_key_page / store_value_page are run by one
// 256-thread workgroup per (unit, frame): the page goes to the arena's store (HBM
// tier) or the staging ring (host tier); the key summary (mean of the frame's T key
// vectors, fp64) goes to dv.summ and, if s_out is given, to that LDS array too.
// red: kBlock / (D / 8) rows of D doubles of LDS scratch.
// ---------------------------------------------------------------------------
template <typename E, int D>
__device__ __forceinline__ void store_key_page(const DeviceView &dv, const E *k_in, char *kdst_base, int u, int fl,
                                               int f, double (&red)[kBlock / (D / 8)][D], double *s_out) {
    constexpr int LPR = D / 8;          // lanes per row, 8 elements each
    constexpr int RP = kBlock / LPR;    // rows per pass
    const int tid = threadIdx.x, cg = tid % LPR, r0 = tid / LPR;
    const int T = dv.T;
    const size_t in_page = ((size_t)fl * dv.U + u) * (size_t)T * D;
    const size_t page = (size_t)u * dv.F + f;          // summary slot
    const bool host = dv.tier == MOSAIC_TIER_HOST;
    const size_t spage = host ? (size_t)(f % dv.SN) * dv.U + u : (size_t)u * dv.PU + f;
    const E *src = k_in + in_page;
    E *dst = reinterpret_cast<E *>(kdst_base) + spage * (size_t)T * D;
    double acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = 0.0;
    for (int t = r0; t < T; t += RP) {
        float v[8];
        Elem<E>::load8(src + (size_t)t * D + cg * 8, v);
        Elem<E>::copy8(src + (size_t)t * D + cg * 8, dst + (size_t)t * D + cg * 8);
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] += (double)v[i];
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) red[r0][cg * 8 + i] = acc[i];
    __syncthreads();
    if (tid < D) {
        double sm = 0.0;
        for (int rr = 0; rr < RP; ++rr) sm += red[rr][tid];
        sm /= (double)T;
        dv.summ[page * D + tid] = sm;
        if (s_out) s_out[tid] = sm;
    }
}

template <typename E, int D>
__device__ __forceinline__ void store_value_page(const DeviceView &dv, const E *v_in, char *vdst_base, int u, int fl,
                                                 int f, double (&red)[kBlock / (D / 8)][D]) {
    constexpr int LPR = D / 8, RP = kBlock / LPR;
    const int tid = threadIdx.x, cg = tid % LPR, r0 = tid / LPR;
    const int T = dv.T;
    const size_t in_page = ((size_t)fl * dv.U + u) * (size_t)T * D;
    const size_t page = (size_t)u * dv.F + f;
    const bool host = dv.tier == MOSAIC_TIER_HOST;
    const size_t spage = host ? (size_t)(f % dv.SN) * dv.U + u : (size_t)u * dv.PU + f;
    // With the global-representative augmentation on, the frame's value summary (mean of
    // its T value vectors, fp64) is formed next to the copy, like the key summary.
    const E *src = v_in + in_page;
    if (!dv.v_transposed) {
        E *dst = reinterpret_cast<E *>(vdst_base) + spage * (size_t)T * D;
        double acc[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = 0.0;
        for (int t = r0; t < T; t += RP) {
            Elem<E>::copy8(src + (size_t)t * D + cg * 8, dst + (size_t)t * D + cg * 8);
            if (dv.vsumm) {
                float v[8];
                Elem<E>::load8(src + (size_t)t * D + cg * 8, v);
#pragma unroll
                for (int i = 0; i < 8; ++i) acc[i] += (double)v[i];
            }
        }
        if (dv.vsumm) {
#pragma unroll
            for (int i = 0; i < 8; ++i) red[r0][cg * 8 + i] = acc[i];
            __syncthreads();
            if (tid < D) {
                double sv = 0.0;
                for (int rr = 0; rr < RP; ++rr) sv += red[rr][tid];
                dv.vsumm[page * D + tid] = sv / (double)T;
            }
        }
        return;
    }
    // Transposed, chunk-blocked value page [Tp/32][D][32] (2-byte elements only):
    // 8 consecutive tokens of one channel form one 16-byte operand of the PV
    // contraction, and the 16 channels x 32 tokens a wavefront loads at once
    // are one contiguous KiB.  Tokens T..Tp-1 are written as zeros.
    if constexpr (sizeof(E) == 2) {
        constexpr int TC = 64;                       // tokens per LDS tile (two chunks)
        __shared__ unsigned short tile[TC][D + 2];
        const int Tp = dv.Tp;
        double vacc = 0.0;
        unsigned short *dst = reinterpret_cast<unsigned short *>(vdst_base) + spage * (size_t)D * Tp;
        for (int tc0 = 0; tc0 < Tp; tc0 += TC) {
            for (int t = r0; t < TC; t += RP) {
                const int tok = tc0 + t;
                uint4 w = make_uint4(0u, 0u, 0u, 0u);
                if (tok < T) w = *reinterpret_cast<const uint4 *>(src + (size_t)tok * D + cg * 8);
                unsigned int *row = reinterpret_cast<unsigned int *>(&tile[t][cg * 8]);
                row[0] = w.x; row[1] = w.y; row[2] = w.z; row[3] = w.w;
            }
            __syncthreads();
            if (dv.vsumm && tid < D) {
                const int nt = min(TC, T - tc0);     // real tokens in this tile
                for (int t = 0; t < nt; ++t) vacc += (double)bf16_to_f32(tile[t][tid]);
            }
            const int ntg = (min(TC, Tp - tc0)) / 8;  // token groups of 8 in this tile
            for (int id = tid; id < D * ntg; id += kBlock) {
                const int d = id / ntg, tg = id % ntg;
                unsigned int w[4];
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    w[j] = (unsigned int)tile[tg * 8 + 2 * j][d] |
                           ((unsigned int)tile[tg * 8 + 2 * j + 1][d] << 16);
                const int tok = tc0 + tg * 8;         // first of the 8 tokens
                *reinterpret_cast<uint4 *>(dst + ((size_t)(tok / kChunk) * D + d) * kChunk + tok % kChunk) =
                    make_uint4(w[0], w[1], w[2], w[3]);
            }
            __syncthreads();
        }
        if (dv.vsumm && tid < D) dv.vsumm[page * D + tid] = vacc / (double)T;
    }
}

// grid (U, n_frames, 2): z = 0 keys, z = 1 values.
template <typename E, int D>
__global__ __launch_bounds__(kBlock) void k_store_summary(DeviceView dv, const E *k_in,
                                                          const E *v_in, int f0) {
    __shared__ double red[kBlock / (D / 8)][D];
    const int u = blockIdx.x, fl = blockIdx.y;
    const bool host = dv.tier == MOSAIC_TIER_HOST;
    if (blockIdx.z == 0) store_key_page<E, D>(dv, k_in, host ? dv.stage_k : dv.k_store, u, fl, f0 + fl, red, nullptr);
    else store_value_page<E, D>(dv, v_in, host ? dv.stage_v : dv.v_store, u, fl, f0 + fl, red);
}

// ---------------------------------------------------------------------------
// Retrieval augmentation, global representatives (paper Sec. V-C): the value of a
// cluster's pseudo token is the mean of its member frames' value summaries, its key the
// cluster's representative.  grid (U, C), 128 threads: one workgroup per cluster lists
// the cluster's frames in ascending order (ballot-free compaction of the assignment
// array: every thread looks at 16 consecutive frames, a scan over the threads' match
// counts gives each match its slot) and adds their value summaries in that order, so
// the sum is one fixed sequence of additions: the same bits on every run, whatever the
// order in which workgroups are scheduled.  It then writes the fp32 key / value rows of
// the pseudo-token tables (zero rows for empty clusters).
// ---------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(128) void k_value_reps(DeviceView dv, int n_frames) {
    constexpr int NT = 128, FPT = 16, CH = NT * FPT;
    const int u = blockIdx.x, j = blockIdx.y, tid = threadIdx.x, C = dv.C;
    const int wave = tid / 64, lane = tid % 64;
    __shared__ int a_sh[CH];
    __shared__ int mem[CH];
    __shared__ int wtot[2];
    const size_t row = (size_t)u * C + j;
    const int nj = dv.n[row];                       // workgroup-uniform
    const int *assign = dv.assign + (size_t)u * dv.F;
    double acc = 0.0;
    for (int c0 = 0; nj > 0 && c0 < n_frames; c0 += CH) {
        const int cend = min(n_frames, c0 + CH);
#pragma unroll
        for (int i = 0; i < FPT; ++i) {
            const int f = c0 + tid + NT * i;
            a_sh[tid + NT * i] = f < cend ? assign[f] : -1;
        }
        __syncthreads();
        unsigned int mask = 0;               // bit i: frame c0 + 16 tid + i belongs to cluster j
#pragma unroll
        for (int i = 0; i < FPT; ++i) mask |= (a_sh[tid * FPT + i] == j ? 1u : 0u) << i;
        const int mine = __popc(mask);
        int incl = mine;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int t = __shfl_up(incl, o, 64);
            if (lane >= o) incl += t;
        }
        if (lane == 63) wtot[wave] = incl;
        __syncthreads();
        int slot = incl - mine + (wave == 1 ? wtot[0] : 0);
        const int filled = wtot[0] + wtot[1];
        while (mask) {
            const int i = __ffs((int)mask) - 1;
            mask &= mask - 1;
            mem[slot++] = c0 + tid * FPT + i;
        }
        __syncthreads();
        if (tid < D) {
            const double *vb = dv.vsumm + (size_t)u * dv.F * D + tid;
            for (int m0 = 0; m0 < filled; m0 += 16) {      // sixteen loads in flight, added in order
                double v[16];
#pragma unroll
                for (int x = 0; x < 16; ++x) v[x] = vb[(size_t)mem[min(m0 + x, filled - 1)] * D];
#pragma unroll
                for (int x = 0; x < 16; ++x)
                    if (m0 + x < filled) acc += v[x];
            }
        }
        __syncthreads();                     // mem / a_sh are rewritten by the next chunk
    }
    if (tid < D) {
        dv.rvsum[row * D + tid] = acc;
        dv.rep_k[row * D + tid] = nj > 0 ? (float)dv.r[row * D + tid] : 0.f;
        dv.rep_v[row * D + tid] = nj > 0 ? (float)(acc / (double)nj) : 0.f;
    }
}

// ---------------------------------------------------------------------------
// Online assignment + Eq. 3, frames f0..f1-1 in order.  grid (U), 256 threads.
// ---------------------------------------------------------------------------
// With MAINT the insertion procedure of the self-adaptive maintainer (Sec. VI,
// Alg. 1 lines 1-10) follows the update: running variance (Eq. 4), threshold
// (Eq. 5) at the size before the insertion, then absorb / split / defer.
enum { kActAbsorb = 1, kActSplit = 2, kActDefer = 3, kActForced = 4 };

template <int D, bool MAINT>
__global__ __launch_bounds__(kBlock) void k_assign_update(DeviceView dv, int f0, int f1) {
    constexpr int EPL = D / 16;  // elements per lane in a 16-lane row group
    const int u = blockIdx.x, tid = threadIdx.x, C = dv.C;
    const int lr = tid % 16, row0 = tid / 16, wave = tid / 64, lane = tid % 64;
    __shared__ double s_sh[D];
    __shared__ double dot_sh[1024];
    __shared__ double red_v[4];
    __shared__ int red_i[4];
    __shared__ double snorm_sh, nsum_sh[2], dsum_sh[2], psum_sh[2];
    __shared__ int act_sh;
    __shared__ SplitShared<MAINT ? D : 16> split_sh;   // (small placeholder when the maintainer is off)
    double *r = dv.r + (size_t)u * C * D;
    double *rn = dv.rnorm + (size_t)u * C;
    int *n = dv.n + (size_t)u * C;

    const bool nested = dv.P > 0;
    // the summary of the next frame travels while the current frame is processed
    double s_ahead = tid < D ? dv.summ[((size_t)u * dv.F + f0) * D + tid] : 0.0;
    for (int f = f0; f < f1; ++f) {
        // candidates: every cluster id, or (nested hierarchy, Sec. V-B) the ids of the frame's
        // visual partition only
        const int part_f = nested ? dv.part[f] : 0;
        // (maintainer: only the ids in use, [0, n_slots), can have members; the table behind them is not read)
        const int lo = nested ? part_f * dv.Cs : 0, hi = nested ? lo + dv.Cs : (MAINT ? min(C, max(dv.n_slots[u], 1)) : C);
        if (tid < D) {
            s_sh[tid] = s_ahead;
            if (f + 1 < f1) s_ahead = dv.summ[((size_t)u * dv.F + f + 1) * D + tid];
        }
        __syncthreads();
        if (wave == 0) {
            double x = 0.0;
            for (int d = lane; d < D; d += 64) x += s_sh[d] * s_sh[d];
            x = wave_sum(x);
            if (lane == 0) snorm_sh = sqrt(x);
        }
        // sizes and norms of this thread's candidates (at most four: C <= 1024), fetched ahead of the rows
        int nj[4];
        double rnj[4];
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            const int j = min(lo + tid + kBlock * x, hi - 1);
            nj[x] = n[j]; rnj[x] = rn[j];
        }
        // Dot products with the candidates' rows, eight rows of a 16-lane group in flight at a time
        // (row index clamped, loads unconditional, no test of the size: a row nobody reads costs
        // nothing extra, a dependent load per row costs a trip to L2)
        for (int jb = lo; jb < hi; jb += 16 * 8) {
            const int passes = min(8, (hi - jb + 15) / 16);   // workgroup-uniform
            const int j0 = jb + row0;
            auto rows = [&](auto full) {      // full: all eight passes (straight-line code); else only `passes`
                double rv[8][EPL];
#pragma unroll
                for (int x = 0; x < 8; ++x) {
                    if (decltype(full)::value || x < passes) {
                        const double *rj = r + (size_t)min(j0 + 16 * x, hi - 1) * D + lr * EPL;
#pragma unroll
                        for (int i = 0; i < EPL; ++i) rv[x][i] = rj[i];
                    }
                }
#pragma unroll
                for (int x = 0; x < 8; ++x) {
                    if (decltype(full)::value || x < passes) {
                        double p = 0.0;
#pragma unroll
                        for (int i = 0; i < EPL; ++i) p += s_sh[lr * EPL + i] * rv[x][i];
                        p = group16_sum(p);
                        if (lr == 0 && j0 + 16 * x < hi) dot_sh[j0 + 16 * x] = p;
                    }
                }
            };
            if (passes == 8) rows(std::true_type{});
            else rows(std::false_type{});
        }
        __syncthreads();
        // argmax of the cosine over non-empty clusters, ties to the lowest id
        double bv = -INFINITY;
        int bi = 0x7fffffff;
        const double sn = snorm_sh;
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            const int j = lo + tid + kBlock * x;
            if (j < hi && nj[x] > 0) {
                const double c = (sn == 0.0 || rnj[x] == 0.0) ? 0.0 : dot_sh[j] / (sn * rnj[x]);
                if (better(c, j, bv, bi)) { bv = c; bi = j; }
            }
        }
        wave_best(bv, bi);
        if (lane == 0) { red_v[wave] = bv; red_i[wave] = bi; }
        __syncthreads();
        // every thread merges the four wavefronts' winners itself
        bv = red_v[0]; bi = red_i[0];
#pragma unroll
        for (int w = 1; w < 4; ++w)
            if (better(red_v[w], red_i[w], bv, bi)) { bv = red_v[w]; bi = red_i[w]; }
        const int a = bi == 0x7fffffff ? lo : bi;
        const int na_i = n[a];
        const double na = (double)na_i;
        double sq = 0.0, dq = 0.0;
        if (tid < D) {
            // Eq. 3 with each operation rounded separately (no contraction)
            const double rv = __ddiv_rn(__dadd_rn(__dmul_rn(na, r[(size_t)a * D + tid]), s_sh[tid]),
                                        na + 1.0);
            r[(size_t)a * D + tid] = rv;
            sq = rv * rv;
            const double t = s_sh[tid] - rv;
            dq = t * t;
        }
        if (wave < 2) {
            sq = wave_sum(sq);
            if (MAINT) dq = wave_sum(dq);
            if (lane == 0) { nsum_sh[wave] = sq; dsum_sh[wave] = dq; }
        }
        // nested hierarchy: the partition's representative in this unit's key space follows the
        // same running mean (Eq. 3 one level up)
        int pn_i = 0;
        if (nested) {
            double *prow = dv.pr + ((size_t)u * dv.P + part_f) * D;
            pn_i = dv.pn[(size_t)u * dv.P + part_f];
            double psq = 0.0;
            if (tid < D) {
                const double pv = ((double)pn_i * prow[tid] + s_sh[tid]) / ((double)pn_i + 1.0);
                prow[tid] = pv;
                psq = pv * pv;
            }
            if (wave < 2) {
                psq = wave_sum(psq);
                if (lane == 0) psum_sh[wave] = psq;
            }
        }
        __syncthreads();   // all threads have read n[a] and written r before the scalars change
        if (tid == 0) {
            if (nested) {
                dv.prn[(size_t)u * dv.P + part_f] = sqrt(D > 64 ? psum_sh[0] + psum_sh[1] : psum_sh[0]);
                dv.pn[(size_t)u * dv.P + part_f] = pn_i + 1;
            }
            rn[a] = sqrt(D > 64 ? nsum_sh[0] + nsum_sh[1] : nsum_sh[0]);
            int act = kActAbsorb;
            if (MAINT) {
                const double dist2 = D > 64 ? dsum_sh[0] + dsum_sh[1] : dsum_sh[0];
                double *var = dv.var + (size_t)u * C;
                const double var_new = (na * var[a] + dist2) / (na + 1.0);                          // Eq. 4
                const double tau = dv.tau_min + (dv.tau_max - dv.tau_min) * exp(-na / dv.tau_n0);   // Eq. 5
                var[a] = var_new;
                const bool on_gpu = dv.maint_mode == MOSAIC_MAINT_EAGER || dv.resident[(size_t)u * C + a] != 0;
                if (var_new <= tau) act = kActAbsorb;
                else if (on_gpu) act = kActSplit;
                else if (dv.n_buf[u] < dv.buf_max) act = kActDefer;
                else act = kActForced;
                if (act == kActDefer || act == kActForced) dv.lazy[(size_t)u * C + a] = 1;
                if (act == kActDefer) {
                    const int b = dv.n_buf[u];
                    dv.buf_frame[(size_t)u * dv.buf_max + b] = f;
                    dv.buf_owner[(size_t)u * dv.buf_max + b] = a;
                    dv.n_buf[u] = b + 1;
                    dv.mt_cnt[(size_t)u * 4 + 2] += 1;
                }
                if (act == kActForced) dv.mt_cnt[(size_t)u * 4 + 3] += 1;
                act_sh = act;
            }
            if (act == kActDefer) {                     // held in the buffer on behalf of cluster a
                dv.assign[(size_t)u * dv.F + f] = -2 - a;
                dv.pos[(size_t)u * dv.F + f] = 0;
            } else {
                n[a] = na_i + 1;
                dv.assign[(size_t)u * dv.F + f] = a;
                dv.pos[(size_t)u * dv.F + f] = na_i;
            }
        }
        __syncthreads();
        if constexpr (MAINT) {
            if (act_sh == kActSplit) {                  // workgroup-uniform
                const int fresh = mt_split_cluster<D>(dv, u, a, f + 1, false, split_sh);
                if (tid == 0) dv.mt_cnt[(size_t)u * 4 + (fresh >= 0 ? 0 : 3)] += 1;
            }
            __syncthreads();
        }
    }
}

// ---------------------------------------------------------------------------
// Online assignment + Eq. 3 with the representative table held in registers
// (maintainer off, C <= THREADS / 2).  grid (U), THREADS threads.
// The frames of a call are strictly sequential and every step of the global-
// memory version above is a dependent round trip to L2 (summary, table rows,
// winner row).  Here each 16-lane group keeps its RPG rows of the unit's table
// (row j = group + (THREADS/16) i) in registers for the whole call, sizes and
// norms sit in LDS, the next frame's summary is fetched while the current frame
// is processed, and the winner's row is updated in place (and written through),
// so nothing in the per-frame chain waits on memory.  Same arithmetic per
// element as the version above; only the norm's additions are grouped by lane.
// ---------------------------------------------------------------------------
// k_in != nullptr (one frame, THREADS = 256): the workgroup first stores frame f0's key
// page and forms its summary itself (the table loads are already in flight by then), so a
// single-frame call needs one launch instead of two.
template <int D, int THREADS, typename E>
__device__ __forceinline__ void assign_update_reg_run(const DeviceView &dv, int u, int f0, int f1, const E *k_in) {
    constexpr int EPL = D / 16, NG = THREADS / 16, RPG = 8, NW = THREADS / 64, ROWS = NG * RPG;
    constexpr int CHUNK = 32;                   // frames whose summaries are staged in LDS at a time
    const int tid = threadIdx.x, C = dv.C;
    const int lr = tid % 16, grp = tid / 16, wave = tid / 64, lane = tid % 64;
    __shared__ __attribute__((aligned(16))) double s_sh[CHUNK][D];
    __shared__ double dot_sh[ROWS], rn_sh[ROWS];
    __shared__ int n_sh[ROWS];
    __shared__ int a_out[CHUNK], p_out[CHUNK];
    __shared__ int chg_sh[ROWS];                // 1 = the cluster's size and norm changed in this call
    __shared__ double red_v[NW];
    __shared__ int red_i[NW];
    __shared__ double psum_sh[2];
    double *r = dv.r + (size_t)u * C * D;
    double rr[RPG][EPL];
#pragma unroll
    for (int i = 0; i < RPG; ++i) {
        const double *rj = r + (size_t)min(grp + NG * i, C - 1) * D + lr * EPL;
        if (NG * i < C) {                 // block-uniform: passes beyond the table are not loaded
#pragma unroll
            for (int e = 0; e < EPL; ++e) rr[i][e] = rj[e];
        } else {
#pragma unroll
            for (int e = 0; e < EPL; ++e) rr[i][e] = 0.0;
        }
    }
    for (int j = tid; j < ROWS; j += THREADS) {
        n_sh[j] = j < C ? dv.n[(size_t)u * C + j] : 0;
        rn_sh[j] = j < C ? dv.rnorm[(size_t)u * C + j] : 0.0;
        chg_sh[j] = 0;
    }
    if (k_in != nullptr) {
        if constexpr (THREADS == kBlock) {
            __shared__ double red[kBlock / (D / 8)][D];
            store_key_page<E, D>(dv, k_in, dv.k_store, u, 0, f0, red, s_sh[0]);      // HBM tier only
        }
    }
    const bool nested = dv.P > 0;
    // The barriers inside the frame loop order LDS traffic only, and the loop touches no global memory: the
    // call's summaries are staged in LDS a chunk at a time, the winner's row stays in registers and is written
    // back once after the last frame, sizes and norms live in LDS, the frames' ids and ranks collect in LDS until
    // the chunk ends.  A full __syncthreads() waits for every outstanding global access of the wavefront, and so
    // does any wait the compiler places for a register a load is still to fill: with the next frame's summary
    // fetched inside the loop and the winner's row written through in every frame, each frame waited once for
    // that load, issued a moment before, and once for the store's acknowledgement.  The nested hierarchy's
    // partition representatives and sizes do go through global memory from one frame to the next, so there the
    // barriers stay full ones.
    auto frame_barrier = [&]() {
        if (nested) __syncthreads();          // workgroup-uniform
        else lds_barrier();
    };
    unsigned int dirty = 0;                   // bit i: this group's row i changed in this call
    // a one-frame call is all latency: its results go straight to memory, with no collection and no write-back pass
    const bool single = f1 - f0 == 1;
    for (int c0 = f0; c0 < f1; c0 += CHUNK) {
        const int nc = min(CHUNK, f1 - c0);
        if (k_in == nullptr) {
            const double *src = dv.summ + ((size_t)u * dv.F + c0) * D;
            for (int i = tid; i < nc * D / 2; i += THREADS)
                *reinterpret_cast<double2 *>(&s_sh[0][0] + 2 * i) = *reinterpret_cast<const double2 *>(src + 2 * i);
        }
        __syncthreads();
        for (int fc = 0; fc < nc; ++fc) {
            const int f = c0 + fc;
            const double *sv = s_sh[fc];
            const int part_f = nested ? dv.part[f] : 0;
            const int lo = nested ? part_f * dv.Cs : 0, hi = nested ? lo + dv.Cs : C;
            // Dot products of the summary with the rows the group holds, four rows at a time written out side by
            // side: four independent multiply-add chains, then their 16-lane reductions step by step in lockstep,
            // so that one chain's latency is filled by the other three (a loop over the rows with the block-uniform
            // test per row kept every row's chain in a basic block of its own: 2100 cycles per frame for 210
            // instructions).  Rows beyond the table or of empty clusters give values nobody reads.  The group also
            // forms |s|^2 from its own share of the channels, the same bits in every group.
            double sl[EPL];
#pragma unroll
            for (int e = 0; e < EPL; ++e) sl[e] = sv[lr * EPL + e];
            double ssq = 0.0;
#pragma unroll
            for (int h = 0; h < RPG / 4; ++h) {
                if (h > 0 && NG * 4 * h >= C) break;                  // block-uniform: passes beyond the table
                double p[4] = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
                for (int e = 0; e < EPL; ++e) {
#pragma unroll
                    for (int k = 0; k < 4; ++k) p[k] += sl[e] * rr[4 * h + k][e];
                    if (h == 0) ssq += sl[e] * sl[e];
                }
#pragma unroll
                for (int k = 0; k < 4; ++k) p[k] += dpp_f64<kDppXor8>(p[k]);
                if (h == 0) ssq += dpp_f64<kDppXor8>(ssq);
#pragma unroll
                for (int k = 0; k < 4; ++k) p[k] += dpp_f64<kDppXor7>(p[k]);
                if (h == 0) ssq += dpp_f64<kDppXor7>(ssq);
#pragma unroll
                for (int k = 0; k < 4; ++k) p[k] += dpp_f64<kDppXor3>(p[k]);
                if (h == 0) ssq += dpp_f64<kDppXor3>(ssq);
#pragma unroll
                for (int k = 0; k < 4; ++k) p[k] += dpp_f64<kDppXor1>(p[k]);
                if (h == 0) ssq += dpp_f64<kDppXor1>(ssq);
                if (lr == 0) {
#pragma unroll
                    for (int k = 0; k < 4; ++k) dot_sh[grp + NG * (4 * h + k)] = p[k];
                }
            }
            const double sn = sqrt(ssq);
            frame_barrier();
            // argmax of the cosine over the candidates, ties to the lowest id (THREADS >= C: at
            // most one candidate per thread)
            double bv = -INFINITY;
            int bi = 0x7fffffff;
            {
                const int j = lo + tid;
                if (j < hi && n_sh[j] > 0) {
                    bv = (sn == 0.0 || rn_sh[j] == 0.0) ? 0.0 : dot_sh[j] / (sn * rn_sh[j]);
                    bi = j;
                }
            }
            wave_best_ascending(bv, bi);        // (ids ascend with the thread: j = lo + tid)
            if (lane == 0) { red_v[wave] = bv; red_i[wave] = bi; }
            // nested hierarchy: the partition's representative follows the same running mean
            int pn_i = 0;
            if (nested) {
                double *prow = dv.pr + ((size_t)u * dv.P + part_f) * D;
                pn_i = dv.pn[(size_t)u * dv.P + part_f];
                double psq = 0.0;
                if (tid < D) {
                    const double pv = ((double)pn_i * prow[tid] + sv[tid]) / ((double)pn_i + 1.0);
                    prow[tid] = pv;
                    psq = pv * pv;
                }
                if (wave < 2) {
                    psq = wave_sum(psq);
                    if (lane == 0) psum_sh[wave] = psq;
                }
            }
            frame_barrier();
            // every thread merges the wavefronts' winners itself (no second barrier for one thread's merge)
            bv = red_v[0]; bi = red_i[0];
#pragma unroll
            for (int w = 1; w < NW; ++w)
                if (better(red_v[w], red_i[w], bv, bi)) { bv = red_v[w]; bi = red_i[w]; }
            const int a = bi == 0x7fffffff ? lo : bi;
            const int ai = __builtin_amdgcn_readfirstlane(a / NG);      // workgroup-uniform: a scalar
            if (grp == a % NG) {                                  // the group that holds row a
                const int na_i = n_sh[a];
                const double na = (double)na_i;
                // Eq. 3 with each operation rounded separately (no contraction).  The division by n + 1, the same
                // divisor for the lane's eight channels: the compiler's division sequence hands a flag from its
                // scaling step to its last step in VCC, so eight of them run one after the other (1400 cycles).
                // Instead y = RN(1 / (n + 1)) once, then per channel q = RN(x y) and two residual corrections
                // q <- RN(q + RN(x - (n + 1) q) y), each residual exact in a fused multiply-add: the first leaves q
                // within half an ulp and a little of x / (n + 1), and from such a q and a correctly rounded y the
                // second returns the correctly rounded quotient (Markstein's theorem; n + 1 is a small integer, so
                // its significand is not all ones, and nothing here is near the ends of the exponent range).
                const double nb = na + 1.0, ny = __ddiv_rn(1.0, nb);
                double sq = 0.0;
#pragma unroll
                for (int i = 0; i < RPG; ++i) {
                    if (i == ai) {                                // scalar branch: one pass runs
#pragma unroll
                        for (int e = 0; e < EPL; ++e) {
                            const double x = __dadd_rn(__dmul_rn(na, rr[i][e]), sl[e]);
                            double rv = __dmul_rn(x, ny);
                            rv = __fma_rn(__fma_rn(-nb, rv, x), ny, rv);
                            rv = __fma_rn(__fma_rn(-nb, rv, x), ny, rv);
                            rr[i][e] = rv;
                            if (single) r[(size_t)a * D + lr * EPL + e] = rv;
                            sq += rv * rv;
                        }
                    }
                }
                if (!single) dirty |= 1u << ai;
                sq = row16_sum(sq);
                if (lr == 0) {
                    const double nr = sqrt(sq);
                    if (single) {
                        dv.rnorm[(size_t)u * C + a] = nr;
                        dv.n[(size_t)u * C + a] = na_i + 1;
                        dv.assign[(size_t)u * dv.F + f] = a;
                        dv.pos[(size_t)u * dv.F + f] = na_i;
                    } else {
                        rn_sh[a] = nr;
                        n_sh[a] = na_i + 1;
                        chg_sh[a] = 1;
                        a_out[fc] = a;
                        p_out[fc] = na_i;
                    }
                }
            }
            if (nested && tid == 0) {
                dv.prn[(size_t)u * dv.P + part_f] = sqrt(D > 64 ? psum_sh[0] + psum_sh[1] : psum_sh[0]);
                dv.pn[(size_t)u * dv.P + part_f] = pn_i + 1;
            }
            if (single) return;                   // workgroup-uniform: nothing follows the only frame
            frame_barrier();
        }
        // the chunk's ids and ranks (the barrier that ended its last frame made them visible)
        if (tid < nc) {
            dv.assign[(size_t)u * dv.F + c0 + tid] = a_out[tid];
            dv.pos[(size_t)u * dv.F + c0 + tid] = p_out[tid];
        }
        __syncthreads();                          // before the next chunk overwrites the staged summaries
    }
    // write back what changed: rows, sizes and norms
#pragma unroll
    for (int i = 0; i < RPG; ++i) {
        if ((dirty >> i) & 1u) {
#pragma unroll
            for (int e = 0; e < EPL; ++e) r[(size_t)(grp + NG * i) * D + lr * EPL + e] = rr[i][e];
        }
    }
    for (int j = tid; j < C; j += THREADS) {
        if (chg_sh[j]) {
            dv.n[(size_t)u * C + j] = n_sh[j];
            dv.rnorm[(size_t)u * C + j] = rn_sh[j];
        }
    }
}

template <int D, int THREADS>
__global__ __launch_bounds__(THREADS) void k_assign_update_reg(DeviceView dv, int f0, int f1) {
    assign_update_reg_run<D, THREADS, float>(dv, blockIdx.x, f0, f1, nullptr);
}

// One frame in one launch (maintainer off, C <= 128, HBM tier, online phase).
// grid (U, 2), 256 threads: y = 0 key page + summary + assignment + Eq. 3, y = 1 value page.
template <typename E, int D>
__global__ __launch_bounds__(kBlock) void k_ingest_one(DeviceView dv, const E *k_in, const E *v_in, int f) {
    if (blockIdx.y == 1) {
        __shared__ double red[kBlock / (D / 8)][D];
        store_value_page<E, D>(dv, v_in, dv.v_store, blockIdx.x, 0, f, red);         // HBM tier only
        return;
    }
    assign_update_reg_run<D, kBlock, E>(dv, blockIdx.x, f, f + 1, k_in);
}

// ---------------------------------------------------------------------------
// Lloyd: seeds from the warm-up buffer.  grid (U), 256 threads.
// r_j = summary of frame floor(j*W/C); every cluster counts as non-empty for
// the first assignment round (n_j = 1 as a placeholder).
// ---------------------------------------------------------------------------
// With the maintainer on only the first c_init ids are seeded (the rest of the
// table is empty until splits fill it) and the maintainer's state is cleared.
template <int D>
__global__ __launch_bounds__(kBlock) void k_lloyd_seed(DeviceView dv, int W) {
    constexpr int EPL = D / 16;
    const int u = blockIdx.x, tid = threadIdx.x, C = dv.C;
    const int Cl = dv.maint_mode ? dv.c_init : C;
    const int lr = tid % 16, row0 = tid / 16;
    for (int j = row0; j < C; j += 16) {
        double *rj = dv.r + ((size_t)u * C + j) * D + lr * EPL;
        if (j >= Cl) {
#pragma unroll
            for (int i = 0; i < EPL; ++i) rj[i] = 0.0;
            if (lr == 0) { dv.rnorm[(size_t)u * C + j] = 0.0; dv.n[(size_t)u * C + j] = 0; }
            continue;
        }
        const int src = (int)(((long long)j * W) / Cl);
        const double *s = dv.summ + ((size_t)u * dv.F + src) * D + lr * EPL;
        double sq = 0.0;
#pragma unroll
        for (int i = 0; i < EPL; ++i) { rj[i] = s[i]; sq += s[i] * s[i]; }
        sq = group16_sum(sq);
        if (lr == 0) { dv.rnorm[(size_t)u * C + j] = sqrt(sq); dv.n[(size_t)u * C + j] = 1; }
    }
    if (dv.maint_mode) {
        for (int j = tid; j < C; j += kBlock) {
            dv.var[(size_t)u * C + j] = 0.0;
            dv.lazy[(size_t)u * C + j] = 0;
            dv.resident[(size_t)u * C + j] = 0;
        }
        if (tid == 0) { dv.n_slots[u] = Cl; dv.n_buf[u] = 0; }
        if (tid < 4) dv.mt_cnt[(size_t)u * 4 + tid] = 0;
    }
}

// ---------------------------------------------------------------------------
// Seeds under the nested hierarchy (Sec. V-B).  grid (U), 256 threads.
// Cluster id j = p*Cs + jj belongs to visual partition p.  With np warm-up
// frames in p and L = min(Cs, np), id j is started (n_j = 1 as a placeholder)
// from the summary of the partition's member floor(jj*np/L) if jj < L and is
// left empty otherwise.
// ---------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(kBlock) void k_lloyd_seed_nested(DeviceView dv, int W) {
    constexpr int EPL = D / 16;
    const int u = blockIdx.x, tid = threadIdx.x, C = dv.C, Cs = dv.Cs;
    const int lr = tid % 16, row0 = tid / 16;
    constexpr int kPartLds = 8192;            // warm-up partitions are scanned out of LDS when they fit
    __shared__ int np_sh[64];
    __shared__ int part_sh[kPartLds];
    const bool in_lds = W <= kPartLds;
    if (in_lds)
        for (int f = tid; f < W; f += kBlock) part_sh[f] = dv.part[f];
    __syncthreads();
    const int *part = in_lds ? part_sh : dv.part;
    // member lists of the partitions, ascending, back to back in the unit's (not yet used)
    // rank array: thread p counts, thread 0 lays out the starts, thread p fills its list
    __shared__ int start_sh[65];
    int *order = dv.pos + (size_t)u * dv.F;
    if (tid < dv.P) {
        int c = 0;
        for (int f = 0; f < W; ++f) c += part[f] == tid;
        np_sh[tid] = c;
    }
    __syncthreads();
    if (tid == 0) {
        int o = 0;
        for (int p = 0; p < dv.P; ++p) { start_sh[p] = o; o += np_sh[p]; }
    }
    __syncthreads();
    if (tid < dv.P) {
        int o = start_sh[tid];
        for (int f = 0; f < W; ++f)
            if (part[f] == tid) order[o++] = f;
    }
    __syncthreads();
    for (int j = row0; j < C; j += 16) {
        const int p = j / Cs, jj = j - p * Cs, np = np_sh[p], L = min(Cs, np);
        double *rj = dv.r + ((size_t)u * C + j) * D + lr * EPL;
        if (jj >= L) {
#pragma unroll
            for (int i = 0; i < EPL; ++i) rj[i] = 0.0;
            if (lr == 0) { dv.rnorm[(size_t)u * C + j] = 0.0; dv.n[(size_t)u * C + j] = 0; }
            continue;
        }
        const int src = order[start_sh[p] + (int)(((long long)jj * np) / L)];
        const double *s = dv.summ + ((size_t)u * dv.F + src) * D + lr * EPL;
        double sq = 0.0;
#pragma unroll
        for (int i = 0; i < EPL; ++i) { rj[i] = s[i]; sq += s[i] * s[i]; }
        sq = group16_sum(sq);
        if (lr == 0) { dv.rnorm[(size_t)u * C + j] = sqrt(sq); dv.n[(size_t)u * C + j] = 1; }
    }
}

// ---------------------------------------------------------------------------
// Partition representatives from the member lists: per unit and visual
// partition the mean of the key summaries of the partition's frames, in
// ascending frame order.  grid (U, P), 128 threads (thread d owns channel d).
// ---------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(128) void k_partition_reps(DeviceView dv, int n_frames) {
    const int u = blockIdx.x, p = blockIdx.y, tid = threadIdx.x, wave = tid / 64, lane = tid % 64;
    __shared__ double nsum_sh[2];
    double acc = 0.0;
    int count = 0;
    for (int f = 0; f < n_frames; ++f) {
        if (dv.part[f] != p) continue;                   // workgroup-uniform
        if (tid < D) acc += dv.summ[((size_t)u * dv.F + f) * D + tid];
        ++count;
    }
    double sq = 0.0;
    if (tid < D) {
        const double rv = count > 0 ? acc / (double)count : 0.0;
        dv.pr[((size_t)u * dv.P + p) * D + tid] = rv;
        sq = rv * rv;
    }
    sq = wave_sum(sq);
    if (lane == 0) nsum_sh[wave] = sq;
    __syncthreads();
    if (tid == 0) {
        dv.prn[(size_t)u * dv.P + p] = sqrt(nsum_sh[0] + nsum_sh[1]);
        dv.pn[(size_t)u * dv.P + p] = count;
    }
}

// ---------------------------------------------------------------------------
// Intra-cluster variance from the member lists (Eq. 2), after a K-means run.
// grid (U, clusters), 256 threads: 16-lane groups take members in turn, the
// group partials are added in a fixed order.
// ---------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(kBlock) void k_exact_var(DeviceView dv, int n_frames) {
    constexpr int EPL = D / 16, NG = kBlock / 16;
    const int u = blockIdx.x, j = blockIdx.y, tid = threadIdx.x, C = dv.C;
    const int lr = tid % 16, grp = tid / 16;
    __shared__ double part[NG];
    const int *assign = dv.assign + (size_t)u * dv.F;
    const double *rj = dv.r + ((size_t)u * C + j) * D + lr * EPL;
    double rv[EPL];
#pragma unroll
    for (int i = 0; i < EPL; ++i) rv[i] = rj[i];
    double acc = 0.0;
    for (int f = grp; f < n_frames; f += NG) {
        if (assign[f] != j) continue;                    // uniform within the 16-lane group
        const double *s = dv.summ + ((size_t)u * dv.F + f) * D + lr * EPL;
        double p = 0.0;
#pragma unroll
        for (int i = 0; i < EPL; ++i) { const double t = s[i] - rv[i]; p += t * t; }
        acc += group16_sum(p);
    }
    if (lr == 0) part[grp] = acc;
    __syncthreads();
    if (tid == 0) {
        double tot = 0.0;
        for (int g = 0; g < NG; ++g) tot += part[g];
        const int cnt = dv.n[(size_t)u * C + j];
        dv.var[(size_t)u * C + j] = cnt > 0 ? tot / (double)cnt : 0.0;
    }
}

// ---------------------------------------------------------------------------
// Lloyd assignment round: similarity table = summaries x representatives^T, a
// dense fp64 contraction, on the matrix cores (v_mfma_f64_16x16x4_f64: A lane
// (row = lane%16, k = lane/16), B lane (col = lane%16, k = lane/16), result
// register v of a lane = element (row 4v + lane/16, col lane%16)).
// grid (U, ceil(F/64)), 256 threads: a wavefront owns 16 frames, keeps their
// summaries in registers as the A operand for the whole call, and sweeps the
// representatives 16 at a time (each tile staged once per workgroup in LDS,
// double buffered, the next tile in flight behind the current tile's MFMAs).  Lane group k
// holds channels 8s + 2k and 8s + 2k + 1 of k-step s (one 16-byte load feeds two
// MFMAs); the order of the additions inside a dot product is therefore not the
// channel order, which moves a similarity by rounding only.
// ---------------------------------------------------------------------------
typedef double f64x4 __attribute__((ext_vector_type(4)));
typedef double f64x2 __attribute__((ext_vector_type(2)));

// Rounds that change nothing are skipped: a round `it` that moved no frame of a unit leaves the same
// members, hence (the sums being one fixed sequence of additions) the same representatives bit for
// bit, hence the same assignments in every later round.  moved[u][it % 3] counts the frames round
// `it` moved; a round whose predecessor moved none returns at once (and so does its update kernel).
// The slot of the round after is cleared by this launch, which neither reads nor counts in it.
//
// Frames whose assignment cannot change are skipped as well, by the distance bounds of accelerated
// K-means (Hamerly, SDM 2010) taken on the unit sphere, where the largest cosine is the smallest chord
// d(s, r) = |s/|s| - r/|r|| = sqrt(2 - 2 cos): a round that computes a frame's similarities leaves
// ub = d(own representative) and lb = d(best other candidate); an update that moves representative j by
// delta_j = d(old r_j, new r_j) can shrink any frame's distance to it by at most delta_j, so after it
// ub + delta_own still bounds the own distance from above and lb - max_{j != own} delta_j the others from
// below (triangle inequality).  While ub + 1e-6 < lb the own representative wins by a margin far above
// the rounding of the similarities (> 5e-13 in the cosine) and the full computation would return the same
// id: a row of 16 frames (what one wavefront multiplies) whose frames all pass only gets the moved bounds
// stored (k_lloyd_bounds); any other is recomputed in full and leaves exact bounds again.  Round 0 computes
// everything.  After the first round a handful of frames per unit keeps moving and a few representatives with
// them, so most rows pass.  The assignments are the same as without the test, by construction.
constexpr double kBoundMargin = 1e-6;

// The bound test of a round it >= 1, for all frames of a unit: grid (U, ceil(F/1024)), 256 threads, a lane per
// frame, sixteen consecutive frames (what one wavefront of k_lloyd_assign multiplies) per 16-lane row.  A row
// whose frames all pass stores their moved bounds; any other is appended to the unit's list of live rows
// (order of arrival: every frame's result is independent of it), which k_lloyd_assign then works through
// four rows per workgroup, so that the few rows still alive fill whole workgroups.
__global__ __launch_bounds__(kBlock) void k_lloyd_bounds(DeviceView dv, int n_frames, int it) {
    const int u = blockIdx.x, tid = threadIdx.x, wave = tid / 64, lane = tid % 64, C = dv.C;
    int *n_live = dv.lloyd_moved + (size_t)dv.U * 3 + (size_t)u * 3;
    if (blockIdx.y == 0 && tid == 0) n_live[(it + 1) % 3] = 0;
    if (dv.lloyd_moved[(size_t)u * 3 + (it - 1) % 3] == 0) return;      // converged (as in k_lloyd_assign)
    __shared__ double top_v[4][2];
    __shared__ int top_j[4];
    // largest and second largest movement of a representative in the last update, and whose the largest was
    const double *delta = dv.lloyd_delta + (size_t)u * C;
    double d1 = 0.0, d2 = 0.0;
    int j1 = -1;
    for (int j = tid; j < C; j += kBlock) {
        const double dj = delta[j];
        if (dj > d1) { d2 = d1; d1 = dj; j1 = j; }
        else if (dj > d2) d2 = dj;
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
        const double o1 = __shfl_xor(d1, o, 64), o2 = __shfl_xor(d2, o, 64);
        const int oj = __shfl_xor(j1, o, 64);
        if (o1 > d1) { d2 = fmax(d1, o2); d1 = o1; j1 = oj; }
        else d2 = fmax(d2, o1);
    }
    if (lane == 0) { top_v[wave][0] = d1; top_v[wave][1] = d2; top_j[wave] = j1; }
    __syncthreads();
    d1 = top_v[0][0]; d2 = top_v[0][1]; j1 = top_j[0];
#pragma unroll
    for (int w = 1; w < 4; ++w) {
        const double o1 = top_v[w][0], o2 = top_v[w][1];
        if (o1 > d1) { d2 = fmax(d1, o2); d1 = o1; j1 = top_j[w]; }
        else d2 = fmax(d2, o1);
    }
    const int fend = min(n_frames, (int)(blockIdx.y + 1) * 1024);
    for (int f0 = blockIdx.y * 1024 + wave * 64; f0 < fend; f0 += kBlock) {
        const int f = f0 + lane;
        bool safe = true;
        double ubn = 0.0, lbn = 0.0;
        if (f < n_frames) {
            const int a_old = dv.assign[(size_t)u * dv.F + f];
            ubn = dv.lloyd_ub[(size_t)u * dv.F + f] + delta[a_old];
            lbn = dv.lloyd_lb[(size_t)u * dv.F + f] - (a_old == j1 ? d2 : d1);
            safe = ubn + kBoundMargin < lbn;
        }
        const unsigned long long unsafe = __ballot(!safe);
        const bool row_live = ((unsafe >> (lane & 48)) & 0xffffull) != 0ull;
        if (!row_live && f < n_frames) {
            dv.lloyd_ub[(size_t)u * dv.F + f] = ubn;
            dv.lloyd_lb[(size_t)u * dv.F + f] = lbn;
        }
        // the wavefront's live rows (at most four) take consecutive slots of the list
        unsigned int rows = 0;
#pragma unroll
        for (int g = 0; g < 4; ++g) rows |= (((unsafe >> (16 * g)) & 0xffffull) != 0ull ? 1u : 0u) << g;
        if (rows) {
            int base = 0;
            if (lane == 0) base = atomicAdd(&n_live[it % 3], __popc(rows));
            base = __shfl(base, 0, 64);
            const int g = lane / 16;
            if ((lane & 15) == 0 && ((rows >> g) & 1u))
                dv.lloyd_live[(size_t)u * ((dv.F + 15) / 16) + base + __popc(rows & ((1u << g) - 1u))] = f0 / 16 + g;
        }
    }
}

// LATER: the instantiation for the rounds after the first.  Their launches are mostly workgroups that find nothing to
// do and lone tasks that are all latency, so it may use more registers (two wavefronts per SIMD are plenty) to start
// every independent load at once: both round counters and the wavefront's list entry together, the frames' old ids
// with the operands, the table built while the operands travel; and its bounds take their roots in fp32.
template <int D, bool LATER>
__global__ __launch_bounds__(kBlock, LATER ? 2 : 3) void k_lloyd_assign(DeviceView dv, int n_frames, int it) {
    constexpr int KS = D / 8;
    const int u = blockIdx.x, tid = threadIdx.x, wave = tid / 64, lane = tid % 64, C = dv.C;
    const int row = lane % 16, kq = lane / 16;
    int *moved = dv.lloyd_moved + (size_t)u * 3;
    if (blockIdx.y == 0 && tid == 0) moved[(it + 1) % 3] = 0;
    // Round 0: one task per workgroup, wavefront w of workgroup y takes frames 64 y + 16 w ...  Later rounds:
    // task t = rows 4 t .. 4 t + 3 of the unit's list of live rows, the workgroups of a unit taking tasks in turn.
    const int n_rows = (dv.F + 15) / 16;
    const int *live_list = dv.lloyd_live + (size_t)u * n_rows;
    int cnt = 0, first_row = 0;
    if constexpr (LATER) {
        const int moved_before = moved[(it - 1) % 3];
        cnt = dv.lloyd_moved[(size_t)dv.U * 3 + (size_t)u * 3 + it % 3];
        first_row = live_list[min((int)blockIdx.y * 4 + wave, n_rows - 1)];
        if (moved_before == 0) return;                         // workgroup-uniform: converged in an earlier round
        if ((int)blockIdx.y * 4 >= cnt) return;                // workgroup-uniform
    }
    const double *r = dv.r + (size_t)u * C * D;
    const int n_tiles = (C + 15) / 16;
    // A tile of 16 representatives is shared by the four wavefronts through LDS (each row is read
    // from L2 once per workgroup); rows are padded by 16 bytes so that the 16 lanes of a k group hit
    // 16 different 16-byte bank groups.  Tile ct+1 travels global -> registers while tile ct is used.
    constexpr int LROW = D + 2, PPT = 16 * D / 2 / kBlock;        // doubles per LDS row; 16-byte pieces per thread
    __shared__ __attribute__((aligned(16))) double b_lds[2][16][LROW];
    f64x2 stg[PPT];
    auto fetch_tile = [&](int ct) {
#pragma unroll
        for (int i = 0; i < PPT; ++i) {
            const int p = tid + kBlock * i, trow = p / (D / 2), seg = p % (D / 2);
            stg[i] = *reinterpret_cast<const f64x2 *>(r + (size_t)min(16 * ct + trow, C - 1) * D + 2 * seg);
        }
    };
    auto stage_tile = [&](int buf) {
#pragma unroll
        for (int i = 0; i < PPT; ++i) {
            const int p = tid + kBlock * i, trow = p / (D / 2), seg = p % (D / 2);
            *reinterpret_cast<f64x2 *>(&b_lds[buf][trow][2 * seg]) = stg[i];
        }
    };
    // The ranking of a frame's similarities does not need the division by |s| |r_j| per candidate: |s| is the
    // same positive factor for every j, so the winner is argmax_j dot_j * (1 / |r_j|).  The fp64 matrix
    // instruction runs on the vector unit's fp64 lanes (counters: no cycle in which both execute), so every
    // vector instruction of the tile epilogue is time taken from the contraction: per candidate one fused
    // multiply-add, dot * scale_j + offset_j, with the pair formed once per workgroup in LDS: (1 / |r_j|, 0) for
    // a candidate, (0, 0) for a zero representative (its cosine is 0), (0, -inf) for an empty cluster and past
    // the table's end.  An all-zero summary gives 0 for every candidate and so the lowest id, as its cosines
    // (all 0) do.
    __shared__ __attribute__((aligned(16))) f64x2 scale_sh[1024 + 16];    // the cluster-count limit of a context, rounded up to tiles
    __shared__ double sn_sh[4][16];
    auto build_table = [&]() {
        for (int j = tid; j < 16 * n_tiles; j += kBlock) {
            f64x2 e = {0.0, -INFINITY};
            if (j < C && dv.n[(size_t)u * C + j] > 0) {
                const double rnj = dv.rnorm[(size_t)u * C + j];
                e.x = rnj == 0.0 ? 0.0 : 1.0 / rnj;
                e.y = 0.0;
            }
            scale_sh[j] = e;
        }
    };
    if constexpr (!LATER) build_table();
    const bool nested = dv.P > 0;
    for (int task = blockIdx.y;; task += gridDim.y) {
        int fbase = task * 64 + wave * 16;
        bool live = true;
        if constexpr (LATER) {
            if (task * 4 >= cnt) break;                         // workgroup-uniform
            live = task * 4 + wave < cnt;
            fbase = !live ? 0 : 16 * (task == (int)blockIdx.y ? first_row : live_list[task * 4 + wave]);
        }
        fetch_tile(0);
        f64x2 a[KS];
        int a_old[4] = {0, 0, 0, 0};     // LATER: the frames' ids before this round, for the lane that finishes them
        if (live) {
            const int f = min(fbase + row, n_frames - 1);
            const double *sp = dv.summ + ((size_t)u * dv.F + f) * D + 2 * kq;
#pragma unroll
            for (int s = 0; s < KS; ++s) a[s] = *reinterpret_cast<const f64x2 *>(sp + 8 * s);
            if constexpr (LATER) {
#pragma unroll
                for (int v = 0; v < 4; ++v) a_old[v] = dv.assign[(size_t)u * dv.F + min(fbase + 4 * v + kq, n_frames - 1)];
            }
        }
        if constexpr (LATER) {
            if (task == (int)blockIdx.y) build_table();        // once, while the summaries are on their way
        }
        if (live) {
            double sq = 0.0;
#pragma unroll
            for (int s = 0; s < KS; ++s) sq += a[s].x * a[s].x + a[s].y * a[s].y;
            sq += __shfl_xor(sq, 16, 64);
            sq += __shfl_xor(sq, 32, 64);
            if (kq == 0) sn_sh[wave][row] = sqrt(sq);
        }
        // the four result rows of this lane: frames fbase + 4v + kq; best and second best similarity (times |s|)
        double bv[4], sv[4];
        int plo[4], phi[4], bi[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            bv[v] = -INFINITY; sv[v] = -INFINITY; bi[v] = 0x7fffffff;
            plo[v] = 0; phi[v] = C;
            if (nested) {        // nested hierarchy: only the ids of the frame's visual partition are candidates
                plo[v] = dv.part[min(fbase + 4 * v + kq, n_frames - 1)] * dv.Cs;
                phi[v] = plo[v] + dv.Cs;
            }
        }
        stage_tile(0);
        __syncthreads();
        for (int ct = 0; ct < n_tiles; ++ct) {
            const int ctn = min(ct + 1, n_tiles - 1);
            fetch_tile(ctn);
            if (live) {
                f64x2 b[KS];
#pragma unroll
                for (int s = 0; s < KS; ++s) b[s] = *reinterpret_cast<const f64x2 *>(&b_lds[ct & 1][row][8 * s + 2 * kq]);
                const f64x2 sc = scale_sh[16 * ct + row];
                // one accumulator chain: back-to-back matrix instructions on the same accumulator sustain 70 TFLOP/s
                // in a probe of nothing else, two alternating accumulators 66, four 58
                f64x4 acc = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
                for (int s = 0; s < KS; ++s) {
                    acc = __builtin_amdgcn_mfma_f64_16x16x4f64(a[s].x, b[s].x, acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f64_16x16x4f64(a[s].y, b[s].y, acc, 0, 0, 0);
                }
                const int j = 16 * ct + row;
                // A lane meets its candidates in ascending id order, so a strict comparison keeps the lowest id of
                // equals; the second best is kept for the bounds.
                if (nested) {
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        double c = __builtin_fma(acc[v], sc.x, sc.y);
                        if (j < plo[v] || j >= phi[v]) c = -INFINITY;
                        bi[v] = c > bv[v] ? j : bi[v];
                        sv[v] = max_f64(sv[v], min_f64(bv[v], c));
                        bv[v] = max_f64(bv[v], c);
                    }
                } else {
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const double c = __builtin_fma(acc[v], sc.x, sc.y);
                        bi[v] = c > bv[v] ? j : bi[v];
                        sv[v] = max_f64(sv[v], min_f64(bv[v], c));
                        bv[v] = max_f64(bv[v], c);
                    }
                }
            }
            stage_tile((ct + 1) & 1);       // the other buffer: last read before the previous barrier
            __syncthreads();
        }
        if (live) {
            // best and second best over the 16 columns a lane group covers (lanes 16k .. 16k + 15)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
#pragma unroll
                for (int o = 8; o >= 1; o >>= 1) {
                    const double ov = __shfl_xor(bv[v], o, 16), os = __shfl_xor(sv[v], o, 16);
                    const int oi = __shfl_xor(bi[v], o, 16);
                    if (better(ov, oi, bv[v], bi[v])) { sv[v] = max_f64(bv[v], os); bv[v] = ov; bi[v] = oi; }
                    else sv[v] = max_f64(sv[v], ov);
                }
                const int f = fbase + 4 * v + kq;
                if (row == 0 && f < n_frames) {
                    const bool none = bv[v] == -INFINITY;            // no candidate at all: the first id of the range
                    const int a_new = none ? plo[v] : bi[v];
                    int *slot = dv.assign + (size_t)u * dv.F + f;
                    const int a_was = LATER ? a_old[v] : *slot;
                    if (a_was != a_new) {
                        *slot = a_new;
                        atomicAdd(&moved[it % 3], 1);
                        // both clusters' sums change; every other cluster's update is skipped (round 0 updates all)
                        dv.lloyd_changed[(size_t)u * C + a_new] = 1;
                        if (a_was >= 0 && a_was < C) dv.lloyd_changed[(size_t)u * C + a_was] = 1;
                    }
                    // chords to the winner and to the best other candidate (a frame without a winner, or an all-zero
                    // summary, whose cosines are all 0, is never skipped)
                    const double sn = sn_sh[wave][4 * v + kq];
                    double ubn = 2.0, lbn = 0.0;
                    if (!none && sn > 0.0) {
                        if constexpr (LATER) {
                            // They only have to bound: roots in fp32 (relative error below 2e-7 with the conversion),
                            // pushed outwards by 1e-6 relative and 1e-9 absolute; an fp64 root is a dozen instructions
                            // and, like the fp64 division, keeps a flag in VCC, so a lane's eight ran one after the other.
                            const double inv = 1.0 / sn;
                            ubn = (double)sqrtf((float)fmax(0.0, 2.0 - 2.0 * (bv[v] * inv))) * (1.0 + 1e-6) + 1e-9;
                            lbn = sv[v] == -INFINITY
                                      ? INFINITY
                                      : fmax(0.0, (double)sqrtf((float)fmax(0.0, 2.0 - 2.0 * (sv[v] * inv))) * (1.0 - 1e-6) - 1e-9);
                        } else {
                            ubn = sqrt(fmax(0.0, 2.0 - 2.0 * (bv[v] / sn)));
                            lbn = sv[v] == -INFINITY ? INFINITY : sqrt(fmax(0.0, 2.0 - 2.0 * (sv[v] / sn)));
                        }
                    }
                    dv.lloyd_ub[(size_t)u * dv.F + f] = ubn;
                    dv.lloyd_lb[(size_t)u * dv.F + f] = lbn;
                }
            }
        }
        if constexpr (!LATER) break;
    }
}

// ---------------------------------------------------------------------------
// Lloyd update round.  grid (U, C), 128 threads (thread d owns channel d).
// Members are found by an order-preserving compaction of the assignment array,
// 2048 frames at a time: the assignments are staged in LDS with coalesced loads,
// every thread then looks at 16 consecutive frames, a scan over the threads' match
// counts gives each match its slot, and the member summaries are added in ascending
// frame order, so the mean is the same sequence of additions a sequential loop would
// perform.  The launch reads every fp64 summary of every unit once (1 KB per frame and
// unit: 470 MB at 112 units x 4096 frames), which is what bounds it.
// ---------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(128) void k_lloyd_update(DeviceView dv, int n_frames, int it) {
    constexpr int NT = 128, FPT = 16, CH = NT * FPT;
    const int u = blockIdx.x, j = blockIdx.y, tid = threadIdx.x, C = dv.C;
    // (a round that moved no frame would rebuild the same sums: see k_lloyd_assign)
    if (it > 0 && dv.lloyd_moved[(size_t)u * 3 + it % 3] == 0) return;
    // A cluster that no frame entered or left in this round (flags set by k_lloyd_assign) has the same
    // members, so the same sums bit for bit: it is not recomputed, and its representative has not moved.
    // Round 0 recomputes every cluster (the online running means are not the ordered sums).
    int *changed = dv.lloyd_changed + (size_t)u * C + j;
    double *delta = dv.lloyd_delta + (size_t)u * C + j;
    if (it > 0 && *changed == 0) {                   // workgroup-uniform: the flag is cleared only after the last barrier
        if (tid == 0) *delta = 0.0;
        return;
    }
    const double norm_old = dv.rnorm[(size_t)u * C + j];
    const int wave = tid / 64, lane = tid % 64;
    __shared__ int a_sh[CH];
    __shared__ int mem[CH];
    __shared__ int wtot[2];
    __shared__ double nsum_sh[2], dsum_sh[2];
    const int *assign = dv.assign + (size_t)u * dv.F;
    int *pos = dv.pos + (size_t)u * dv.F;
    double acc = 0.0;
    int count = 0;
    for (int c0 = 0; c0 < n_frames; c0 += CH) {
        const int cend = min(n_frames, c0 + CH);
#pragma unroll
        for (int i = 0; i < FPT; ++i) {
            const int f = c0 + tid + NT * i;
            a_sh[tid + NT * i] = f < cend ? assign[f] : -1;
        }
        __syncthreads();
        unsigned int mask = 0;               // bit i: frame c0 + 16 tid + i belongs to cluster j
#pragma unroll
        for (int i = 0; i < FPT; ++i) mask |= (a_sh[tid * FPT + i] == j ? 1u : 0u) << i;
        const int mine = __popc(mask);
        int incl = mine;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int t = __shfl_up(incl, o, 64);
            if (lane >= o) incl += t;
        }
        if (lane == 63) wtot[wave] = incl;
        __syncthreads();
        int slot = incl - mine + (wave == 1 ? wtot[0] : 0);
        const int filled = wtot[0] + wtot[1];   // members found in this chunk (same in every thread)
        while (mask) {
            const int i = __ffs((int)mask) - 1;
            mask &= mask - 1;
            const int f = c0 + tid * FPT + i;
            mem[slot] = f;
            pos[f] = count + slot;
            ++slot;
        }
        __syncthreads();
        if (tid < D) {
            // sixteen members' loads in flight at a time (index clamped, loads unconditional), added in order
            // (thirty-two: slower, 75 against 68 us on average over a pass of config 2)
            constexpr int NL = 16;
            const double *sb = dv.summ + (size_t)u * dv.F * D + tid;
            for (int m0 = 0; m0 < filled; m0 += NL) {
                double v[NL];
#pragma unroll
                for (int x = 0; x < NL; ++x) v[x] = sb[(size_t)mem[min(m0 + x, filled - 1)] * D];
#pragma unroll
                for (int x = 0; x < NL; ++x)
                    if (m0 + x < filled) acc += v[x];
            }
        }
        count += filled;
    }
    if (count == 0) {                      // keeps its representative, skipped from now on
        if (tid == 0) { dv.n[(size_t)u * C + j] = 0; *delta = 0.0; *changed = 0; }
        return;
    }
    double sq = 0.0, rv = 0.0, r_old = 0.0;
    if (tid < D) {
        r_old = dv.r[((size_t)u * C + j) * D + tid];
        rv = acc / (double)count;
        dv.r[((size_t)u * C + j) * D + tid] = rv;
        sq = rv * rv;
    }
    sq = wave_sum(sq);
    if (lane == 0) nsum_sh[wave] = sq;
    __syncthreads();
    // how far the representative moved on the unit sphere (chord between the old and the new direction): what
    // k_lloyd_assign's bounds are moved by; 2, the largest chord there is, if either is the zero vector
    const double norm_new = sqrt(nsum_sh[0] + nsum_sh[1]);
    const bool both = norm_old > 0.0 && norm_new > 0.0;
    double dd = 0.0;
    if (tid < D && both) {
        const double t = r_old / norm_old - rv / norm_new;
        dd = t * t;
    }
    dd = wave_sum(dd);
    if (lane == 0) dsum_sh[wave] = dd;
    __syncthreads();
    if (tid == 0) {
        dv.rnorm[(size_t)u * C + j] = norm_new;
        dv.n[(size_t)u * C + j] = count;
        *delta = both ? sqrt(dsum_sh[0] + dsum_sh[1]) : 2.0;
        *changed = 0;
    }
}

// ---------------------------------------------------------------------------
// Host tier: store staged pages into their cluster's slab in pinned host memory
// (device stores over PCIe, 16 bytes per lane, whole pages contiguous).
// A few dozen workgroups share the (unit, frame, keys | values) items: the launch
// runs on the copy stream beside the next batch's staging and assignment, and
// one workgroup per page would hold the chip while it waits for the link.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void k_offload(DeviceView dv, int f0, int n) {
    const int n_items = dv.U * n * 2;
    for (int it = blockIdx.x; it < n_items; it += gridDim.x) {
        const int val = it & 1, u = (it >> 1) % dv.U, fl = (it >> 1) / dv.U, f = f0 + fl;
        const size_t bytes = val ? dv.vpage : dv.kpage;
        const size_t spage = (size_t)(f % dv.SN) * dv.U + u;
        const int hp = dv.dest[(size_t)u * dv.SN + fl];        // page within the unit's host pool
        const size_t hoff = (size_t)u * dv.h_ustride + (size_t)(hp / dv.SFh) * dv.h_bstride + (size_t)(hp % dv.SFh) * bytes;
        const uint4 *src = reinterpret_cast<const uint4 *>((val ? dv.stage_v : dv.stage_k) + spage * bytes);
        uint4 *dst = reinterpret_cast<uint4 *>((val ? dv.host_v : dv.host_k) + hoff);
        for (size_t i = threadIdx.x; i < bytes / 16; i += kBlock) dst[i] = src[i];
    }
}

// ---------------------------------------------------------------------------
// Host tier: cluster fetch.  One launch moves every missing page of a layer's
// selection from the pinned slabs into the GPU cluster cache: the kernel loads
// straight from host memory over PCIe (16 bytes per lane), which streams at the
// rate of a large DMA copy and costs one launch instead of one runtime call per
// slab.  grid: a few dozen workgroups that share the (unit, page, keys | values) items.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void k_fetch(DeviceView dv, int u0, int n_units, int max_moves) {
    // items = (unit, move, keys | values), dealt round-robin to a SMALL fixed number of workgroups: the link
    // needs ~150 KB in flight, and workgroups parked on PCIe loads would otherwise hold the wave slots and
    // registers that the attention and selection kernels of the neighbouring layers are waiting for
    const int n_items = n_units * max_moves * 2;
    for (int it = blockIdx.x; it < n_items; it += gridDim.x) {
        const int val = it & 1, i = (it >> 1) % max_moves, u = u0 + (it >> 1) / max_moves;
        if (i >= dv.n_moves[u]) continue;                                   // block-uniform
        const int hp = dv.moves[((size_t)u * dv.F + i) * 2], cp = dv.moves[((size_t)u * dv.F + i) * 2 + 1];
        const size_t bytes = val ? dv.vpage : dv.kpage;
        const char *src = (val ? dv.host_v : dv.host_k) + (size_t)u * dv.h_ustride +
                          (size_t)(hp / dv.SFh) * dv.h_bstride + (size_t)(hp % dv.SFh) * bytes;
        char *dst = (val ? dv.v_store + (size_t)u * dv.v_ustride : dv.k_store + (size_t)u * dv.k_ustride) + (size_t)cp * bytes;
        const uint4 *s4 = reinterpret_cast<const uint4 *>(src);
        uint4 *d4 = reinterpret_cast<uint4 *>(dst);
        const size_t n16 = bytes / 16;
        for (size_t j = threadIdx.x; j < n16; j += 4 * kBlock) {           // four 16-byte loads in flight per thread
            uint4 x[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) x[q] = s4[min(j + (size_t)q * kBlock, n16 - 1)];
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (j + (size_t)q * kBlock < n16) d4[j + (size_t)q * kBlock] = x[q];
        }
    }
}

template <typename F> hipError_t checked(F &&launch) {
    launch();
    return hipGetLastError();
}

} // namespace

hipError_t launch_store_summary(const DeviceView &dv, const void *k_in, const void *v_in, int f0,
                                int n_frames, hipStream_t s) {
    dim3 grid(dv.U, n_frames, 2);
    return checked([&] {
        if (dv.esize == 4) {
            if (dv.D == 64) k_store_summary<float, 64><<<grid, kBlock, 0, s>>>(dv, (const float *)k_in, (const float *)v_in, f0);
            else k_store_summary<float, 128><<<grid, kBlock, 0, s>>>(dv, (const float *)k_in, (const float *)v_in, f0);
        } else {
            if (dv.D == 64) k_store_summary<unsigned short, 64><<<grid, kBlock, 0, s>>>(dv, (const unsigned short *)k_in, (const unsigned short *)v_in, f0);
            else k_store_summary<unsigned short, 128><<<grid, kBlock, 0, s>>>(dv, (const unsigned short *)k_in, (const unsigned short *)v_in, f0);
        }
    });
}

hipError_t launch_ingest_one(const DeviceView &dv, const void *k_in, const void *v_in, int f, hipStream_t s) {
    dim3 grid(dv.U, 2);
    return checked([&] {
        if (dv.esize == 4) {
            if (dv.D == 64) k_ingest_one<float, 64><<<grid, kBlock, 0, s>>>(dv, (const float *)k_in, (const float *)v_in, f);
            else k_ingest_one<float, 128><<<grid, kBlock, 0, s>>>(dv, (const float *)k_in, (const float *)v_in, f);
        } else {
            if (dv.D == 64) k_ingest_one<unsigned short, 64><<<grid, kBlock, 0, s>>>(dv, (const unsigned short *)k_in, (const unsigned short *)v_in, f);
            else k_ingest_one<unsigned short, 128><<<grid, kBlock, 0, s>>>(dv, (const unsigned short *)k_in, (const unsigned short *)v_in, f);
        }
    });
}

hipError_t launch_value_reps(const DeviceView &dv, int n_frames, hipStream_t s) {
    const dim3 grid(dv.U, dv.C);
    return checked([&] {
        if (dv.D == 64) k_value_reps<64><<<grid, 128, 0, s>>>(dv, n_frames);
        else k_value_reps<128><<<grid, 128, 0, s>>>(dv, n_frames);
    });
}

hipError_t launch_offload(const DeviceView &dv, int f0, int n, hipStream_t s) {
    const long long items = (long long)dv.U * n * 2;
    // 16 workgroups (posted stores keep the link full; config 3 ingest with 4 / 8 / 16 / 64 / 256 / 1024 workgroups:
    // 12.5 / 13.9 / 14.0 / 13.2 / 12.7 / 12.6 k frames/s -- the more of them, the more they slow the staging and
    // assignment kernels that run beside them)
    const int blocks = (int)std::min<long long>(items, 16);
    return checked([&] { k_offload<<<blocks, kBlock, 0, s>>>(dv, f0, n); });
}

hipError_t launch_fetch(const DeviceView &dv, int u0, int n_units, int max_moves, hipStream_t s) {
    if (max_moves <= 0) return hipSuccess;
    // 64 workgroups (measured on config 3: 16 / 32 / 64 / 96 / 128 / 256 / one per page and operand give a warm
    // decode step of 6.15 / 6.19 / 6.01 / 6.28 / 6.25 / 6.53 / 6.71 ms and 53.4 .. 55.2 GB/s over the link)
    const long long items = (long long)n_units * max_moves * 2;
    const int blocks = (int)std::min<long long>(items, 64);
    return checked([&] { k_fetch<<<blocks, kBlock, 0, s>>>(dv, u0, n_units, max_moves); });
}

hipError_t launch_assign_update(const DeviceView &dv, int f0, int f1, hipStream_t s) {
    return checked([&] {
        if (dv.maint_mode) {
            if (dv.D == 64) k_assign_update<64, true><<<dv.U, kBlock, 0, s>>>(dv, f0, f1);
            else k_assign_update<128, true><<<dv.U, kBlock, 0, s>>>(dv, f0, f1);
        } else if (dv.C <= 128) {          // table in registers: 8 rows per 16-lane group
            if (dv.D == 64) k_assign_update_reg<64, 256><<<dv.U, 256, 0, s>>>(dv, f0, f1);
            else k_assign_update_reg<128, 256><<<dv.U, 256, 0, s>>>(dv, f0, f1);
        } else if (dv.C <= 256) {
            if (dv.D == 64) k_assign_update_reg<64, 512><<<dv.U, 512, 0, s>>>(dv, f0, f1);
            else k_assign_update_reg<128, 512><<<dv.U, 512, 0, s>>>(dv, f0, f1);
        } else {
            if (dv.D == 64) k_assign_update<64, false><<<dv.U, kBlock, 0, s>>>(dv, f0, f1);
            else k_assign_update<128, false><<<dv.U, kBlock, 0, s>>>(dv, f0, f1);
        }
    });
}

hipError_t launch_lloyd(const DeviceView &dv, int n_frames, int iters, bool seed_from_warmup,
                        hipStream_t s) {
    hipError_t e = hipSuccess;
    if (seed_from_warmup) {
        e = checked([&] {
            if (dv.P > 0) {
                if (dv.D == 64) k_lloyd_seed_nested<64><<<dv.U, kBlock, 0, s>>>(dv, n_frames);
                else k_lloyd_seed_nested<128><<<dv.U, kBlock, 0, s>>>(dv, n_frames);
            } else {
                if (dv.D == 64) k_lloyd_seed<64><<<dv.U, kBlock, 0, s>>>(dv, n_frames);
                else k_lloyd_seed<128><<<dv.U, kBlock, 0, s>>>(dv, n_frames);
            }
        });
        if (e != hipSuccess) return e;
    }
    dim3 ga(dv.U, (n_frames + 63) / 64), gu(dv.U, dv.C);
    // the rounds' moved-frame counters, live-row counters and, behind them, the clusters' changed flags
    if ((e = hipMemsetAsync(dv.lloyd_moved, 0, ((size_t)dv.U * 6 + (size_t)dv.U * dv.C) * 4, s)) != hipSuccess) return e;
    for (int it = 0; it < iters; ++it) {
        if (it > 0) {
            e = checked([&] { k_lloyd_bounds<<<dim3(dv.U, (n_frames + 1023) / 1024), kBlock, 0, s>>>(dv, n_frames, it); });
            if (e != hipSuccess) return e;
        }
        // (later rounds: a workgroup per task of four live rows, the rest of the grid exits at once; fewer
        // workgroups that take tasks in turn were slower, 80 against 59 us per round: a unit whose rows mostly
        // stay alive then keeps its few workgroups busy for several tasks)
        const dim3 gi = ga;
        e = checked([&] {
            if (it == 0) {
                if (dv.D == 64) k_lloyd_assign<64, false><<<gi, kBlock, 0, s>>>(dv, n_frames, it);
                else k_lloyd_assign<128, false><<<gi, kBlock, 0, s>>>(dv, n_frames, it);
            } else {
                if (dv.D == 64) k_lloyd_assign<64, true><<<gi, kBlock, 0, s>>>(dv, n_frames, it);
                else k_lloyd_assign<128, true><<<gi, kBlock, 0, s>>>(dv, n_frames, it);
            }
        });
        if (e != hipSuccess) return e;
        e = checked([&] {
            if (dv.D == 64) k_lloyd_update<64><<<gu, 128, 0, s>>>(dv, n_frames, it);
            else k_lloyd_update<128><<<gu, 128, 0, s>>>(dv, n_frames, it);
        });
        if (e != hipSuccess) return e;
    }
    if (dv.maint_mode) {
        const dim3 gv(dv.U, dv.c_init);
        e = checked([&] {
            if (dv.D == 64) k_exact_var<64><<<gv, kBlock, 0, s>>>(dv, n_frames);
            else k_exact_var<128><<<gv, kBlock, 0, s>>>(dv, n_frames);
        });
    }
    return e;
}

hipError_t launch_partition_reps(const DeviceView &dv, int n_frames, hipStream_t s) {
    const dim3 g(dv.U, dv.P);
    return checked([&] {
        if (dv.D == 64) k_partition_reps<64><<<g, 128, 0, s>>>(dv, n_frames);
        else k_partition_reps<128><<<g, 128, 0, s>>>(dv, n_frames);
    });
}

} // namespace mosaic
