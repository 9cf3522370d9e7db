// Retrieval augmentation, global representatives (paper Sec. V-C), device side: the
// attention partial of one row tile over a unit's clusters as pseudo tokens.  The
// attention kernels run it in extra workgroups of their own launch (the part depends on
// the query and the clustering only), so it costs no kernel boundary of its own.
#pragma once
#include "mosaic_internal.h"

namespace mosaic {

template <typename E> __device__ __forceinline__ float rp_to_f32(E v);
template <> __device__ __forceinline__ float rp_to_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ float rp_to_f32<unsigned short>(unsigned short v) { return bf16_to_f32(v); }

// Retrieval augmentation, global representatives (paper Sec. V-C): attention of one
// row tile over the unit's non-empty clusters as pseudo tokens (key = representative,
// value = mean of the members' values), written as one more partial (running maximum in
// the log2 domain, sum, unnormalised output) that the combine kernel merges with the
// split partials.  One workgroup of 256 threads per (row tile, unit).  Keys and values
// come from the fp32 tables rep_k / rep_v [C][D] (built whenever the clustering changed).
// Clusters are taken 256 at a time: logits with one thread per (cluster, four rows),
// each streaming its key row with independent 16-byte loads; row statistics with one
// 16-lane group per query row; then the weighted value sum with one thread per
// (channel, half of the rows); blocks of clusters are chained by a running maximum.
template <typename E, int D>
__device__ void attend_reps_partial(const DeviceView &dv, int u0, int uc, int tile, const E *q, int Tq) {
    constexpr int CB = 256, HALF = kBlock / D, RPT = kRowTile / HALF;   // rows per thread in phase 3
    const int u = u0 + uc, tid = threadIdx.x;
    const int lr = tid % 16, grp = tid / 16;
    const int G = dv.G, Hq = dv.Hq, C = dv.C, lc = uc / dv.Hkv, h = u % dv.Hkv, R = Tq * G;
    __shared__ float q_sh[kRowTile][D];
    __shared__ float w_sh[kRowTile][CB];       // logits, then weights
    __shared__ float m_sh[kRowTile], l_sh[kRowTile], a_sh[kRowTile];
    for (int i = tid; i < kRowTile * D; i += kBlock) {
        const int row = i / D, d = i % D, gr = tile * kRowTile + row;
        float v = 0.f;
        if (gr < R) {
            const int t = gr / G, g = gr % G;
            v = rp_to_f32<E>(q[(((size_t)lc * Tq + t) * Hq + (size_t)h * G + g) * D + d]);
        }
        q_sh[row][d] = v;
    }
    if (tid < kRowTile) { m_sh[tid] = -INFINITY; l_sh[tid] = 0.f; }
    const float sl2 = 1.4426950408889634f / sqrtf((float)D);
    const float *rk = dv.rep_k + (size_t)u * C * D;
    const float *rv = dv.rep_v + (size_t)u * C * D;
    const int *n = dv.n + (size_t)u * C;
    const int d3 = tid % D, half = tid / D;
    const int n_rq = (min(kRowTile, max(R - tile * kRowTile, 0)) + 3) / 4;
    float o[RPT];
#pragma unroll
    for (int i = 0; i < RPT; ++i) o[i] = 0.f;
    __syncthreads();
    for (int c0 = 0; c0 < C; c0 += CB) {
        const int cn = min(CB, C - c0);
        // ---- logits: item = (cluster jj, row quad rq), rows 4*rq .. 4*rq+3; only the row quads
        //      that hold query rows, clusters up to the next multiple of 16 (the rest get -inf) ----
        const int cnp = min(CB, (cn + 15) / 16 * 16);
        for (int item = tid; item < cnp * n_rq; item += kBlock) {
            const int jj = item % cnp, rq = item / cnp;
            float acc[4] = {0.f, 0.f, 0.f, 0.f};
            const bool live = jj < cn && n[c0 + jj] > 0;
            const float4 *kr = reinterpret_cast<const float4 *>(rk + (size_t)(c0 + min(jj, cn - 1)) * D);
#pragma unroll 16
            for (int d4 = 0; d4 < D / 4; ++d4) {
                const float4 kv = kr[d4];
#pragma unroll
                for (int x = 0; x < 4; ++x) {
                    const float *qr = &q_sh[4 * rq + x][4 * d4];
                    acc[x] += qr[0] * kv.x + qr[1] * kv.y + qr[2] * kv.z + qr[3] * kv.w;
                }
            }
#pragma unroll
            for (int x = 0; x < 4; ++x) w_sh[4 * rq + x][jj] = live ? acc[x] * sl2 : -INFINITY;
        }
        __syncthreads();
        // ---- row statistics: group `grp` owns row `grp` (rows without a query keep weight 0) ----
        {
            const int row = grp;
            const bool has_q = row < 4 * n_rq;
            float mx = -INFINITY;
            if (has_q)
                for (int jj = lr; jj < cnp; jj += 16) mx = fmaxf(mx, w_sh[row][jj]);
#pragma unroll
            for (int x = 8; x >= 1; x >>= 1) mx = fmaxf(mx, __shfl_xor(mx, x, 16));
            const float mo = m_sh[row], mn = fmaxf(mo, mx);
            float sum = 0.f;
            for (int jj = lr; jj < cnp; jj += 16) {
                const float s = has_q ? w_sh[row][jj] : -INFINITY;
                const float w = s > -INFINITY ? exp2f(s - mn) : 0.f;
                w_sh[row][jj] = w;
                sum += w;
            }
#pragma unroll
            for (int x = 8; x >= 1; x >>= 1) sum += __shfl_xor(sum, x, 16);
            if (lr == 0) {
                const float alpha = mo > -INFINITY ? exp2f(mo - mn) : 0.f;
                a_sh[row] = alpha;
                l_sh[row] = l_sh[row] * alpha + sum;
                m_sh[row] = mn;
            }
        }
        __syncthreads();
        // ---- weighted sum of the value representatives (weights beyond cn are 0) ----
#pragma unroll
        for (int i = 0; i < RPT; ++i) o[i] *= a_sh[half * RPT + i];
        for (int jj0 = 0; jj0 < cnp; jj0 += 32) {       // cnp is a multiple of 16: 16 or 32 per pass
            float vv[32];
#pragma unroll
            for (int x = 0; x < 32; ++x) vv[x] = rv[(size_t)(c0 + min(jj0 + x, cn - 1)) * D + d3];
#pragma unroll
            for (int x = 0; x < 32; ++x) {
                const int jj = min(jj0 + x, cnp - 1);
                const float wz = jj0 + x < cnp ? 1.f : 0.f;
#pragma unroll
                for (int i = 0; i < RPT; ++i) o[i] += wz * w_sh[half * RPT + i][jj] * vv[x];
            }
        }
        __syncthreads();
    }
    const size_t entry = (size_t)u * dv.nt_max + tile;
#pragma unroll
    for (int i = 0; i < RPT; ++i) dv.aug_o[(entry * kRowTile + half * RPT + i) * D + d3] = o[i];
    if (tid < kRowTile) {
        dv.aug_ml[entry * 2 * kRowTile + tid] = m_sh[tid];
        dv.aug_ml[entry * 2 * kRowTile + kRowTile + tid] = l_sh[tid];
    }
}

} // namespace mosaic
