// Query Retrieval, selection part (paper Sec. V-C; top-K of Sec. VII-B):
// one workgroup per unit computes the mean query, scores every representative
// of the GPU-resident index, ranks them, and lists the pages of the chosen
// clusters.  Nothing is copied: attention later reads the pages in place.
#include "mosaic_internal.h"

namespace mosaic {

namespace {

__device__ __forceinline__ double group16_sum(double x) {
#pragma unroll
    for (int o = 8; o >= 1; o >>= 1) x += __shfl_xor(x, o, 16);
    return x;
}

template <typename E> __device__ __forceinline__ double to_f64(E v);
template <> __device__ __forceinline__ double to_f64<float>(float v) { return (double)v; }
template <> __device__ __forceinline__ double to_f64<unsigned short>(unsigned short v) {
    return (double)bf16_to_f32(v);
}

// grid (n_units), 256 threads.  u0 is a multiple of Hkv.
template <typename E, int D>
__global__ __launch_bounds__(kBlock) void k_retrieve(DeviceView dv, int u0, const E *q, int Tq,
                                                     int n_frames, int score_mode) {
    constexpr int EPL = D / 16;
    const int uc = blockIdx.x, u = u0 + uc, tid = threadIdx.x;
    const int C = dv.C, G = dv.G, Hq = dv.Hq, k = dv.k;
    const int lc = uc / dv.Hkv, h = u % dv.Hkv;
    const int lr = tid % 16, row0 = tid / 16;
    __shared__ double qbar[D];
    __shared__ double sc_sh[1024];
    __shared__ int rank_sh[1024];   // selection rank of cluster j, or -1
    __shared__ int ids_sh[1024];
    __shared__ int off_sh[1025];
    __shared__ int n_live_sh;
    const double *r = dv.r + (size_t)u * C * D;
    const double *rn = dv.rnorm + (size_t)u * C;
    const int *n = dv.n + (size_t)u * C;

    if (tid == 0) n_live_sh = 0;
    // mean query over the Tq tokens and the G query heads of this KV head
    if (tid < D) {
        const E *qb = q + (size_t)lc * Tq * Hq * D;
        double acc = 0.0;
        for (int t = 0; t < Tq; ++t)
            for (int g = 0; g < G; ++g)
                acc += to_f64<E>(qb[((size_t)t * Hq + (size_t)h * G + g) * D + tid]);
        qbar[tid] = acc / (double)(Tq * G);
    }
    __syncthreads();
    // score_j = (qbar . r_j) / |r_j|   (plain dot product in score_mode 1)
    for (int j = row0; j < C; j += 16) {
        double p = 0.0;
        const bool live = n[j] > 0;
        if (live) {
            const double *rj = r + (size_t)j * D + lr * EPL;
#pragma unroll
            for (int i = 0; i < EPL; ++i) p += qbar[lr * EPL + i] * rj[i];
        }
        p = group16_sum(p);
        if (lr == 0) {
            double sc = -INFINITY;
            if (live) sc = score_mode == 1 ? p : (rn[j] == 0.0 ? 0.0 : p / rn[j]);
            sc_sh[j] = sc;
            dv.scores[(size_t)u * C + j] = sc;
        }
    }
    __syncthreads();
    // rank among non-empty clusters by (score descending, id ascending)
    for (int j = tid; j < C; j += kBlock) {
        int rk = -1;
        if (n[j] > 0) {
            const double sj = sc_sh[j];
            rk = 0;
            for (int i = 0; i < C; ++i) {
                const double si = sc_sh[i];
                rk += (n[i] > 0) && (si > sj || (si == sj && i < j));
            }
            atomicAdd(&n_live_sh, 1);
            if (rk < k) ids_sh[rk] = j; else rk = -1;
        }
        rank_sh[j] = rk;
    }
    __syncthreads();
    const int n_ids = min(k, n_live_sh);
    if (tid == 0) {
        int o = 0;
        off_sh[0] = 0;
        for (int i = 0; i < n_ids; ++i) { o += n[ids_sh[i]]; off_sh[i + 1] = o; }
        dv.n_ids[u] = n_ids;
        dv.n_sel[u] = o;
    }
    for (int i = tid; i < k; i += kBlock) dv.ids[(size_t)u * k + i] = i < n_ids ? ids_sh[i] : -1;
    __syncthreads();
    // page list: clusters in selection order, member frames ascending
    const int *assign = dv.assign + (size_t)u * dv.F;
    const int *pos = dv.pos + (size_t)u * dv.F;
    int *sel = dv.sel_pages + (size_t)u * dv.F;
    for (int f = tid; f < n_frames; f += kBlock) {
        const int c = assign[f];
        if (c < 0) continue;
        const int rk = rank_sh[c];
        if (rk >= 0) sel[off_sh[rk] + pos[f]] = f;
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

hipError_t launch_retrieve(const DeviceView &dv, int u0, int n_units, const void *q, int Tq,
                           int n_frames, int score_mode, hipStream_t s) {
    if (dv.esize == 4) {
        if (dv.D == 64) k_retrieve<float, 64><<<n_units, kBlock, 0, s>>>(dv, u0, (const float *)q, Tq, n_frames, score_mode);
        else k_retrieve<float, 128><<<n_units, kBlock, 0, s>>>(dv, u0, (const float *)q, Tq, n_frames, score_mode);
    } else {
        if (dv.D == 64) k_retrieve<unsigned short, 64><<<n_units, kBlock, 0, s>>>(dv, u0, (const unsigned short *)q, Tq, n_frames, score_mode);
        else k_retrieve<unsigned short, 128><<<n_units, kBlock, 0, s>>>(dv, u0, (const unsigned short *)q, Tq, n_frames, score_mode);
    }
    return hipGetLastError();
}

hipError_t launch_expand_tok_idx(const DeviceView &dv, int u0, int n_units, hipStream_t s) {
    k_expand_tok_idx<<<n_units, kBlock, 0, s>>>(dv, u0);
    return hipGetLastError();
}

} // namespace mosaic
