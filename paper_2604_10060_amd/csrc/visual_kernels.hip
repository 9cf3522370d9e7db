// Visual level of the nested visual-semantic hierarchy (paper Sec. V-B (1)):
// the per-frame visual embeddings are clustered once per stream, with the same
// modified K-means as the key summaries (cosine criterion, representative =
// mean of the members, Eq. 1 / Eq. 3), into P partitions that every unit's
// semantic clustering is then confined to.
//   k_visual_store   warm-up embeddings (fp32) -> the visual level's fp64 state array
//   k_visual_seed / k_visual_lloyd_assign / _update   initial P-means over the warm-up embeddings
//   k_visual_assign  greedy assignment + running-mean update, frame by frame
// One stream has one visual level and P <= 64: the online kernel is a single wide
// workgroup (frames are strictly sequential), the K-means rounds spread frames and
// centroids over workgroups; a wavefront computes a (frame, centroid) cosine with
// its lanes striding the Dv channels.
#include "mosaic_internal.h"

namespace mosaic {

namespace {

constexpr int kVisBlock = 1024, kVisWaves = kVisBlock / 64;

// (every call site has the whole wavefront active)
__device__ __forceinline__ double wave_sum(double x) { return wave64_sum(x); }
__device__ __forceinline__ bool better(double v, int i, double bv, int bi) {
    return v > bv || (v == bv && i < bi);
}

// grid (n_frames), 256 threads
__global__ __launch_bounds__(256) void k_visual_store(DeviceView dv, const float *e_in, int f0) {
    const int i = blockIdx.x;
    const float *src = e_in + (size_t)i * dv.Dv;
    double *dst = dv.vemb + (size_t)(f0 + i) * dv.Dv;
    for (int d = threadIdx.x; d < dv.Dv; d += 256) dst[d] = (double)src[d];
}

// Sum of one value per thread over the workgroup, in a fixed order.  Every thread
// gets the result.  red: kVisWaves doubles of LDS.
__device__ __forceinline__ double block_sum(double x, double *red) {
    const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
    x = wave_sum(x);
    __syncthreads();                 // the previous use of red is over
    if (lane == 0) red[wave] = x;
    __syncthreads();
    double t = 0.0;
#pragma unroll
    for (int w = 0; w < kVisWaves; ++w) t += red[w];
    return t;
}

// The non-empty centroid most similar (cosine) to embedding e, ties to the lowest
// id; `live_all` treats every centroid as non-empty.  Called by one wavefront.
__device__ __forceinline__ int visual_nearest(const DeviceView &dv, const double *e, bool live_all) {
    const int lane = threadIdx.x % 64, Dv = dv.Dv;
    double en = 0.0;
    for (int d = lane; d < Dv; d += 64) en += e[d] * e[d];
    en = sqrt(wave_sum(en));
    double bv = -INFINITY;
    int bi = 0x7fffffff;
    for (int p = 0; p < dv.P; ++p) {
        if (!live_all && dv.vn[p] <= 0) continue;        // wave-uniform
        const double *rp = dv.vr + (size_t)p * Dv;
        double x = 0.0;
        for (int d = lane; d < Dv; d += 64) x += e[d] * rp[d];
        x = wave_sum(x);
        const double rn = dv.vrn[p];
        const double c = (en == 0.0 || rn == 0.0) ? 0.0 : x / (en * rn);
        if (better(c, p, bv, bi)) { bv = c; bi = p; }
    }
    return bi == 0x7fffffff ? 0 : bi;
}

// Initial clustering of the visual level over the first W embeddings: seeds =
// embeddings of frames floor(p*W/P), every centroid live in the first
// assignment round, `iters` rounds; a centroid left without members keeps its
// vector and is skipped afterwards.  Three small kernels per round trip of the
// algorithm, launched back to back on the stream:
//   k_visual_seed          grid (P): copy the seed embedding, its norm
//   k_visual_lloyd_assign  grid (ceil(W/16)): one wavefront per frame
//   k_visual_lloyd_update  grid (P): members summed in ascending frame order
__global__ __launch_bounds__(kVisBlock) void k_visual_seed(DeviceView dv, int W) {
    const int tid = threadIdx.x, p = blockIdx.x, Dv = dv.Dv;
    __shared__ double red[kVisWaves];
    const double *src = dv.vemb + (size_t)(((long long)p * W) / dv.P) * Dv;
    double sq = 0.0;
    for (int d = tid; d < Dv; d += kVisBlock) { const double v = src[d]; dv.vr[(size_t)p * Dv + d] = v; sq += v * v; }
    sq = block_sum(sq, red);
    if (tid == 0) { dv.vrn[p] = sqrt(sq); dv.vn[p] = 0; }
}

__global__ __launch_bounds__(kVisBlock) void k_visual_lloyd_assign(DeviceView dv, int W, int live_all) {
    const int f = blockIdx.x * kVisWaves + threadIdx.x / 64;
    if (f >= W) return;                                  // wave-uniform; no barrier in this kernel
    const int a = visual_nearest(dv, dv.vemb + (size_t)f * dv.Dv, live_all != 0);
    if (threadIdx.x % 64 == 0) dv.part[f] = a;
}

__global__ __launch_bounds__(kVisBlock) void k_visual_lloyd_update(DeviceView dv, int W) {
    const int tid = threadIdx.x, p = blockIdx.x, Dv = dv.Dv;
    constexpr int kPartLds = 8192;            // the assignments are scanned out of LDS when they fit
    __shared__ double red[kVisWaves];
    __shared__ int part_sh[kPartLds];
    const bool in_lds = W <= kPartLds;
    if (in_lds)
        for (int f = tid; f < W; f += kVisBlock) part_sh[f] = dv.part[f];
    __syncthreads();
    const int *part = in_lds ? part_sh : dv.part;
    int count = 0;
    for (int f = 0; f < W; ++f) count += part[f] == p;
    if (count == 0) {                                    // workgroup-uniform
        if (tid == 0) dv.vn[p] = 0;
        return;
    }
    double sq = 0.0;
    for (int d = tid; d < Dv; d += kVisBlock) {
        double acc = 0.0;
        for (int f = 0; f < W; ++f)
            if (part[f] == p) acc += dv.vemb[(size_t)f * Dv + d];
        const double rv = acc / (double)count;
        dv.vr[(size_t)p * Dv + d] = rv;
        sq += rv * rv;
    }
    sq = block_sum(sq, red);
    if (tid == 0) { dv.vrn[p] = sqrt(sq); dv.vn[p] = count; }
}

// Frames f0..f1-1, in order: partition = most similar non-empty visual centroid,
// which then moves by Eq. 3.  grid (1), kVisBlock threads.  e_in: the fp32
// embeddings of these frames as the caller passed them; the kernel also files
// them in the visual level's state array.  Per frame: the embedding is staged in
// LDS, wavefront w scores centroids w, w+16, ..., thread 0 picks the winner, all
// threads update its row.
__global__ __launch_bounds__(kVisBlock) void k_visual_assign(DeviceView dv, const float *e_in, int f0, int f1) {
    const int tid = threadIdx.x, wave = tid / 64, lane = tid % 64, Dv = dv.Dv, P = dv.P;
    __shared__ double e_sh[4096];
    __shared__ double red[kVisWaves];
    __shared__ double bv_sh[kVisWaves];
    __shared__ int bi_sh[kVisWaves];
    __shared__ int win_sh;
    for (int f = f0; f < f1; ++f) {
        const float *src = e_in + (size_t)(f - f0) * Dv;
        for (int d = tid; d < Dv; d += kVisBlock) {
            const double v = (double)src[d];
            e_sh[d] = v;
            dv.vemb[(size_t)f * Dv + d] = v;
        }
        __syncthreads();
        double en = 0.0;
        for (int d = lane; d < Dv; d += 64) en += e_sh[d] * e_sh[d];
        en = sqrt(wave_sum(en));
        double bv = -INFINITY;
        int bi = 0x7fffffff;
        for (int p = wave; p < P; p += kVisWaves) {
            if (dv.vn[p] <= 0) continue;                 // wave-uniform
            const double *rp = dv.vr + (size_t)p * Dv;
            double x = 0.0;
            for (int d = lane; d < Dv; d += 64) x += e_sh[d] * rp[d];
            x = wave_sum(x);
            const double rn = dv.vrn[p];
            const double c = (en == 0.0 || rn == 0.0) ? 0.0 : x / (en * rn);
            if (better(c, p, bv, bi)) { bv = c; bi = p; }
        }
        if (lane == 0) { bv_sh[wave] = bv; bi_sh[wave] = bi; }
        __syncthreads();
        if (tid == 0) {
            for (int w = 1; w < kVisWaves; ++w)
                if (better(bv_sh[w], bi_sh[w], bv, bi)) { bv = bv_sh[w]; bi = bi_sh[w]; }
            const int a = bi == 0x7fffffff ? 0 : bi;
            win_sh = a;
            dv.part[f] = a;
        }
        __syncthreads();
        const int a = win_sh;
        const double na = (double)dv.vn[a];
        double sq = 0.0;
        for (int d = tid; d < Dv; d += kVisBlock) {
            // Eq. 3, each operation rounded separately
            const double rv = __ddiv_rn(__dadd_rn(__dmul_rn(na, dv.vr[(size_t)a * Dv + d]), e_sh[d]), na + 1.0);
            dv.vr[(size_t)a * Dv + d] = rv;
            sq += rv * rv;
        }
        sq = block_sum(sq, red);     // (its barriers also order the reads of vn[a] before the update)
        if (tid == 0) { dv.vrn[a] = sqrt(sq); dv.vn[a] = (int)na + 1; }
        __syncthreads();
    }
}

hipError_t after_launch() {
    return hipGetLastError();
}

} // namespace

hipError_t launch_visual_store(const DeviceView &dv, const float *e_in, int f0, int n_frames, hipStream_t s) {
    k_visual_store<<<n_frames, 256, 0, s>>>(dv, e_in, f0);
    return after_launch();
}

hipError_t launch_visual_lloyd(const DeviceView &dv, int W, int iters, hipStream_t s) {
    k_visual_seed<<<dv.P, kVisBlock, 0, s>>>(dv, W);
    hipError_t e = after_launch();
    for (int it = 0; it < iters && e == hipSuccess; ++it) {
        k_visual_lloyd_assign<<<(W + kVisWaves - 1) / kVisWaves, kVisBlock, 0, s>>>(dv, W, it == 0);
        if ((e = after_launch()) != hipSuccess) break;
        k_visual_lloyd_update<<<dv.P, kVisBlock, 0, s>>>(dv, W);
        e = after_launch();
    }
    return e;
}

hipError_t launch_visual_assign(const DeviceView &dv, const float *e_in, int f0, int f1, hipStream_t s) {
    k_visual_assign<<<1, kVisBlock, 0, s>>>(dv, e_in, f0, f1);
    return after_launch();
}

} // namespace mosaic
