// Attention over the retrieved KV (paper Sec. V-A (2)): vector-ALU split-KV
// kernel (fp32 or bf16 pages, values stored [T][D]) and the combine kernel that
// merges the per-split partials of either kernel family.
//
// Work decomposition shared by both families:
//   rows     the unit's G*Tq query rows, row r = t*G + g, in tiles of 16
//   chunks   32 tokens inside one page; a unit has n_sel * ceil(T/32) chunks
//   splits   contiguous chunk ranges; one workgroup per (split, row tile, unit)
// Each workgroup keeps an online softmax in the log2 domain (logits are
// multiplied by log2(e)/sqrt(D) once) and writes (max, sum, unnormalised O).
#include "mosaic_internal.h"
#include "attend_reps_device.h"

namespace mosaic {

namespace {

template <typename E> __device__ __forceinline__ float to_f32(E v);
template <> __device__ __forceinline__ float to_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f32<unsigned short>(unsigned short v) {
    return bf16_to_f32(v);
}
template <typename E> __device__ __forceinline__ void load8f(const E *p, float (&v)[8]);
template <> __device__ __forceinline__ void load8f<float>(const float *p, float (&v)[8]) {
    const float4 a = *reinterpret_cast<const float4 *>(p);
    const float4 b = *reinterpret_cast<const float4 *>(p + 4);
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
    v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}
template <> __device__ __forceinline__ void load8f<unsigned short>(const unsigned short *p,
                                                                   float (&v)[8]) {
    const uint4 a = *reinterpret_cast<const uint4 *>(p);
    const unsigned int w[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        v[2 * i] = __uint_as_float(w[i] << 16);
        v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
}
template <typename E> __device__ __forceinline__ void store_out(E *p, float v);
template <> __device__ __forceinline__ void store_out<float>(float *p, float v) { *p = v; }
template <> __device__ __forceinline__ void store_out<unsigned short>(unsigned short *p, float v) {
    *p = f32_to_bf16_rne(v);
}

__device__ __forceinline__ float group16_max(float x) {
#pragma unroll
    for (int o = 8; o >= 1; o >>= 1) x = fmaxf(x, __shfl_xor(x, o, 16));
    return x;
}
__device__ __forceinline__ float group16_sumf(float x) {
#pragma unroll
    for (int o = 8; o >= 1; o >>= 1) x += __shfl_xor(x, o, 16);
    return x;
}

// grid (n_units * n_splits [+ n_units with the global-representative augmentation], NT), 256 threads:
// thread (row = tid/16, tl = tid%16)
template <typename E, int D>
__global__ __launch_bounds__(kBlock) void k_attend_valu(DeviceView dv, int u0, int n_units, const E *q,
                                                        int Tq, int B) {
    constexpr int DPT = D / 16;   // output channels per thread
    constexpr int CG = D / 8;     // 8-element groups per token row
    if ((int)blockIdx.x >= B) {   // extra columns: the global representatives' part (augmentation)
        attend_reps_partial<E, D>(dv, u0, (int)blockIdx.x - B, blockIdx.y, q, Tq);
        return;
    }
    const SplitSlot slot = split_slot<false>(dv.n_sel + u0, n_units, B, blockIdx.x);
    if (slot.uc < 0) return;      // block-uniform: no barrier reached yet
    const int split = slot.split, n_splits = slot.S, tile = blockIdx.y, uc = slot.uc, u = u0 + uc;
    const int NT = gridDim.y, tid = threadIdx.x, row = tid / 16, tl = tid % 16;
    const int G = dv.G, Hq = dv.Hq, T = dv.T;
    const int lc = uc / dv.Hkv, h = u % dv.Hkv, R = Tq * G;
    __shared__ float q_sh[kRowTile][D];
    __shared__ float k_sh[kChunk][D + 1];
    __shared__ float v_sh[kChunk][D];
    __shared__ float p_sh[kRowTile][kChunk];

    const float sl2 = 1.4426950408889634f / sqrtf((float)D);
    for (int idx = tid; idx < kRowTile * D; idx += kBlock) {
        const int rr = idx / D, d = idx % D, gr = tile * kRowTile + rr;
        float v = 0.f;
        if (gr < R) {
            const int t = gr / G, g = gr % G;
            v = to_f32<E>(q[(((size_t)lc * Tq + t) * Hq + (size_t)h * G + g) * D + d]) * sl2;
        }
        q_sh[rr][d] = v;
    }
    const int cpp = dv.chunks_per_page;
    const int NC = dv.n_sel[u] * cpp;
    const int cps = (NC + n_splits - 1) / n_splits;
    const int c0 = split * cps, c1 = min(NC, c0 + cps);
    const int *sel = dv.sel_pages + (size_t)u * dv.F;

    float m = -INFINITY, l = 0.f, acc[DPT];
#pragma unroll
    for (int i = 0; i < DPT; ++i) acc[i] = 0.f;
    __syncthreads();

    for (int c = c0; c < c1; ++c) {
        const int page = sel[c / cpp], t0 = (c % cpp) * kChunk, nt = min(kChunk, T - t0);
        const E *kp = reinterpret_cast<const E *>(k_page(dv, u, page)) + (size_t)t0 * D;
        const E *vp = reinterpret_cast<const E *>(v_page(dv, u, page)) + (size_t)t0 * D;
        for (int item = tid; item < kChunk * CG; item += kBlock) {
            const int tok = item / CG, cg = item % CG;
            float kv[8], vv[8];
            if (tok < nt) {
                load8f<E>(kp + (size_t)tok * D + cg * 8, kv);
                load8f<E>(vp + (size_t)tok * D + cg * 8, vv);
            } else {
#pragma unroll
                for (int i = 0; i < 8; ++i) { kv[i] = 0.f; vv[i] = 0.f; }
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) { k_sh[tok][cg * 8 + i] = kv[i]; v_sh[tok][cg * 8 + i] = vv[i]; }
        }
        __syncthreads();
        float s0 = 0.f, s1 = 0.f;
        for (int d = 0; d < D; ++d) {
            const float qv = q_sh[row][d];
            s0 += qv * k_sh[tl][d];
            s1 += qv * k_sh[tl + 16][d];
        }
        if (tl >= nt) s0 = -INFINITY;
        if (tl + 16 >= nt) s1 = -INFINITY;
        const float mnew = fmaxf(m, group16_max(fmaxf(s0, s1)));
        const float alpha = exp2f(m - mnew);
        const float p0 = exp2f(s0 - mnew), p1 = exp2f(s1 - mnew);
        l = l * alpha + group16_sumf(p0 + p1);
        m = mnew;
        p_sh[row][tl] = p0;
        p_sh[row][tl + 16] = p1;
        __syncthreads();
#pragma unroll
        for (int i = 0; i < DPT; ++i) acc[i] *= alpha;
        for (int t = 0; t < kChunk; ++t) {
            const float p = p_sh[row][t];
#pragma unroll
            for (int i = 0; i < DPT; ++i) acc[i] += p * v_sh[t][tl + 16 * i];
        }
        __syncthreads();
    }
    const size_t entry = (size_t)slot.base * NT + (size_t)tile * n_splits + split;
#pragma unroll
    for (int i = 0; i < DPT; ++i) dv.part_o[(entry * kRowTile + row) * D + tl + 16 * i] = acc[i];
    if (tl == 0) {     // fp32 weights throughout: the two normalisers coincide
        dv.part_ml[entry * kMlRows * kRowTile + row] = m;
        dv.part_ml[entry * kMlRows * kRowTile + kRowTile + row] = l;
        dv.part_ml[entry * kMlRows * kRowTile + 2 * kRowTile + row] = l;
    }
}

// Weighted sum of one unit's split partials for 32 output channels of one row tile
// (the per-thread share): log-sum-exp weights into w_sh, row maxima and normalisers
// into M_sh / L_sh, partial sums into acc.  The workgroup takes rows rbase .. rbase + nr - 1 of the
// tile; RMAX = 4, 8 or 16 bounds nr, MAXS the splits handled.  A thread keeps 128
// partial values in registers per pass, i.e. 64 splits of 16 rows or 128 splits of 8
// rows; MAXS beyond that (a unit that retrieved far more than the others of its launch)
// takes further passes, each one more memory round trip.
// The partial loads of the first pass are issued first, ahead of the (independent) loads
// and barriers of the weight computation: the partials were written by other compute
// units, so every load is a full memory round trip, and the two round trips overlap.
// Split and row indices are clamped instead of tested, so the loads are unconditional
// (straight-line code); what a clamped load brings is never used.
template <int D, int MAXS, int RMAX>
__device__ __forceinline__ void combine_accumulate(const DeviceView &dv, size_t e0, int n_splits, int rbase, int nr, int dg,
                                                   float (*w_sh)[kRowTile], float (*pm)[kRowTile],
                                                   float (*pl)[kRowTile], float (*px)[kRowTile], float *M_sh,
                                                   float *L_sh, float *X_sh, float (&acc)[kRowTile]) {
    constexpr int SPP = 64 * (kRowTile / RMAX);  // splits per pass (128 partial values per thread) ...
    constexpr int NB = (MAXS < SPP ? MAXS : SPP) / 8;   // ... in batches of 8 (fewer when the unit cannot have that many)
    const int tid = threadIdx.x, sg = tid / 32, col = tid % 32;
    float v[NB][RMAX];
    auto load_pass = [&](int s0) {
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const int s = min(s0 + sg + 8 * i, max(n_splits - 1, 0));
            const float *po = dv.part_o + (e0 + s) * kRowTile * D + dg * 32 + col;
#pragma unroll
            for (int r = 0; r < RMAX; ++r) v[i][r] = po[(size_t)(rbase + min(r, nr - 1)) * D];
        }
    };
    load_pass(0);
    {   // per-row maximum and normaliser over the splits
        const int row = tid % 16, part = tid / 16;
        float mr[MAXS / 16], lr[MAXS / 16], xr[MAXS / 16];
        float mx = -INFINITY;
#pragma unroll
        for (int i = 0; i < MAXS / 16; ++i) {
            const int s = part + 16 * i;
            mr[i] = -INFINITY; lr[i] = 0.f; xr[i] = 0.f;
            if (s < n_splits) {
                mr[i] = dv.part_ml[(e0 + s) * kMlRows * kRowTile + row];
                lr[i] = dv.part_ml[(e0 + s) * kMlRows * kRowTile + kRowTile + row];
                xr[i] = dv.part_ml[(e0 + s) * kMlRows * kRowTile + 2 * kRowTile + row];
            }
            mx = fmaxf(mx, mr[i]);
        }
        pm[part][row] = mx;
        __syncthreads();
        float M = -INFINITY;
#pragma unroll
        for (int p = 0; p < 16; ++p) M = fmaxf(M, pm[p][row]);
        float ls = 0.f, xs = 0.f;
#pragma unroll
        for (int i = 0; i < MAXS / 16; ++i) {
            const int s = part + 16 * i;
            if (s < n_splits) {
                const float w = M > -INFINITY ? exp2f(mr[i] - M) : 0.f;
                w_sh[s][row] = w;
                ls += w * lr[i];
                xs += w * xr[i];
            }
        }
        pl[part][row] = ls;
        px[part][row] = xs;
        __syncthreads();
        if (part == 0) {
            float Ls = 0.f, Xs = 0.f;
#pragma unroll
            for (int p = 0; p < 16; ++p) { Ls += pl[p][row]; Xs += px[p][row]; }
            M_sh[row] = M;
            L_sh[row] = Ls;
            X_sh[row] = Xs;
        }
    }
#pragma unroll
    for (int r = 0; r < kRowTile; ++r) acc[r] = 0.f;
    for (int s0 = 0; s0 < (MAXS > SPP ? n_splits : 1); s0 += SPP) {
        if (MAXS > SPP && s0 > 0) load_pass(s0);
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const int s = s0 + sg + 8 * i;
            if (s < n_splits) {
#pragma unroll
                for (int r = 0; r < RMAX; ++r) acc[r] += w_sh[s][min(rbase + r, kRowTile - 1)] * v[i][r];
            }
        }
    }
}

// Merge of the per-split partials (log-sum-exp weights), normalisation, output.
// grid (D/32, NT, n_units), 256 threads.  A workgroup owns 32 output channels of
// one row tile; its 8 groups of 32 threads share the splits, so the partial
// buffer is read with many independent 128-byte loads in flight.
template <typename E, int D>
__global__ __launch_bounds__(kBlock) void k_attend_combine(DeviceView dv, int u0, int n_units, int Tq,
                                                           int B, int uniform_S, E *out, float *lse) {
    // grid.x = (D / 32) * RS: RS workgroups share a tile's rows (a decode step's heaviest unit has up to 256
    // partials to merge, and the launch lasts as long as that unit's workgroups: with its rows shared by two
    // workgroups each thread reads half as much, all of it in one pass)
    constexpr int DG = D / 32;
    const int dg = blockIdx.x % DG, rs = blockIdx.x / DG, RS = gridDim.x / DG;
    const int tile = blockIdx.y, uc = blockIdx.z, u = u0 + uc, NT = gridDim.y;
    const int tid = threadIdx.x;
    const int G = dv.G, Hq = dv.Hq, lc = uc / dv.Hkv, h = u % dv.Hkv, R = Tq * G;
    const int rows = min(kRowTile, R - tile * kRowTile);
    const int rper = (rows + RS - 1) / RS, rbase = rs * rper, nr = min(rper, rows - rbase);
    if (nr <= 0) return;                         // block-uniform: no barrier reached yet
    // uniform_S > 0: every unit has exactly that many splits (the fused decode step); else the
    // splits were shared out by retrieved size and split_slot() says how
    SplitSlot slot{uc, 0, uniform_S, uc * uniform_S, 0};
    if (uniform_S <= 0) slot = split_slot<true>(dv.n_sel + u0, n_units, B, uc);
    const int n_splits = slot.S;                 // 0 if the unit retrieved nothing
    const size_t e0 = (size_t)slot.base * NT + (size_t)tile * n_splits;
    __shared__ float w_sh[kMaxUnitSplits][kRowTile];
    __shared__ float pm[16][kRowTile], pl[16][kRowTile], px[16][kRowTile];
    __shared__ float M_sh[kRowTile], L_sh[kRowTile], X_sh[kRowTile];
    __shared__ float red[8][kRowTile][33];
    const int sg = tid / 32, col = tid % 32;
    float acc[kRowTile];
#define MOSAIC_COMBINE(MAXS, RMAX) \
    combine_accumulate<D, MAXS, RMAX>(dv, e0, n_splits, rbase, nr, dg, w_sh, pm, pl, px, M_sh, L_sh, X_sh, acc)
    if (rper <= 1) {             // block-uniform choices
        if (n_splits <= 64) MOSAIC_COMBINE(64, 1);
        else if (n_splits <= 128) MOSAIC_COMBINE(128, 1);
        else MOSAIC_COMBINE(kMaxUnitSplits, 1);
    } else if (rper <= 2) {
        if (n_splits <= 64) MOSAIC_COMBINE(64, 2);
        else if (n_splits <= 128) MOSAIC_COMBINE(128, 2);
        else MOSAIC_COMBINE(kMaxUnitSplits, 2);
    } else if (rper <= 4) {
        if (n_splits <= 32) MOSAIC_COMBINE(32, 4);
        else if (n_splits <= 64) MOSAIC_COMBINE(64, 4);
        else if (n_splits <= 128) MOSAIC_COMBINE(128, 4);
        else MOSAIC_COMBINE(kMaxUnitSplits, 4);
    } else if (rper <= 8) {
        if (n_splits <= 16) MOSAIC_COMBINE(16, 8);
        else if (n_splits <= 32) MOSAIC_COMBINE(32, 8);
        else if (n_splits <= 64) MOSAIC_COMBINE(64, 8);
        else if (n_splits <= 128) MOSAIC_COMBINE(128, 8);
        else MOSAIC_COMBINE(kMaxUnitSplits, 8);
    } else {
        if (n_splits <= 16) MOSAIC_COMBINE(16, 16);
        else if (n_splits <= 64) MOSAIC_COMBINE(64, 16);
        else MOSAIC_COMBINE(kMaxUnitSplits, 16);
    }
#undef MOSAIC_COMBINE
#pragma unroll
    for (int r = 0; r < kRowTile; ++r) red[sg][r][col] = acc[r];
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int rl = sg + 8 * j;                    // row inside this workgroup's share
        if (rl >= nr) continue;
        const int r = rbase + rl;
        float o = 0.f;
#pragma unroll
        for (int q = 0; q < 8; ++q) o += red[q][rl][col];
        // Lr: normaliser of the output (the weights the value contraction used, bf16-rounded in the
        // MFMA kernels); Xr: the same sum over the unrounded fp32 weights, for the log-sum-exp
        float Lr = L_sh[r], Xr = X_sh[r], Mr = M_sh[r];
        if (dv.aug_reps) {                            // one more partial: the representatives' part
            const size_t ae = (size_t)u * dv.nt_max + tile;
            const float ma = dv.aug_ml[ae * 2 * kRowTile + r], la = dv.aug_ml[ae * 2 * kRowTile + kRowTile + r];
            const float oa = dv.aug_o[(ae * kRowTile + r) * D + dg * 32 + col];
            const float Mn = fmaxf(Mr, ma);
            const float wa = Mr > -INFINITY ? exp2f(Mr - Mn) : 0.f, wb = ma > -INFINITY ? exp2f(ma - Mn) : 0.f;
            o = o * wa + oa * wb;
            Lr = Lr * wa + la * wb;
            Xr = Xr * wa + la * wb;                   // (the representatives' weights are fp32)
            Mr = Mn;
        }
        const int gr = tile * kRowTile + r, t = gr / G, g = gr % G;
        const size_t orow = ((size_t)lc * Tq + t) * Hq + (size_t)h * G + g;
        store_out<E>(out + orow * D + dg * 32 + col, Lr > 0.f ? o / Lr : 0.f);
        if (dg == 0 && col == 0 && lse != nullptr)
            lse[orow] = Xr > 0.f ? (Mr + log2f(Xr)) * 0.6931471805599453f : -INFINITY;
    }
}

} // namespace

hipError_t launch_attend_valu(const DeviceView &dv, int u0, int n_units, const void *q, int Tq,
                              int n_splits, hipStream_t s, hipEvent_t ev0, hipEvent_t ev1) {
    const int NT = (Tq * dv.G + kRowTile - 1) / kRowTile;
    const int B = n_units * n_splits;
    const dim3 grid(B + (dv.aug_reps ? n_units : 0), NT), block(kBlock);
    if (dv.esize == 4) {
        if (dv.D == 64) launch_timed((k_attend_valu<float, 64>), grid, block, 0, s, ev0, ev1, dv, u0, n_units, (const float *)q, Tq, B);
        else launch_timed((k_attend_valu<float, 128>), grid, block, 0, s, ev0, ev1, dv, u0, n_units, (const float *)q, Tq, B);
    } else {
        if (dv.D == 64) launch_timed((k_attend_valu<unsigned short, 64>), grid, block, 0, s, ev0, ev1, dv, u0, n_units, (const unsigned short *)q, Tq, B);
        else launch_timed((k_attend_valu<unsigned short, 128>), grid, block, 0, s, ev0, ev1, dv, u0, n_units, (const unsigned short *)q, Tq, B);
    }
    return hipGetLastError();
}

hipError_t launch_attend_combine(const DeviceView &dv, int u0, int n_units, int Tq, int n_splits,
                                 void *out, float *lse, hipStream_t s, bool uniform) {
    const int us = uniform ? n_splits : 0;
    const int NT = (Tq * dv.G + kRowTile - 1) / kRowTile;
    const int B = n_units * n_splits;
    // One row tile (a decode step) of a few units: up to eight workgroups share a tile's rows, as long as the launch
    // stays within about two workgroups per CU (per-layer launch of config 2: 1075 -> 1048 / 1033 / 1027 us per step
    // with 2 / 4 / 8; the all-layers launch, 112 units, is left alone: 542 -> 562 us with 8).
    const int RS = NT == 1 ? std::max(1, std::min(8, 512 / (n_units * (dv.D / 32)))) : 1;
    dim3 grid(dv.D / 32 * RS, NT, n_units);
    if (dv.esize == 4) {
        if (dv.D == 64) k_attend_combine<float, 64><<<grid, kBlock, 0, s>>>(dv, u0, n_units, Tq, B, us, (float *)out, lse);
        else k_attend_combine<float, 128><<<grid, kBlock, 0, s>>>(dv, u0, n_units, Tq, B, us, (float *)out, lse);
    } else {
        if (dv.D == 64) k_attend_combine<unsigned short, 64><<<grid, kBlock, 0, s>>>(dv, u0, n_units, Tq, B, us, (unsigned short *)out, lse);
        else k_attend_combine<unsigned short, 128><<<grid, kBlock, 0, s>>>(dv, u0, n_units, Tq, B, us, (unsigned short *)out, lse);
    }
    return hipGetLastError();
}

} // namespace mosaic
