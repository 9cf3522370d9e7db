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

namespace mosaic {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ bf16x8 ld_frag(const unsigned short *p) {
    const uint4 w = *reinterpret_cast<const uint4 *>(p);
    return __builtin_bit_cast(bf16x8, w);
}
__device__ __forceinline__ bf16x8 zero_frag() {
    return __builtin_bit_cast(bf16x8, make_uint4(0u, 0u, 0u, 0u));
}
// two fp32 -> packed bf16 (round to nearest even, hardware convert)
__device__ __forceinline__ unsigned int pack_bf16(float a, float b) {
    const f32x2 v = {a, b};
    return __builtin_bit_cast(unsigned int, __builtin_convertvector(v, bf16x2));
}
__device__ __forceinline__ float bf16_lo(unsigned int w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(unsigned int w) { return __uint_as_float(w & 0xffff0000u); }

// One 32-token step of the online softmax for the 16 query rows of a tile.
// kf: 2 key tiles x KK k-steps; vf: DB channel blocks.  n_valid = tokens of the
// chunk that exist (the rest are clamped re-reads and get weight 0).
template <int D>
__device__ __forceinline__ void chunk_step(const bf16x8 (&kf)[2 * (D / 32)], const bf16x8 (&vf)[D / 16],
                                           const bf16x8 (&qf)[D / 32], int n_valid, int g, float sl2,
                                           f32x4 (&acc)[D / 16], float &m, float &l) {
    constexpr int KK = D / 32, DB = D / 16;
    f32x4 s[2];
#pragma unroll
    for (int tau = 0; tau < 2; ++tau) {
        s[tau] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < KK; ++kk)
            s[tau] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[tau * KK + kk], qf[kk], s[tau], 0, 0, 0);
    }
    float sv[8];
    float cmax = -INFINITY;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        sv[j] = (8 * g + j) < n_valid ? s[j / 4][j % 4] * sl2 : -INFINITY;
        cmax = fmaxf(cmax, sv[j]);
    }
    cmax = fmaxf(cmax, __shfl_xor(cmax, 16, 64));
    cmax = fmaxf(cmax, __shfl_xor(cmax, 32, 64));
    const float mnew = fmaxf(m, cmax);
    const float alpha = __builtin_amdgcn_exp2f(m - mnew);
    unsigned int pw[4];
    float psum = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        pw[j] = pack_bf16(__builtin_amdgcn_exp2f(sv[2 * j] - mnew),
                          __builtin_amdgcn_exp2f(sv[2 * j + 1] - mnew));
        psum += bf16_lo(pw[j]) + bf16_hi(pw[j]);   // the normaliser uses the rounded weights
    }
    l = l * alpha + psum;
    m = mnew;
    const bf16x8 pf = __builtin_bit_cast(bf16x8, make_uint4(pw[0], pw[1], pw[2], pw[3]));
#pragma unroll
    for (int db = 0; db < DB; ++db) {
        acc[db] = acc[db] * alpha;
        acc[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[db], pf, acc[db], 0, 0, 0);
    }
}

// Issue the 16-byte operand loads of one chunk.  Tokens beyond the page's T are
// clamped to the last token (valid memory, weight 0 later); the value blocks are
// zero-padded to 32 tokens at ingest.
template <int D>
__device__ __forceinline__ void issue_chunk(const unsigned short *kpage, const unsigned short *vchunk,
                                            int t0, int T, int g, int n, bf16x8 (&kf)[2 * (D / 32)],
                                            bf16x8 (&vf)[D / 16]) {
    constexpr int KK = D / 32, DB = D / 16;
#pragma unroll
    for (int tau = 0; tau < 2; ++tau) {
        const int tok = min(t0 + 8 * (n / 4) + 4 * tau + (n % 4), T - 1);
        const unsigned short *kr = kpage + (size_t)tok * D + 8 * g;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) kf[tau * KK + kk] = ld_frag(kr + 32 * kk);
    }
    const unsigned short *vr = vchunk + n * 32 + 8 * g;
#pragma unroll
    for (int db = 0; db < DB; ++db) vf[db] = ld_frag(vr + 16 * db * 32);
}

template <int D>
__device__ __forceinline__ void load_q(const DeviceView &dv, const unsigned short *q, int lc, int h,
                                       int Tq, int row, int g, bf16x8 (&qf)[D / 32]) {
    constexpr int KK = D / 32;
    const int G = dv.G;
    if (row < Tq * G) {
        const int t = row / G, gg = row % G;
        const unsigned short *qr = q + (((size_t)lc * Tq + t) * dv.Hq + (size_t)h * G + gg) * D;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) qf[kk] = ld_frag(qr + 32 * kk + 8 * g);
    } else {
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) qf[kk] = zero_frag();
    }
}

// ---------------------------------------------------------------------------
// Decode shape: at most 16 query rows per unit (one row tile).
// grid (n_splits, 1, n_units), 4 waves.  Chunks are dealt round-robin:
// wave w of split s takes chunks s + S*(w + 4*i), so chunk indices (and the
// page ids behind them) are known before the selection size has arrived, and
// the next chunk's operands are in flight while the current one is reduced.
// ---------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(kBlock, 2) void k_attend_decode_mfma(DeviceView dv, int u0,
                                                                  const unsigned short *q, int Tq,
                                                                  int n_splits) {
    constexpr int KK = D / 32, DB = D / 16;
    const int split = blockIdx.x, uc = blockIdx.z, u = u0 + uc;
    const int tid = threadIdx.x, wave = tid / 64, lane = tid % 64, g = lane / 16, n = lane % 16;
    const int T = dv.T, F = dv.F, cpp = dv.chunks_per_page;
    const int lc = uc / dv.Hkv, h = u % dv.Hkv, R = Tq * dv.G;
    const int *sel = dv.sel_pages + (size_t)u * F;
    const int stride = 4 * n_splits, first = split + n_splits * wave;

    const int nsel = dv.n_sel[u];
    // page ids of this wave's first 64 chunks, one per lane, loaded speculatively
    int pgs = sel[min((first + stride * lane) / cpp, F - 1)];
    bf16x8 qf[KK];
    load_q<D>(dv, q, lc, h, Tq, n, g, qf);

    const unsigned short *kbase = reinterpret_cast<const unsigned short *>(dv.k_store) + (size_t)u * F * T * D;
    const unsigned short *vbase = reinterpret_cast<const unsigned short *>(dv.v_store) + (size_t)u * F * D * dv.Tp;
    const size_t kpage_elems = (size_t)T * D, vpage_elems = (size_t)D * dv.Tp;
    const float sl2 = 1.4426950408889634f / sqrtf((float)D);

    f32x4 acc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db) acc[db] = f32x4{0.f, 0.f, 0.f, 0.f};
    float m = -INFINITY, l = 0.f;

    const int NC = nsel * cpp;
    const int n_my = first < NC ? (NC - first + stride - 1) / stride : 0;

    bf16x8 kA[2 * KK], vA[DB], kB[2 * KK], vB[DB];
    auto issue = [&](int i, bf16x8 (&kf)[2 * KK], bf16x8 (&vf)[DB]) {
        if ((i & 63) == 0 && i > 0) pgs = sel[min((first + stride * (i + lane)) / cpp, F - 1)];
        const int ci = first + stride * i, cc = ci % cpp;
        const int page = __builtin_amdgcn_readlane(pgs, i & 63);
        issue_chunk<D>(kbase + (size_t)page * kpage_elems,
                       vbase + (size_t)page * vpage_elems + (size_t)cc * D * 32, cc * kChunk, T, g, n,
                       kf, vf);
    };
    auto valid = [&](int i) { return min(kChunk, T - ((first + stride * i) % cpp) * kChunk); };

    if (n_my > 0) {
        int i = 0;
        issue(0, kA, vA);
        while (true) {
            if (i + 1 < n_my) issue(i + 1, kB, vB);
            chunk_step<D>(kA, vA, qf, valid(i), g, sl2, acc, m, l);
            if (++i >= n_my) break;
            if (i + 1 < n_my) issue(i + 1, kA, vA);
            chunk_step<D>(kB, vB, qf, valid(i), g, sl2, acc, m, l);
            if (++i >= n_my) break;
        }
    }
    l += __shfl_xor(l, 16, 64);
    l += __shfl_xor(l, 32, 64);

    // merge the four waves, write one partial per workgroup
    __shared__ float o_sh[4][D][kRowTile + 1];
    __shared__ float m_sh[4][kRowTile], l_sh[4][kRowTile];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i = 0; i < 4; ++i) o_sh[wave][16 * db + 4 * g + i][n] = acc[db][i];
    if (g == 0) { m_sh[wave][n] = m; l_sh[wave][n] = l; }
    __syncthreads();
    const int row = tid / 16, dl = tid % 16;
    if (row >= R) return;
    float M = -INFINITY;
#pragma unroll
    for (int w = 0; w < 4; ++w) M = fmaxf(M, m_sh[w][row]);
    float wgt[4], Lsum = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        wgt[w] = M > -INFINITY ? __builtin_amdgcn_exp2f(m_sh[w][row] - M) : 0.f;
        Lsum += wgt[w] * l_sh[w][row];
    }
    const size_t entry = (size_t)uc * n_splits + split;   // one row tile
    float *po = dv.part_o + (entry * kRowTile + row) * D;
#pragma unroll
    for (int d = dl; d < D; d += 16) {
        float o = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) o += wgt[w] * o_sh[w][d][row];
        po[d] = o;
    }
    if (dl == 0) {
        dv.part_ml[entry * 2 * kRowTile + row] = M;
        dv.part_ml[entry * 2 * kRowTile + kRowTile + row] = Lsum;
    }
}

// ---------------------------------------------------------------------------
// Multi-token questions: wave w owns row tile 4*blockIdx.y + w and walks the
// contiguous chunk range of its split, next chunk prefetched.
// grid (n_splits, ceil(NT/4), n_units).  With n_splits a multiple of 8 the
// workgroups that re-read the same keys/values land on the same XCD (ids
// congruent mod 8), so the re-reads hit that XCD's L2.
// ---------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(kBlock, 2) void k_attend_prefill_mfma(DeviceView dv, int u0,
                                                                   const unsigned short *q, int Tq,
                                                                   int n_splits, int NT) {
    constexpr int KK = D / 32, DB = D / 16;
    const int split = blockIdx.x, uc = blockIdx.z, u = u0 + uc;
    const int tid = threadIdx.x, wave = tid / 64, lane = tid % 64, g = lane / 16, n = lane % 16;
    const int tile = (int)blockIdx.y * 4 + wave;
    if (tile >= NT) return;   // no barriers in this kernel
    const int T = dv.T, F = dv.F, cpp = dv.chunks_per_page;
    const int lc = uc / dv.Hkv, h = u % dv.Hkv;
    const int *sel = dv.sel_pages + (size_t)u * F;
    bf16x8 qf[KK];
    load_q<D>(dv, q, lc, h, Tq, tile * kRowTile + n, g, qf);
    const int NC = dv.n_sel[u] * cpp;
    const int cps = (NC + n_splits - 1) / n_splits;
    const int c0 = split * cps, c1 = min(NC, c0 + cps);
    const unsigned short *kbase = reinterpret_cast<const unsigned short *>(dv.k_store) + (size_t)u * F * T * D;
    const unsigned short *vbase = reinterpret_cast<const unsigned short *>(dv.v_store) + (size_t)u * F * D * dv.Tp;
    const size_t kpage_elems = (size_t)T * D, vpage_elems = (size_t)D * dv.Tp;
    const float sl2 = 1.4426950408889634f / sqrtf((float)D);

    f32x4 acc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db) acc[db] = f32x4{0.f, 0.f, 0.f, 0.f};
    float m = -INFINITY, l = 0.f;
    bf16x8 kA[2 * KK], vA[DB], kB[2 * KK], vB[DB];
    auto issue = [&](int c, bf16x8 (&kf)[2 * KK], bf16x8 (&vf)[DB]) {
        const int page = sel[c / cpp], cc = c % cpp;
        issue_chunk<D>(kbase + (size_t)page * kpage_elems,
                       vbase + (size_t)page * vpage_elems + (size_t)cc * D * 32, cc * kChunk, T, g, n,
                       kf, vf);
    };
    auto valid = [&](int c) { return min(kChunk, T - (c % cpp) * kChunk); };
    if (c0 < c1) {
        int c = c0;
        issue(c, kA, vA);
        while (true) {
            if (c + 1 < c1) issue(c + 1, kB, vB);
            chunk_step<D>(kA, vA, qf, valid(c), g, sl2, acc, m, l);
            if (++c >= c1) break;
            if (c + 1 < c1) issue(c + 1, kA, vA);
            chunk_step<D>(kB, vB, qf, valid(c), g, sl2, acc, m, l);
            if (++c >= c1) break;
        }
    }
    l += __shfl_xor(l, 16, 64);
    l += __shfl_xor(l, 32, 64);
    const size_t entry = ((size_t)uc * NT + tile) * n_splits + split;
    float *po = dv.part_o + (entry * kRowTile + n) * D;
#pragma unroll
    for (int db = 0; db < DB; ++db)
        *reinterpret_cast<float4 *>(po + 16 * db + 4 * g) =
            make_float4(acc[db][0], acc[db][1], acc[db][2], acc[db][3]);
    if (g == 0) {
        dv.part_ml[entry * 2 * kRowTile + n] = m;
        dv.part_ml[entry * 2 * kRowTile + kRowTile + n] = l;
    }
}

} // namespace

hipError_t launch_attend_mfma(const DeviceView &dv, int u0, int n_units, const void *q, int Tq,
                              int n_splits, hipStream_t s, hipEvent_t ev0, hipEvent_t ev1) {
    const int NT = (Tq * dv.G + kRowTile - 1) / kRowTile;
    const unsigned short *qq = (const unsigned short *)q;
    const dim3 block(kBlock);
    if (NT == 1) {
        const dim3 grid(n_splits, 1, n_units);
        if (dv.D == 64) hipExtLaunchKernelGGL(k_attend_decode_mfma<64>, grid, block, 0, s, ev0, ev1, 0, dv, u0, qq, Tq, n_splits);
        else hipExtLaunchKernelGGL(k_attend_decode_mfma<128>, grid, block, 0, s, ev0, ev1, 0, dv, u0, qq, Tq, n_splits);
    } else {
        const dim3 grid(n_splits, (NT + 3) / 4, n_units);
        if (dv.D == 64) hipExtLaunchKernelGGL(k_attend_prefill_mfma<64>, grid, block, 0, s, ev0, ev1, 0, dv, u0, qq, Tq, n_splits, NT);
        else hipExtLaunchKernelGGL(k_attend_prefill_mfma<128>, grid, block, 0, s, ev0, ev1, 0, dv, u0, qq, Tq, n_splits, NT);
    }
    return hipGetLastError();
}

} // namespace mosaic
