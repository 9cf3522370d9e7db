// Attention over the retrieved KV on the matrix cores (bf16 pages, values
// stored transposed [D][Tp]); paper Sec. V-A (2).  The G*Tq query rows of a
// unit form the small dense operand, so both the logits (K Q^T) and the output
// (V^T P^T) are 16x16x32 bf16 MFMA contractions fed straight from global
// memory with 16-byte loads: no LDS staging, no register transposes.
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
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ bf16x8 ld_frag(const unsigned short *p) {
    const uint4 w = *reinterpret_cast<const uint4 *>(p);
    return __builtin_bit_cast(bf16x8, w);
}
__device__ __forceinline__ bf16x8 zero_frag() {
    return __builtin_bit_cast(bf16x8, make_uint4(0u, 0u, 0u, 0u));
}

// grid (n_splits, DECODE ? 1 : ceil(NT/4), n_units), 256 threads = 4 waves.
// DECODE (one row tile): the waves share the split's chunks (wave w takes
// chunks c0+w, c0+w+4, ...) and merge through LDS.  Otherwise wave w owns row
// tile 4*blockIdx.y + w and walks every chunk of the split.
template <int D, bool DECODE>
__global__ __launch_bounds__(kBlock) void k_attend_mfma(DeviceView dv, int u0,
                                                        const unsigned short *q, int Tq,
                                                        int n_splits, int NT) {
    constexpr int KK = D / 32;   // k-steps of the logit contraction
    constexpr int DB = D / 16;   // 16-channel blocks of the output
    const int split = blockIdx.x, uc = blockIdx.z, u = u0 + uc;
    const int tid = threadIdx.x, wave = tid / 64, lane = tid % 64, g = lane / 16, n = lane % 16;
    const int tile = DECODE ? 0 : (int)blockIdx.y * 4 + wave;
    if (!DECODE && tile >= NT) return;   // no barriers on this path
    const int G = dv.G, Hq = dv.Hq, T = dv.T, Tp = dv.Tp, F = dv.F;
    const int lc = uc / dv.Hkv, h = u % dv.Hkv, R = Tq * G;

    bf16x8 qf[KK];
    {
        const int gr = tile * kRowTile + n;
        if (gr < R) {
            const int t = gr / G, gg = gr % G;
            const unsigned short *qr = q + (((size_t)lc * Tq + t) * Hq + (size_t)h * G + gg) * D;
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) qf[kk] = ld_frag(qr + 32 * kk + 8 * g);
        } else {
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) qf[kk] = zero_frag();
        }
    }
    const int cpp = dv.chunks_per_page;
    const int NC = dv.n_sel[u] * cpp;
    const int cps = (NC + n_splits - 1) / n_splits;
    const int c0 = split * cps, c1 = min(NC, c0 + cps);
    const int *sel = dv.sel_pages + (size_t)u * F;
    const unsigned short *kbase = reinterpret_cast<const unsigned short *>(dv.k_store) + (size_t)u * F * T * D;
    const unsigned short *vbase = reinterpret_cast<const unsigned short *>(dv.v_store) + (size_t)u * F * D * Tp;
    const float sl2 = 1.4426950408889634f / sqrtf((float)D);

    f32x4 acc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db) acc[db] = f32x4{0.f, 0.f, 0.f, 0.f};
    float m = -INFINITY, l = 0.f;

    for (int c = DECODE ? c0 + wave : c0; c < c1; c += DECODE ? 4 : 1) {
        const int page = sel[c / cpp], t0 = (c % cpp) * kChunk;
        const unsigned short *kp = kbase + (size_t)page * T * D;
        const unsigned short *vp = vbase + (size_t)page * D * Tp;
        f32x4 s[2];
#pragma unroll
        for (int tau = 0; tau < 2; ++tau) {
            const int tok = t0 + 8 * (n / 4) + 4 * tau + (n % 4);
            s[tau] = f32x4{0.f, 0.f, 0.f, 0.f};
            const bool valid = tok < T;
            const unsigned short *kr = kp + (size_t)(valid ? tok : 0) * D + 8 * g;
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) {
                const bf16x8 a = valid ? ld_frag(kr + 32 * kk) : zero_frag();
                s[tau] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, qf[kk], s[tau], 0, 0, 0);
            }
        }
        float sv[8];
        float cmax = -INFINITY;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int tok = t0 + 8 * g + j;
            sv[j] = tok < T ? s[j / 4][j % 4] * sl2 : -INFINITY;
            cmax = fmaxf(cmax, sv[j]);
        }
        cmax = fmaxf(cmax, __shfl_xor(cmax, 16, 64));
        cmax = fmaxf(cmax, __shfl_xor(cmax, 32, 64));
        const float mnew = fmaxf(m, cmax);
        const float alpha = exp2f(m - mnew);
        unsigned int pw[4];
        float psum = 0.f;
#pragma unroll
        for (int j = 0; j < 8; j += 2) {
            const unsigned short b0 = f32_to_bf16_rne(exp2f(sv[j] - mnew));
            const unsigned short b1 = f32_to_bf16_rne(exp2f(sv[j + 1] - mnew));
            psum += bf16_to_f32(b0) + bf16_to_f32(b1);   // the sum uses the rounded weights
            pw[j / 2] = (unsigned int)b0 | ((unsigned int)b1 << 16);
        }
        l = l * alpha + psum;
        m = mnew;
        const bf16x8 pf = __builtin_bit_cast(bf16x8, make_uint4(pw[0], pw[1], pw[2], pw[3]));
        const bool vvalid = t0 + 8 * g < Tp;
        const unsigned short *vr = vp + (size_t)n * Tp + (vvalid ? t0 + 8 * g : 0);
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            const bf16x8 a = vvalid ? ld_frag(vr + (size_t)(16 * db) * Tp) : zero_frag();
            acc[db] = acc[db] * alpha;
            acc[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, pf, acc[db], 0, 0, 0);
        }
    }
    l += __shfl_xor(l, 16, 64);
    l += __shfl_xor(l, 32, 64);

    if constexpr (!DECODE) {
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
    } else {
        __shared__ float o_sh[4][D][kRowTile + 1];
        __shared__ float m_sh[4][kRowTile], l_sh[4][kRowTile];
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int i = 0; i < 4; ++i) o_sh[wave][16 * db + 4 * g + i][n] = acc[db][i];
        if (g == 0) { m_sh[wave][n] = m; l_sh[wave][n] = l; }
        __syncthreads();
        const int row = tid / 16, dl = tid % 16;
        float M = -INFINITY;
#pragma unroll
        for (int w = 0; w < 4; ++w) M = fmaxf(M, m_sh[w][row]);
        float wgt[4], L = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            wgt[w] = M > -INFINITY ? exp2f(m_sh[w][row] - M) : 0.f;
            L += wgt[w] * l_sh[w][row];
        }
        const size_t entry = (size_t)uc * n_splits + split;   // NT == 1
        float *po = dv.part_o + (entry * kRowTile + row) * D;
        for (int d = dl; d < D; d += 16) {
            float o = 0.f;
#pragma unroll
            for (int w = 0; w < 4; ++w) o += wgt[w] * o_sh[w][d][row];
            po[d] = o;
        }
        if (dl == 0) {
            dv.part_ml[entry * 2 * kRowTile + row] = M;
            dv.part_ml[entry * 2 * kRowTile + kRowTile + row] = L;
        }
    }
}

} // namespace

hipError_t launch_attend_mfma(const DeviceView &dv, int u0, int n_units, const void *q, int Tq,
                              int n_splits, hipStream_t s) {
    const int NT = (Tq * dv.G + kRowTile - 1) / kRowTile;
    const unsigned short *qq = (const unsigned short *)q;
    if (NT == 1) {
        dim3 grid(n_splits, 1, n_units);
        if (dv.D == 64) k_attend_mfma<64, true><<<grid, kBlock, 0, s>>>(dv, u0, qq, Tq, n_splits, NT);
        else k_attend_mfma<128, true><<<grid, kBlock, 0, s>>>(dv, u0, qq, Tq, n_splits, NT);
    } else {
        dim3 grid(n_splits, (NT + 3) / 4, n_units);
        if (dv.D == 64) k_attend_mfma<64, false><<<grid, kBlock, 0, s>>>(dv, u0, qq, Tq, n_splits, NT);
        else k_attend_mfma<128, false><<<grid, kBlock, 0, s>>>(dv, u0, qq, Tq, n_splits, NT);
    }
    return hipGetLastError();
}

} // namespace mosaic
