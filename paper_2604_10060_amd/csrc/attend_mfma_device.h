// Device helpers shared by the bf16 MFMA attention kernels: operand fragments of
// v_mfma_f32_16x16x32_bf16, the online-softmax chunk step, the operand loads of one
// 32-token chunk, and the merge of a workgroup's four wavefronts into one partial.
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
#pragma once
#include "mosaic_internal.h"

namespace mosaic {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ bf16x8 ld_frag(const unsigned short *p) {
    const uint4 w = *reinterpret_cast<const uint4 *>(p);
    return __builtin_bit_cast(bf16x8, w);
}
// The decode kernels read every K/V operand once per step.  When the stored KV is far larger than
// the chip's caches the loads carry the non-temporal hint (nothing worth keeping is displaced and
// the lines are not allocated for reuse): 562 -> 519 us for a 3.3 GB launch.  A small store (all of
// it fits the 256 MB memory-side cache) is read faster without the hint.
__device__ __forceinline__ bf16x8 ld_frag_stream(const unsigned short *p) {
    typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
    const u32x4_t w = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p));
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

// Online softmax with a lazily updated reference: the running reference m of a
// row (log2 domain) is only raised -- and the accumulators only rescaled -- when
// some logit exceeds it by more than kLazy; until then weights are
// exp2(s - m) <= 2^kLazy, exact in fp32/bf16 range, and (m, sum, O) stay a
// consistent triple for the later log-sum-exp merge.  The cross-lane maximum and
// the rescale therefore leave the common path.
constexpr float kLazy = 8.0f;

// R row tiles of 16 query rows share one chunk's operands (kf: 2 key tiles x KK
// k-steps; vf: DB channel blocks).  n_valid = tokens of the chunk that exist
// (the rest are clamped re-reads and get weight 0).  Three phases -- all logit
// MFMAs, all softmax arithmetic, all output MFMAs -- so the independent chains
// of the tiles overlap.
// The normaliser l is either a per-lane float (sum of this lane's 8 weights; the caller
// adds the four lane groups at the end) or an f32x4 accumulator fed by one more MFMA
// whose A operand is all ones: every element of it is then the row's full sum over
// the 32 tokens, and the 8 adds per tile leave the vector ALU.
// lx is the per-lane sum of the UNROUNDED fp32 weights (this lane's 8 tokens of a row): the
// output divides by l, whose weights are the bf16-rounded ones the PV contraction used, while the
// log-sum-exp the caller gets is formed from lx, so it carries fp32 rounding only.
template <int D, int R, typename LT>
__device__ __forceinline__ void chunk_step_multi(const bf16x8 (&kf)[2 * (D / 32)], const bf16x8 (&vf)[D / 16],
                                                 const bf16x8 (&qf)[R][D / 32], int n_valid, int g,
                                                 float sl2, f32x4 (&acc)[R][D / 16], float (&m)[R],
                                                 LT (&l)[R], float (&lx)[R]) {
    constexpr int KK = D / 32, DB = D / 16;
    constexpr bool kSumByMfma = sizeof(LT) == sizeof(f32x4);
    f32x4 s[R][2];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int tau = 0; tau < 2; ++tau) {
            s[r][tau] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < KK; ++kk)
                s[r][tau] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[tau * KK + kk], qf[r][kk], s[r][tau], 0, 0, 0);
        }
    if (n_valid < kChunk) {             // ragged last chunk of a page (wave-uniform)
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int j = 0; j < 8; ++j)
                if (8 * g + j >= n_valid) s[r][j / 4][j % 4] = -INFINITY;
    }
    bf16x8 pf[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const float c0 = fmaxf(fmaxf(s[r][0][0], s[r][0][1]), fmaxf(s[r][0][2], s[r][0][3]));
        const float c1 = fmaxf(fmaxf(s[r][1][0], s[r][1][1]), fmaxf(s[r][1][2], s[r][1][3]));
        float cm = fmaxf(c0, c1) * sl2;
        if (__builtin_amdgcn_ballot_w64(cm > m[r] + kLazy)) {   // rare, wave-uniform
            cm = fmaxf(cm, __shfl_xor(cm, 16, 64));
            cm = fmaxf(cm, __shfl_xor(cm, 32, 64));
            const float mnew = fmaxf(m[r], cm);
            const float alpha = __builtin_amdgcn_exp2f(m[r] - mnew);
            l[r] = l[r] * alpha;
            lx[r] = lx[r] * alpha;
            m[r] = mnew;
#pragma unroll
            for (int db = 0; db < DB; ++db) acc[r][db] = acc[r][db] * alpha;
        }
        const float nm = -m[r];
        unsigned int pw[4];
        float xs = 0.f;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[r][(2 * j) / 4][(2 * j) % 4], sl2, nm));
            const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[r][(2 * j + 1) / 4][(2 * j + 1) % 4], sl2, nm));
            pw[j] = pack_bf16(p0, p1);
            xs += p0 + p1;
        }
        lx[r] += xs;
        pf[r] = __builtin_bit_cast(bf16x8, make_uint4(pw[0], pw[1], pw[2], pw[3]));
        if constexpr (!kSumByMfma) {               // the normaliser uses the rounded weights
            float psum = 0.f;
#pragma unroll
            for (int j = 0; j < 4; ++j) psum += bf16_lo(pw[j]) + bf16_hi(pw[j]);
            l[r] += psum;
        }
    }
    if constexpr (kSumByMfma) {
        const bf16x8 ones = __builtin_bit_cast(bf16x8, make_uint4(0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u));
#pragma unroll
        for (int r = 0; r < R; ++r) l[r] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, pf[r], l[r], 0, 0, 0);
    }
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int db = 0; db < DB; ++db)
            acc[r][db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[db], pf[r], acc[r][db], 0, 0, 0);
}

// Single-tile form used by the decode kernel.
template <int D>
__device__ __forceinline__ void chunk_step(const bf16x8 (&kf)[2 * (D / 32)], const bf16x8 (&vf)[D / 16],
                                           const bf16x8 (&qf)[D / 32], int n_valid, int g, float sl2,
                                           f32x4 (&acc)[D / 16], float &m, float &l, float &lx) {
    const bf16x8 (&q1)[1][D / 32] = reinterpret_cast<const bf16x8 (&)[1][D / 32]>(qf);
    f32x4 (&a1)[1][D / 16] = reinterpret_cast<f32x4 (&)[1][D / 16]>(acc);
    float (&m1)[1] = reinterpret_cast<float (&)[1]>(m);
    float (&l1)[1] = reinterpret_cast<float (&)[1]>(l);
    float (&x1)[1] = reinterpret_cast<float (&)[1]>(lx);
    chunk_step_multi<D, 1, float>(kf, vf, q1, n_valid, g, sl2, a1, m1, l1, x1);
}

// Issue the 16-byte operand loads of one chunk.  Tokens beyond the page's T are
// clamped to the last token (valid memory, weight 0 later); the value blocks are
// zero-padded to 32 tokens at ingest.
template <int D, bool STREAM>
__device__ __forceinline__ void issue_chunk(const unsigned short *kpage, const unsigned short *vchunk,
                                            int t0, int T, int g, int n, bf16x8 (&kf)[2 * (D / 32)],
                                            bf16x8 (&vf)[D / 16]) {
    constexpr int KK = D / 32, DB = D / 16;
#pragma unroll
    for (int tau = 0; tau < 2; ++tau) {
        const int tok = min(t0 + 8 * (n / 4) + 4 * tau + (n % 4), T - 1);
        const unsigned short *kr = kpage + (size_t)tok * D + 8 * g;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) kf[tau * KK + kk] = STREAM ? ld_frag_stream(kr + 32 * kk) : ld_frag(kr + 32 * kk);
    }
    const unsigned short *vr = vchunk + n * 32 + 8 * g;
#pragma unroll
    for (int db = 0; db < DB; ++db) vf[db] = STREAM ? ld_frag_stream(vr + 16 * db * 32) : ld_frag(vr + 16 * db * 32);
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

// Merge of the four wavefronts' running (m, l, O) of one row tile and store of the
// workgroup's partial at `entry` (shared by the decode kernels).  All threads call it.
template <int D>
__device__ __forceinline__ void merge_waves_store(const DeviceView &dv, const f32x4 (&acc)[D / 16], float m, float l,
                                                  float lx, int R, size_t entry) {
    constexpr int DB = D / 16;
    const int tid = threadIdx.x, wave = tid / 64, lane = tid % 64, g = lane / 16, n = lane % 16;
    l += __shfl_xor(l, 16, 64);
    l += __shfl_xor(l, 32, 64);
    lx += __shfl_xor(lx, 16, 64);
    lx += __shfl_xor(lx, 32, 64);
    __shared__ float o_sh[4][D][kRowTile + 1];
    __shared__ float m_sh[4][kRowTile], l_sh[4][kRowTile], x_sh[4][kRowTile];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i = 0; i < 4; ++i) o_sh[wave][16 * db + 4 * g + i][n] = acc[db][i];
    if (g == 0) { m_sh[wave][n] = m; l_sh[wave][n] = l; x_sh[wave][n] = lx; }
    __syncthreads();
    const int row = tid / 16, dl = tid % 16;
    if (row >= R) return;
    float M = -INFINITY;
#pragma unroll
    for (int w = 0; w < 4; ++w) M = fmaxf(M, m_sh[w][row]);
    float wgt[4], Lsum = 0.f, Xsum = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        wgt[w] = M > -INFINITY ? __builtin_amdgcn_exp2f(m_sh[w][row] - M) : 0.f;
        Lsum += wgt[w] * l_sh[w][row];
        Xsum += wgt[w] * x_sh[w][row];
    }
    float *po = dv.part_o + (entry * kRowTile + row) * D;
#pragma unroll
    for (int d = dl; d < D; d += 16) {
        float o = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) o += wgt[w] * o_sh[w][d][row];
        po[d] = o;
    }
    if (dl == 0) {
        dv.part_ml[entry * kMlRows * kRowTile + row] = M;
        dv.part_ml[entry * kMlRows * kRowTile + kRowTile + row] = Lsum;
        dv.part_ml[entry * kMlRows * kRowTile + 2 * kRowTile + row] = Xsum;
    }
}


} // namespace mosaic
