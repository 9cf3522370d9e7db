// Multi-token questions (paper Sec. V-A (2): attention of a question chunk over the retrieved
// KV), MFMA-bound.  A workgroup of NW wavefronts owns NW * 16 * kPrefillTiles query rows: wave w
// holds kPrefillTiles row tiles of 16 in registers and all waves walk the same chunk range, so
// each 32-token K/V chunk is fetched from memory once per workgroup, placed in LDS and read as
// MFMA operands by every wave.  NW = 4 is what is launched (two workgroups per CU).  NW = 8 (one
// workgroup of 256 rows per CU, eight LDS slots per operand, loads issued three barrier
// intervals ahead) runs at the same rate (627 against 630 TFLOP/s on 256-token questions), i.e.
// neither the loads' latency nor the L2 -> LDS volume is what bounds this kernel.
//
// Global -> LDS without registers: every lane's 16-byte load is written by the memory pipeline
// straight into LDS (lane l of a wavefront's load lands at base + 16 l), so the copy holds no
// staging registers, issues no LDS stores and computes no store addresses; which 16 bytes a lane
// fetches is free, so the layout below is produced by choosing the SOURCE address per lane.
// LDS holds NW key slots and NW value slots of one chunk each (chunk c lives in slot c % NW); the
// loads of a chunk are issued NW / 2 - 1 barrier intervals (of two chunks) before it is used, and
// a barrier only waits for the loads that are due (s_waitcnt vmcnt(N), younger ones stay in flight).
//
// LDS layout (per 32-token chunk: 32 x D keys / D x 32 values, both unpadded):
//   keys    row slot s = 16 tau + 4 j + i holds token 8 j + 4 tau + i  (MFMA slot order: lane
//           (g, n) of key tile tau then owns the logits of tokens 8 g .. 8 g + 7, the k-slots of
//           the value contraction), 16-byte pieces of a row XOR-swizzled with the row number;
//   values  [channel][32 tokens] as in memory, pieces XOR-swizzled with channel / 4.
//   A 16-lane group's operand read (16 rows, one piece each) then covers all 64 banks once.
//
// What bounds it (D = 128, 256-token questions: 0.25 of the bf16 MFMA peak).  Per 16 x 32 block of
// logits a wave issues 17 MFMAs (272 cycles of the matrix pipe) and about 45 vector-ALU
// instructions, 8 of them exp2 (about 210 cycles of the vector pipe): scale-and-shift, exp2, two
// sums (the bf16-rounded one by MFMA, the exact one for the log-sum-exp on the ALU), convert,
// maximum -- what a 32-bit softmax needs without packed two-element instructions.  A loop of
// independent instructions with this mix runs at 0.6-0.7 of the MFMA peak on this chip (a wave64
// VALU instruction issues every 4 cycles, exp2 every 8, an MFMA every 16; two VALU instructions
// per MFMA hide completely, further ones add 5-10 cycles each), so the mix is not the limit.
// Taking parts out of the kernel: without the softmax arithmetic 107 us instead of 129, without
// the LDS operand reads 114, without the global -> LDS traffic 103, with nothing but the MFMAs and
// the row-maximum check 67 -- the parts add up almost linearly, i.e. they hardly overlap: the
// chain LDS read -> MFMA -> softmax -> MFMA is dependent, and two wavefronts per SIMD (all that
// two row tiles of accumulators leave room for) do not cover it.
//
// A group is one (unit, split) slot -- split_slot() shares the slots out over the units by
// retrieved size -- and its n_row_blocks workgroups read the same K/V range.  Workgroups go to
// the 8 XCDs round-robin by id and are dispatched in id order, so the 1-D grid is laid out as
// id = 8 * (row block + n_row_blocks * (group / 8)) + group % 8: a group's workgroups share one
// XCD (one L2) and have neighbouring dispatch slots there, which keeps them together in time --
// also when the grid exceeds the chip or several streams' kernels interleave -- so the group's
// K/V is fetched from memory once and found in L2 by the rest.
#include <mutex>

#include "mosaic_internal.h"
#include "attend_mfma_device.h"
#include "attend_reps_device.h"

namespace mosaic {

namespace {

typedef __attribute__((address_space(1))) const void *gptr_t;
typedef __attribute__((address_space(3))) void *lptr_t;
typedef const __attribute__((address_space(4))) int *cint_ptr;

// maximum of three floats in one instruction (no NaNs reach it: logits are finite or -inf)
__device__ __forceinline__ float max3(float a, float b, float c) {
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

// s_waitcnt that waits until at most n vector-memory loads of this wave are outstanding (and for nothing else)
template <int N>
__device__ __forceinline__ void wait_vmem_le() {
    __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}

template <int D, bool AUG, int NW>
__global__ __launch_bounds__(64 * NW, NW == 4 ? 2 : 1) void k_attend_prefill_mfma(DeviceView dv, int u0, int n_units,
                                                                                    const unsigned short *q, int Tq,
                                                                                    int NT, int n_groups, int n_row_blocks,
                                                                                    int group_blocks) {
    static_assert(!AUG || 64 * NW == kBlock, "the representatives' workgroups are written for kBlock threads");
    constexpr int KK = D / 32, DB = D / 16, RTW = kPrefillTiles;
    constexpr int KSEG = D / 8;                  // 16-byte pieces per key row
    constexpr int KRP = 16 / KSEG;               // key rows per 256 bytes (1 at D = 128, 2 at D = 64)
    constexpr int KBYTES = kChunk * D * 2, VBYTES = D * kChunk * 2;
    constexpr int NS = NW;                       // LDS slots per operand
    constexpr int DIST = NS / 2 - 1;             // barrier intervals (of two chunks) between a chunk's loads and its use
    constexpr int KW = KBYTES / 1024, VW = VBYTES / 1024;   // wavefront-sized loads per chunk
    constexpr int LPW = (KW + VW) / NW;          // ... per wave: loads number wave + NW i, keys first
    static_assert(LPW >= 1 && (KW + VW) % NW == 0 && 2 * (DIST - 1) * LPW < 64, "load schedule");
    constexpr int kPending = 2 * (DIST - 1) * LPW;           // loads of a wave that may stay in flight across a barrier
    const int tid = threadIdx.x, wave = tid / 64, lane = tid % 64, g = lane / 16, n = lane % 16;
    if constexpr (AUG) {
        if ((int)blockIdx.x >= group_blocks) {   // extra workgroups: the global representatives' part (augmentation)
            const int idx = (int)blockIdx.x - group_blocks;
            attend_reps_partial<unsigned short, D>(dv, u0, idx / NT, idx % NT, q, Tq);
            return;
        }
    }
    const int xcd = (int)blockIdx.x % 8, seq = (int)blockIdx.x / 8;
    const int grp = (seq / n_row_blocks) * 8 + xcd, yb = seq % n_row_blocks;
    if (grp >= n_groups) return;                   // block-uniform: no barrier reached yet
    const SplitSlot slot = split_slot<false>(dv.n_sel + u0, n_units, n_groups, grp);
    if (slot.uc < 0) return;
    // (wave-uniform values are moved to scalar registers: page ids are then read with scalar loads,
    // which nothing waits for until they are used a page later, and addresses are scalar arithmetic)
    const int uc = __builtin_amdgcn_readfirstlane(slot.uc), u = u0 + uc;
    const int split = __builtin_amdgcn_readfirstlane(slot.split), n_splits = __builtin_amdgcn_readfirstlane(slot.S);
    const int slot_base = __builtin_amdgcn_readfirstlane(slot.base);
    const int T = dv.T, F = dv.F, cpp = dv.chunks_per_page;
    const int lc = uc / dv.Hkv, h = u % dv.Hkv;
    const int tile0 = (yb * NW + wave) * RTW;
    // LDS (dynamic): NS key slots, then NS value slots, one chunk each
    extern __shared__ __attribute__((aligned(1024))) unsigned char prefill_lds[];

    bf16x8 qf[RTW][KK];
#pragma unroll
    for (int r = 0; r < RTW; ++r) load_q<D>(dv, q, lc, h, Tq, (tile0 + r) * kRowTile + n, g, qf[r]);

    // the page list was written by an earlier launch and is read-only here: constant address space, so
    // that a wave-uniform read of it is a scalar load
    const cint_ptr sel = (cint_ptr)(dv.sel_pages + (size_t)u * F);
    const int NC = __builtin_amdgcn_readfirstlane(slot.n) * cpp;
    const int cps = (NC + n_splits - 1) / n_splits;
    const int c0 = __builtin_amdgcn_readfirstlane(split * cps);
    const int c1 = __builtin_amdgcn_readfirstlane(min(NC, c0 + cps));
    const float sl2 = 1.4426950408889634f / sqrtf((float)D);

    f32x4 acc[RTW][DB], l[RTW];                    // l: row sums, kept by an all-ones MFMA
    float m[RTW], lx[RTW], bar[RTW];               // bar: a raw logit above it raises the row's reference m
#pragma unroll
    for (int r = 0; r < RTW; ++r) {
        m[r] = -INFINITY; bar[r] = -INFINITY; l[r] = f32x4{0.f, 0.f, 0.f, 0.f}; lx[r] = 0.f;
#pragma unroll
        for (int db = 0; db < DB; ++db) acc[r][db] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    // What this lane fetches of every chunk (fixed for the kernel's life).  Load i of the wave is
    // wavefront-load number wave + NW i of the chunk: numbers below KW cover the key block, the
    // rest the value block; a load covers LDS pieces 64 * number + lane of its block.
    constexpr bool kWhole = KW % NW == 0;          // every wave loads keys and values (else LPW = 1: one or the other)
    static_assert(kWhole || LPW == 1, "load schedule");
    auto is_key = [&](int i) { return kWhole ? i < KW / NW : wave < KW; };
    int ld_tok[LPW], ld_off[LPW], ld_koff[LPW], ld_dst[LPW];   // token within the chunk (keys); element offset (in the row / in the chunk); LDS byte offset in the slot
#pragma unroll
    for (int i = 0; i < LPW; ++i) {
        const int num = wave + NW * i;
        if (is_key(i)) {                           // wave-uniform
            const int P = num * 64 + lane, row = P / KSEG, phys = P % KSEG;
            const int seg = phys ^ ((row / KRP) % KSEG);
            const int tau = row / 16, rem = row % 16;
            ld_tok[i] = 8 * (rem / 4) + 4 * tau + rem % 4;
            ld_off[i] = seg * 8;
            ld_koff[i] = ld_tok[i] * D + seg * 8;
            ld_dst[i] = num * 1024;
        } else {
            const int P = (num - KW) * 64 + lane, row = P / 4, phys = P % 4;
            ld_tok[i] = 0; ld_koff[i] = 0;
            ld_off[i] = row * kChunk + (phys ^ ((row / 4) % 4)) * 8;
            ld_dst[i] = (num - KW) * 1024;
        }
    }
    // ... and where it reads its operands: key rows 16 tau + n, pieces 4 kk + g; value rows 16 db + n, piece g
    int kr_off[KK];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) kr_off[kk] = n * (D * 2) + (((4 * kk + g) ^ ((n / KRP) % KSEG)) * 16);
    const int vr_off = n * (kChunk * 2) + ((g ^ ((n / 4) % 4)) * 16);

    // Chunks are fetched in order by two cursors (keys run one chunk ahead of values, see below).  A cursor
    // (chunk nf = chunk cc of the pi-th selected page) advances by increments, page addresses are worked
    // out once per page, and the id of the page after the current one is read (a scalar load) a whole
    // page ahead, so no fetch waits on a dependent load or divides.  Past the end a cursor stays on the
    // last chunk: such loads re-read valid memory, land in slots nobody reads, and keep the number of
    // loads per barrier interval constant, which is what the partial waits count on.
    struct Cursor { int nf, pi, cc, pg_next, slot; const unsigned short *p; };
    const int cl = c1 - 1, n_pages = NC / cpp;
    const char *const kbase = dv.k_store + (size_t)u * dv.k_ustride;
    const char *const vbase = dv.v_store + (size_t)u * dv.v_ustride;
    auto page_ptr = [&](const char *base, size_t psize, int page) {
        return reinterpret_cast<const unsigned short *>(base + (size_t)page * psize);
    };
    auto start = [&](Cursor &cu, const char *base, size_t psize) {
        cu.nf = c0; cu.pi = c0 / cpp; cu.cc = c0 - cu.pi * cpp; cu.pg_next = 0; cu.slot = 0; cu.p = nullptr;
        if (c0 < c1) {
            cu.p = page_ptr(base, psize, sel[cu.pi]);
            cu.pg_next = sel[min(cu.pi + 1, n_pages - 1)];
        }
    };
    auto advance = [&](Cursor &cu, const char *base, size_t psize) {      // wave-uniform
        cu.slot = (cu.slot + 1) & (NS - 1);
        if (cu.nf < cl) {
            ++cu.nf;
            if (++cu.cc == cpp) {
                cu.cc = 0; ++cu.pi;
                cu.p = page_ptr(base, psize, cu.pg_next);
                cu.pg_next = sel[min(cu.pi + 1, n_pages - 1)];
            }
        }
    };
    Cursor kc, vc;
    start(kc, kbase, dv.kpage);
    start(vc, vbase, dv.vpage);
    // this wave's loads of the key cursor's chunk (into the cursor's key slot), then the cursor moves on
    auto fetch_k = [&]() {
        const int t0 = kc.cc * kChunk;
        unsigned char *const dst = prefill_lds + kc.slot * KBYTES;
        // (scalar base, 32-bit lane offset: the chunk's first token goes into the base, and only a page's
        // ragged last chunk clamps token numbers)
        const unsigned short *const kp = kc.p + (size_t)t0 * D;
        const bool whole = t0 + kChunk <= T;           // wave-uniform
#pragma unroll
        for (int i = 0; i < LPW; ++i)
            if (is_key(i)) {
                const unsigned off = whole ? (unsigned)ld_koff[i] : (unsigned)((min(t0 + ld_tok[i], T - 1) - t0) * D + ld_off[i]);
                __builtin_amdgcn_global_load_lds((gptr_t)(kp + off), (lptr_t)(dst + ld_dst[i]), 16, 0, 0);
            }
        advance(kc, kbase, dv.kpage);
    };
    auto fetch_v = [&]() {
        const unsigned short *vp = vc.p + (size_t)vc.cc * D * kChunk;
        unsigned char *const dst = prefill_lds + NS * KBYTES + vc.slot * VBYTES;
#pragma unroll
        for (int i = 0; i < LPW; ++i)
            if (!is_key(i))
                __builtin_amdgcn_global_load_lds((gptr_t)(vp + (unsigned)ld_off[i]), (lptr_t)(dst + ld_dst[i]), 16, 0, 0);
        advance(vc, vbase, dv.vpage);
    };
    // The loads are issued as the sequence K0 | V0 K1 | V1 K2 | V2 K3 | ...: a wave issues LPW loads per
    // pair (V c, K c+1).  A barrier interval needs everything up to its second chunk's pair and may leave
    // the 2 (DIST - 1) younger pairs in flight; then the workgroup meets.
    auto publish = [&]() {
        wait_vmem_le<kPending>();
        lds_barrier();          // (a full __syncthreads() would wait for the younger pairs as well)
    };
    auto ldk = [&](int s, bf16x8 (&kf)[2 * KK]) {
        const unsigned char *const kb = prefill_lds + s * KBYTES;
#pragma unroll
        for (int tau = 0; tau < 2; ++tau)
#pragma unroll
            for (int kk = 0; kk < KK; ++kk)
                kf[tau * KK + kk] = __builtin_bit_cast(
                    bf16x8, *reinterpret_cast<const uint4 *>(kb + tau * 16 * D * 2 + kr_off[kk]));
    };
    auto ldv = [&](int s, bf16x8 (&vf)[DB]) {
        const unsigned char *const vb = prefill_lds + NS * KBYTES + s * VBYTES;
#pragma unroll
        for (int db = 0; db < DB; ++db)
            vf[db] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(vb + db * 16 * kChunk * 2 + vr_off));
    };

    // ---- the pipeline -------------------------------------------------------------------------
    // A UNIT is (chunk j, row tile r), x = 2 j + r.  Per unit: Q(x) = 2 KK logit MFMAs, SM(x) = the
    // softmax arithmetic on the vector ALU, P(x) = 1 + DB output MFMAs.  Inside a wavefront the
    // matrix pipe and the vector ALU only overlap when independent MFMA and VALU instructions
    // alternate in the instruction stream, so the loop is software-pipelined: the logits of a
    // chunk are formed one step before their softmax, and step j runs
    //     check(2j);      Q(2j + 2)         || SM(2j)
    //     check(2j + 1);  Q(2j + 3), P(2j)  || SM(2j + 1)
    //                     P(2j + 1)
    // where check(x) is the maximum of the unit's logits against the row's lazy reference (rarely
    // a mask of a ragged chunk or a rescale -- the only branches, kept outside the groups so that
    // each group is one scheduling region).  check(x) follows P(x - 2), the previous unit of the
    // same row tile, so a rescale sees every earlier contribution of its rows.
    // Step j needs K(j + 1) and V(j) in LDS.  Two steps per barrier interval.
    static_assert(RTW == 2, "the pipeline below alternates two row tiles");
    f32x4 S[RTW][2], S2[RTW][2];                     // logits of the two units waiting for their softmax (two buffers, used in turn)
    const bf16x8 ones = __builtin_bit_cast(bf16x8, make_uint4(0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u));
    int c_cc = c0 - (c0 / cpp) * cpp;                // chunk inside its page, of the chunk whose softmax is next
    const int n_chunks = c1 - c0;

    auto logits = [&](const bf16x8 (&kf)[2 * KK], int r, f32x4 (&s)[2]) {
#pragma unroll
        for (int tau = 0; tau < 2; ++tau) s[tau] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < KK; ++kk)
#pragma unroll
            for (int tau = 0; tau < 2; ++tau)
                s[tau] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[tau * KK + kk], qf[r][kk], s[tau], 0, 0, 0);
    };
    auto output = [&](const bf16x8 (&vf)[DB], bf16x8 pf, int r) {
        l[r] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, pf, l[r], 0, 0, 0);
#pragma unroll
        for (int db = 0; db < DB; ++db)
            acc[r][db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[db], pf, acc[r][db], 0, 0, 0);
    };
    auto check = [&](int r, f32x4 (&s)[2], int n_valid) {
        if (n_valid < kChunk) {             // ragged last chunk of a page, or a step past the end (wave-uniform)
#pragma unroll
            for (int j = 0; j < 8; ++j)
                if (8 * g + j >= n_valid) s[j / 4][j % 4] = -INFINITY;
        }
        // (three-operand maxima written out: the compiler's own fmaxf chain quiets every MFMA result first,
        // six more instructions per unit; the raw maximum is compared with the row's bar (m + kLazy) / sl2,
        // kept up to date by the rare branch, so the common path has no scaling)
        float cm = max3(s[0][0], s[0][1], s[0][2]);
        cm = max3(cm, s[0][3], s[1][0]);
        cm = max3(cm, s[1][1], s[1][2]);
        cm = max3(cm, s[1][3], s[1][3]);
        if (__builtin_amdgcn_ballot_w64(cm > bar[r])) {   // rare, wave-uniform
            cm = cm * sl2;
            cm = fmaxf(cm, __shfl_xor(cm, 16, 64));
            cm = fmaxf(cm, __shfl_xor(cm, 32, 64));
            const float mnew = fmaxf(m[r], cm);
            const float alpha = __builtin_amdgcn_exp2f(m[r] - mnew);
            l[r] = l[r] * alpha;
            lx[r] = lx[r] * alpha;
            m[r] = mnew;
            bar[r] = (mnew + kLazy) / sl2;
#pragma unroll
            for (int db = 0; db < DB; ++db) acc[r][db] = acc[r][db] * alpha;
        }
    };
    auto softmax = [&](int r, const f32x4 (&s)[2]) -> bf16x8 {
        const float nm = -m[r];
        unsigned int pw[4];
        float xs = 0.f;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[(2 * j) / 4][(2 * j) % 4], sl2, nm));
            const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[(2 * j + 1) / 4][(2 * j + 1) % 4], sl2, nm));
            pw[j] = pack_bf16(p0, p1);
            xs += p0 + p1;
        }
        lx[r] += xs;
        return __builtin_bit_cast(bf16x8, make_uint4(pw[0], pw[1], pw[2], pw[3]));
    };
// one MFMA, then two vector-ALU instructions, ... : the order the scheduler is asked for inside a group
#define MOSAIC_ALTERNATE_1()  __builtin_amdgcn_sched_group_barrier(0x008, 1, 0); __builtin_amdgcn_sched_group_barrier(0x002, 2, 0);
#define MOSAIC_ALTERNATE_4()  MOSAIC_ALTERNATE_1() MOSAIC_ALTERNATE_1() MOSAIC_ALTERNATE_1() MOSAIC_ALTERNATE_1()
#define MOSAIC_ALTERNATE_17() MOSAIC_ALTERNATE_4() MOSAIC_ALTERNATE_4() MOSAIC_ALTERNATE_4() MOSAIC_ALTERNATE_4() MOSAIC_ALTERNATE_1()
    // step j: key slot sk holds K(j + 1), value slot sv holds V(j); n_valid = tokens of chunk j (0 past the end)
    auto step = [&](int sk, int sv, int n_valid, f32x4 (&S)[RTW][2], f32x4 (&Sn)[RTW][2]) {   // consumes S, leaves the next chunk's logits in Sn
        bf16x8 kf[2 * KK], vf[DB];
        ldk(sk, kf);
        check(0, S[0], n_valid);
        __builtin_amdgcn_sched_barrier(0);
        // Q(2j + 2) || SM(2j)
        ldv(sv, vf);
        logits(kf, 0, Sn[0]);
        const bf16x8 pf0 = softmax(0, S[0]);
        MOSAIC_ALTERNATE_4() MOSAIC_ALTERNATE_4()
        __builtin_amdgcn_sched_barrier(0);
        check(1, S[1], n_valid);
        __builtin_amdgcn_sched_barrier(0);
        // Q(2j + 3), P(2j) || SM(2j + 1)
        output(vf, pf0, 0);
        logits(kf, 1, Sn[1]);
        const bf16x8 pf1 = softmax(1, S[1]);
        MOSAIC_ALTERNATE_17()
        __builtin_amdgcn_sched_barrier(0);
        // P(2j + 1)
        output(vf, pf1, 1);
    };
    auto next_valid = [&](int j) {                    // tokens of chunk j that exist; advances the in-page cursor
        const int nv = j < n_chunks ? min(kChunk, T - c_cc * kChunk) : 0;
        c_cc = c_cc + 1 == cpp ? 0 : c_cc + 1;
        return nv;
    };

    if (c0 < c1) {
        fetch_k();                                    // K0 | V0 K1 | V1 K2 | ... | V(2 DIST - 1) K(2 DIST)
#pragma unroll
        for (int i = 0; i < 2 * DIST; ++i) { fetch_v(); fetch_k(); }
        publish();                                    // K0, K1, K2, V0, V1 are in LDS
        {   // Q(0), Q(1): the first chunk's logits
            bf16x8 kf[2 * KK];
            ldk(0, kf);
            logits(kf, 0, S[0]);
            logits(kf, 1, S[1]);
        }
        __syncthreads();                              // (key slot 0 is written again from the first interval on)
        for (int j = 0; j < n_chunks; j += 2) {       // barrier interval of steps j, j + 1
            fetch_v(); fetch_k();                     // V(j + 2 DIST), K(j + 2 DIST + 1): slots last read one interval ago
            fetch_v(); fetch_k();
            step((j + 1) & (NS - 1), j & (NS - 1), next_valid(j), S, S2);
            step((j + 2) & (NS - 1), (j + 1) & (NS - 1), next_valid(j + 1), S2, S);
            publish();
        }
    }
#undef MOSAIC_ALTERNATE_17
#undef MOSAIC_ALTERNATE_4
#undef MOSAIC_ALTERNATE_1
#pragma unroll
    for (int r = 0; r < RTW; ++r) {
        const int tile = tile0 + r;
        if (tile >= NT) break;
        const float lr = l[r][0];
        float xr = lx[r];                              // this lane's 8 tokens per chunk: add the four lane groups
        xr += __shfl_xor(xr, 16, 64);
        xr += __shfl_xor(xr, 32, 64);
        const size_t entry = (size_t)slot_base * NT + (size_t)tile * n_splits + split;
        float *po = dv.part_o + (entry * kRowTile + n) * D;
#pragma unroll
        for (int db = 0; db < DB; ++db)
            *reinterpret_cast<float4 *>(po + 16 * db + 4 * g) =
                make_float4(acc[r][db][0], acc[r][db][1], acc[r][db][2], acc[r][db][3]);
        if (g == 0) {
            dv.part_ml[entry * kMlRows * kRowTile + n] = m[r];
            dv.part_ml[entry * kMlRows * kRowTile + kRowTile + n] = lr;
            dv.part_ml[entry * kMlRows * kRowTile + 2 * kRowTile + n] = xr;
        }
    }
}

} // namespace

hipError_t launch_attend_prefill(const DeviceView &dv, int u0, int n_units, const unsigned short *q, int Tq,
                                 int n_splits, hipStream_t s, hipEvent_t ev0, hipEvent_t ev1) {
    constexpr int NW = kPrefillWaves;
    const int NT = (Tq * dv.G + kRowTile - 1) / kRowTile;
    // dynamic LDS: NW key slots and NW value slots of one chunk (32 x D bf16) each
    const size_t lds = (size_t)2 * NW * (kChunk * dv.D * 2);
    static std::once_flag attr_once;          // process-wide, but set exactly once whichever handle comes first
    std::call_once(attr_once, [] {
        const int big = 2 * NW * kChunk * 128 * 2;
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(&k_attend_prefill_mfma<64, true, NW>), hipFuncAttributeMaxDynamicSharedMemorySize, big);
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(&k_attend_prefill_mfma<64, false, NW>), hipFuncAttributeMaxDynamicSharedMemorySize, big);
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(&k_attend_prefill_mfma<128, true, NW>), hipFuncAttributeMaxDynamicSharedMemorySize, big);
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(&k_attend_prefill_mfma<128, false, NW>), hipFuncAttributeMaxDynamicSharedMemorySize, big);
    });
    const int n_groups = n_units * n_splits, rb = (NT + NW * kPrefillTiles - 1) / (NW * kPrefillTiles);
    const int gb = (n_groups + 7) / 8 * 8 * rb;
    const dim3 grid(gb + (dv.aug_reps ? n_units * NT : 0)), block(64 * NW);
    auto go = [&](auto kern) { launch_timed(kern, grid, block, lds, s, ev0, ev1, dv, u0, n_units, q, Tq, NT, n_groups, rb, gb); };
    if (dv.aug_reps) { if (dv.D == 64) go(k_attend_prefill_mfma<64, true, NW>); else go(k_attend_prefill_mfma<128, true, NW>); }
    else { if (dv.D == 64) go(k_attend_prefill_mfma<64, false, NW>); else go(k_attend_prefill_mfma<128, false, NW>); }
    return hipGetLastError();
}

} // namespace mosaic
