// Exact top-k ranking of up to 1024 scored representatives by one 1024-thread
// workgroup (paper Sec. V-C / VII-B: the top-K clusters by query relevance).
//
// Order: score descending, id ascending; only live entries (n_sh[j] > 0) take
// part.  Result: rank_sh[j] = rank of entry j if it is live and among the k
// best, else -1; ids_sh[rank] = j for those; the return value (same in every
// thread) is the number of live entries.
//
// Counting, for every entry, how many entries beat it costs R^2 fp64
// comparisons, which dominates a query once R reaches a few hundred.  Only the
// k best ranks are needed, so the entries are first binned by a monotone map of
// their score onto 1024 bins; a suffix count over the bins gives the highest
// bin b* from which on at least k entries lie, and only the entries in bins
// >= b* (k of them plus the rest of one bin) are ranked exactly against each
// other.  Every entry outside outranks none of them (its bin is lower, the map
// is monotone), so their mutual ranks are their global ranks: the result is the
// same as that of the full comparison, whatever the score distribution (if all
// scores fall into one bin the candidates are simply all live entries).
#pragma once
#include <hip/hip_runtime.h>

namespace mosaic {

constexpr int kTopkBins = 1024;

struct TopkShared {
    int hist[kTopkBins];
    double red_min[16], red_max[16];
    int wave_tot[16];
    int bstar, n_live, n_cand;
};

// cnt_sh, cand_sh: 1024 ints of scratch each (contents destroyed).  R <= 1024.
// All 1024 threads of the workgroup must call it; it contains barriers.
// Precondition (saves a barrier on the small-table path): cnt_sh[0..R) and
// sh.n_live were set to zero by the caller before its latest barrier.
__device__ __forceinline__ int topk_rank(const double *sc_sh, const int *n_sh, int R, int k,
                                         int *rank_sh, int *ids_sh, int *cnt_sh, int *cand_sh,
                                         TopkShared &sh) {
    constexpr int BLK = 1024;
    const int tid = threadIdx.x, wave = tid / 64, lane = tid % 64;
    const bool live = tid < R && n_sh[tid] > 0;
    const double s = live ? sc_sh[tid] : 0.0;
    if (R <= 128) {
        // Small tables: the direct count over all pairs, 2^pl threads per entry (the largest power of
        // two that fits the workgroup: shifts instead of integer divisions).  The pairs are compared
        // on fp32 roundings of the scores (rounding is monotone, so a strict fp32 order is the fp64
        // order; fp64 compares run at a quarter of the rate and were what this count waited for);
        // an entry whose rounding collides with another one's is settled exactly afterwards.
        float *key_sh = reinterpret_cast<float *>(cand_sh);
        if (tid < R) key_sh[tid] = live ? (float)s : -INFINITY;
        __syncthreads();
        const int pl = 31 - __clz(BLK / R);
        const int j = tid >> pl, part = tid & ((1 << pl) - 1);
        if (j < R && n_sh[j] > 0) {
            const float fj = key_sh[j];
            const int i0 = (R * part) >> pl, i1 = (R * (part + 1)) >> pl;
            int c = 0, ceq = 0;  // (an entry that is not live carries -inf and neither outranks nor equals a live one)
#pragma unroll 8
            for (int i = i0; i < i1; ++i) {
                const float fi = key_sh[i];
                c += fi > fj;
                ceq += fi == fj;
            }
            atomicAdd(&cnt_sh[j], c + (ceq << 16));     // c <= 128, ceq <= 128
        }
        __syncthreads();
        int rk = -1;
        if (live) {
            const int v = cnt_sh[tid];
            rk = v & 0xffff;
            if ((v >> 16) > 1) {                        // collisions (the entry itself counts once): exact order among them
                const float fj = key_sh[tid];
                for (int i = 0; i < R; ++i) {
                    if (i == tid || key_sh[i] != fj) continue;
                    const double si = sc_sh[i];
                    rk += (si > s) || (si == s && i < tid);
                }
            }
            if (rk < k) ids_sh[rk] = tid; else rk = -1;
        }
        if (tid < R) rank_sh[tid] = rk;
        // live entries: one LDS atomic per wavefront (64 lanes adding to one word serialize)
        const unsigned long long lb = __ballot(live);
        if (lane == 0 && lb) atomicAdd(&sh.n_live, __popcll(lb));
        __syncthreads();
        return sh.n_live;
    }
    // ---- score range of the live entries ----
    double mn = live ? s : INFINITY, mx = live ? s : -INFINITY;
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
        mn = fmin(mn, __shfl_xor(mn, o, 64));
        mx = fmax(mx, __shfl_xor(mx, o, 64));
    }
    if (lane == 0) { sh.red_min[wave] = mn; sh.red_max[wave] = mx; }
    sh.hist[tid] = 0;
    cnt_sh[tid] = 0;
    if (tid == 0) sh.n_cand = 0;
    __syncthreads();
#pragma unroll
    for (int w = 0; w < 16; ++w) { mn = fmin(mn, sh.red_min[w]); mx = fmax(mx, sh.red_max[w]); }
    // ---- monotone binning ----
    int bin = 0;
    if (live && mx > mn) {
        bin = (int)((s - mn) / (mx - mn) * (double)(kTopkBins - 1));
        bin = min(max(bin, 0), kTopkBins - 1);
    }
    if (live) atomicAdd(&sh.hist[bin], 1);
    __syncthreads();
    // ---- suffix counts over the bins: thread t looks at bin 1023 - t ----
    const int hv = sh.hist[kTopkBins - 1 - tid];
    int incl = hv;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int t = __shfl_up(incl, o, 64);
        if (lane >= o) incl += t;
    }
    if (lane == 63) sh.wave_tot[wave] = incl;
    __syncthreads();
    int before = 0, total = 0;
#pragma unroll
    for (int w = 0; w < 16; ++w) {
        const int t = sh.wave_tot[w];
        before += w < wave ? t : 0;
        total += t;
    }
    incl += before;                          // entries in bins >= 1023 - tid
    if (incl >= k && incl - hv < k) sh.bstar = kTopkBins - 1 - tid;     // exactly one thread if total >= k
    if (tid == 0 && total < k) sh.bstar = 0;
    __syncthreads();
    // ---- candidates: everything from bin b* upwards ----
    const bool cand = live && bin >= sh.bstar;
    {   // compaction with one LDS atomic per wavefront
        const unsigned long long cb = __ballot(cand);
        int base = 0;
        if (lane == 0 && cb) base = atomicAdd(&sh.n_cand, __popcll(cb));
        base = __shfl(base, 0, 64);
        if (cand) cand_sh[base + __popcll(cb & ((1ull << lane) - 1ull))] = tid;
    }
    __syncthreads();
    const int M = sh.n_cand;
    // ---- exact ranks among the candidates, `per` threads per candidate ----
    const int per = M > 0 ? max(1, BLK / M) : 1;
    for (int item = tid; item < M * per; item += BLK) {
        const int a = item / per, part = item - a * per;
        const int j = cand_sh[a];
        const double sj = sc_sh[j];
        const int i0 = (M * part) / per, i1 = (M * (part + 1)) / per;
        int c = 0;
#pragma unroll 4
        for (int x = i0; x < i1; ++x) {
            const int i = cand_sh[x];
            const double si = sc_sh[i];
            c += (si > sj) || (si == sj && i < j);
        }
        if (c) atomicAdd(&cnt_sh[j], c);
    }
    __syncthreads();
    int rk = -1;
    if (cand) {
        rk = cnt_sh[tid];
        if (rk < k) ids_sh[rk] = tid; else rk = -1;
    }
    if (tid < R) rank_sh[tid] = rk;
    __syncthreads();
    return total;
}

} // namespace mosaic
