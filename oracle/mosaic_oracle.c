/*
 * CPU oracle for the cluster-driven KV-cache hot path (test infrastructure).
 *
 * Plain, slow, fp64, one (layer, KV head) "unit" at a time.  It exists only to
 * check the HIP library and to be timed beside it as a baseline; the product
 * never calls it.  It shares no code with the HIP sources.
 *
 * Every function follows one passage of the paper; where the paper is silent
 * the reading taken is stated at the function.  Nothing is blocked, fused or
 * reordered beyond what the passage states.
 *
 * Parity pins (tests marked "not gpu"): summary vs numpy mean; online centroid
 * vs the batch mean of Eq. 1; assignment and Lloyd steps vs exhaustive search;
 * selection vs a full lexicographic sort; gather invariants (whole clusters,
 * partition); attention vs dense softmax attention when k covers all clusters.
 * The self-adaptive maintainer (Sec. VI) is pinned by a hand-worked Eq. 3/4
 * fixture, closed forms of Eq. 5, Eq. 2 against numpy, Split against a numpy
 * two-means, equality with the plain online rule when the threshold is out of
 * reach, and the state transitions of Alg. 1 (buffered singletons, their
 * visibility to retrieval, materialization on retrieval, conservation); the
 * readings inside Alg. 1 by a hand-worked fixture whose verdict flips between
 * tau(|C|) and tau(|C| + 1) (the size before the insertion enters Eq. 5),
 * Eq. 3 / Eq. 4 in numpy on the owner of a buffered state (statistics move,
 * size does not), singleton scores in both score modes against numpy, and
 * reset + re-ingest against a fresh unit.
 * The nested visual-semantic hierarchy (Sec. V-B) and two-stage retrieval
 * (Sec. V-C) are pinned by the special cases P = 1 and top_p = P (both must
 * be the flat path), the nesting invariant, seeds read back after zero
 * K-means rounds, a per-partition brute-force K-means, a numpy argmax over the
 * partition's clusters only, and a whole-array numpy two-stage selection.
 * End-to-end retrieval *quality* has no value in the paper to pin it to:
 * parity unpinned for that quantity only (it is reported, never gated).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    int C, D, T, max_frames, warmup, lloyd_iters, recluster_every, score_mode;
    int n_frames;          /* frames ingested so far */
    int ready;             /* 1 once the initial clustering has run */
    double *summ;          /* [max_frames][D] per-frame key summaries */
    double *r;             /* [C][D] cluster representatives (Eq. 1 / Eq. 3) */
    int *n;                /* [C] cluster sizes in frames */
    int *assign;           /* [max_frames] frame -> cluster, -1 while buffered */
    double lloyd_min_gap;  /* smallest winner/runner-up relative gap seen in
                              the latest Lloyd run (diagnostic only) */
    int n_lloyd_runs;
    /* self-adaptive maintenance (Sec. VI); maint_mode 0 = off */
    int warmup_arg;        /* warm-up length as passed (0 = default) */
    int n_slots;           /* cluster ids in use: [0, n_slots); C when off */
    int c_init;            /* clusters the initial K-means builds (maintenance on) */
    int maint_mode;        /* 1 = split at once, 2 = deferred split (Alg. 1) */
    double tau_min, tau_max, n0;   /* Eq. 5 */
    int split_iters, buf_max;
    double *var;           /* [C] running intra-cluster variance (Eq. 2 / Eq. 4) */
    int *lazy;             /* [C] lazy-split flag */
    int *resident;         /* [C] 1 = the cluster's contents are on the GPU */
    int resident_external; /* 1 = the caller says what is on the GPU (a cache model); retrieval leaves the flags alone */
    int *buf_frame, *buf_owner;    /* GPU-side buffer of singletons: frame, owning cluster */
    int n_buf;
    long n_split_now, n_split_deferred, n_deferred, n_forced_absorb;
    int last_action;       /* what the latest online insertion did (ORC_ACT_*) */
    double last_var, last_tau;     /* the two sides of its threshold test */
    double split_min_gap;  /* smallest relative gap of any comparison inside the
                              latest Split (diagnostic only) */
    /* nested visual-semantic hierarchy (Sec. V-B); n_part 0 = flat */
    int n_part;            /* visual partitions P; cluster ids [p*Cs, (p+1)*Cs) belong to partition p */
    int Cs;                /* semantic clusters per partition, C / P */
    int *part;             /* [max_frames] frame -> visual partition */
} orc_unit;

enum { ORC_ACT_NONE = 0, ORC_ACT_ABSORB = 1, ORC_ACT_SPLIT = 2, ORC_ACT_DEFER = 3,
       ORC_ACT_FORCED_ABSORB = 4 };

typedef struct {
    int winner;     /* chosen cluster */
    int runner_up;  /* second best, -1 if there is none */
    double gap;     /* |a-b| / max(|a|,|b|,1e-30) of their similarities */
    double sim;     /* similarity of the winner */
} orc_decision;

void orc_unit_score(const orc_unit *u, const double *qbar, double *score);
int orc_select(const double *score, const int *n, int C, int k, int *ids, double *gap_k);
int orc_unit_ingest(orc_unit *u, const double *k_frame, int force, orc_decision *dec);
void orc_summary(const double *k_frame, int T, int D, double *s);

static double rel_gap(double a, double b)
{
    double m = fmax(fmax(fabs(a), fabs(b)), 1e-30);
    return fabs(a - b) / m;
}

static double dot(const double *a, const double *b, int D)
{
    double s = 0.0;
    for (int d = 0; d < D; ++d) s += a[d] * b[d];
    return s;
}

/* Cosine similarity (Sec. V-B, "Clustering Criterion").  A zero vector has no
 * direction: its similarity to anything is taken as 0. */
static double cosine(const double *a, const double *b, int D)
{
    double na = sqrt(dot(a, a, D)), nb = sqrt(dot(b, b, D));
    if (na == 0.0 || nb == 0.0) return 0.0;
    return dot(a, b, D) / (na * nb);
}

orc_unit *orc_unit_new(int C, int D, int T, int max_frames, int warmup,
                       int lloyd_iters, int recluster_every, int score_mode)
{
    orc_unit *u = (orc_unit *)calloc(1, sizeof(orc_unit));
    u->C = C; u->D = D; u->T = T; u->max_frames = max_frames;
    u->warmup = warmup > 0 ? warmup : 2 * C;
    u->warmup_arg = warmup; u->n_slots = C; u->split_min_gap = INFINITY;
    u->lloyd_iters = lloyd_iters; u->recluster_every = recluster_every;
    u->score_mode = score_mode;
    u->summ = (double *)calloc((size_t)max_frames * D, sizeof(double));
    u->r = (double *)calloc((size_t)C * D, sizeof(double));
    u->n = (int *)calloc((size_t)C, sizeof(int));
    u->assign = (int *)malloc((size_t)max_frames * sizeof(int));
    for (int f = 0; f < max_frames; ++f) u->assign[f] = -1;
    u->lloyd_min_gap = INFINITY;
    return u;
}

void orc_unit_free(orc_unit *u)
{
    if (!u) return;
    free(u->summ); free(u->r); free(u->n); free(u->assign);
    free(u->var); free(u->lazy); free(u->resident); free(u->buf_frame); free(u->buf_owner);
    free(u->part);
    free(u);
}

void orc_unit_reset(orc_unit *u)
{
    u->n_frames = 0; u->ready = 0; u->n_lloyd_runs = 0;
    u->lloyd_min_gap = INFINITY;
    memset(u->r, 0, (size_t)u->C * u->D * sizeof(double));
    memset(u->n, 0, (size_t)u->C * sizeof(int));
    for (int f = 0; f < u->max_frames; ++f) u->assign[f] = -1;
    if (u->n_part > 0)
        for (int f = 0; f < u->max_frames; ++f) u->part[f] = -1;
    if (u->maint_mode) {
        memset(u->var, 0, (size_t)u->C * sizeof(double));
        memset(u->lazy, 0, (size_t)u->C * sizeof(int));
        memset(u->resident, 0, (size_t)u->C * sizeof(int));
        u->n_buf = 0; u->n_slots = u->c_init;
        u->n_split_now = u->n_split_deferred = u->n_deferred = u->n_forced_absorb = 0;
        u->last_action = ORC_ACT_NONE; u->split_min_gap = INFINITY;
    }
}

/* The unit that is clustered is the frame: its "KV state" (Sec. VI-A) is the
 * mean of the frame's T key vectors.  k_frame is [T][D]. */
void orc_summary(const double *k_frame, int T, int D, double *s)
{
    for (int d = 0; d < D; ++d) {
        double acc = 0.0;
        for (int t = 0; t < T; ++t) acc += k_frame[(size_t)t * D + d];
        s[d] = acc / (double)T;
    }
}

/* Greedy rule of Sec. VI-A: the cluster whose representative is most similar
 * (cosine, Sec. V-B) among the non-empty ones; equal similarities go to the
 * lowest cluster id.  `all_live` treats every cluster as non-empty (first
 * Lloyd iteration from seeds). */
static void nearest_in(const orc_unit *u, const double *s, int all_live,
                       int lo, int hi, orc_decision *dec)
{
    int best = -1, second = -1;
    double bs = -INFINITY, ss = -INFINITY;
    for (int j = lo; j < hi; ++j) {
        if (!all_live && u->n[j] == 0) continue;
        double c = cosine(s, u->r + (size_t)j * u->D, u->D);
        if (best < 0 || c > bs) { second = best; ss = bs; best = j; bs = c; }
        else if (second < 0 || c > ss) { second = j; ss = c; }
    }
    if (best < 0) { best = lo; bs = 0.0; }     /* no live cluster at all */
    dec->winner = best; dec->runner_up = second; dec->sim = bs;
    dec->gap = second >= 0 ? rel_gap(bs, ss) : INFINITY;
}

/* Candidates of frame f: all cluster ids in use, or -- under the nested
 * hierarchy (Sec. V-B "Nested Hierarchy": a new state is compared only with
 * the clusters of its own visual partition) -- the ids of partition part[f]. */
static void nearest(const orc_unit *u, int f, const double *s, int all_live,
                    orc_decision *dec)
{
    if (u->n_part > 0) {
        const int p = u->part[f];
        nearest_in(u, s, all_live, p * u->Cs, (p + 1) * u->Cs, dec);
    } else {
        nearest_in(u, s, all_live, 0, u->n_slots, dec);
    }
}

/* Modified K-means of Sec. V-B: `iters` rounds of (assign every stored summary
 * by the greedy cosine rule, then set each representative to the mean of its
 * members, Eq. 1).  A cluster left without members keeps its previous
 * representative and is skipped by later assignments.  Members are summed in
 * ascending frame order. */
static void lloyd(orc_unit *u, int first_all_live)
{
    const int F = u->n_frames, C = u->n_slots, D = u->D;
    u->lloyd_min_gap = INFINITY;
    for (int it = 0; it < u->lloyd_iters; ++it) {
        int all_live = first_all_live && it == 0;
        for (int f = 0; f < F; ++f) {
            orc_decision dec;
            nearest(u, f, u->summ + (size_t)f * D, all_live, &dec);
            u->assign[f] = dec.winner;
            if (dec.gap < u->lloyd_min_gap) u->lloyd_min_gap = dec.gap;
        }
        for (int j = 0; j < C; ++j) {
            int cnt = 0;
            for (int f = 0; f < F; ++f) cnt += (u->assign[f] == j);
            u->n[j] = cnt;
            if (cnt == 0) continue;
            double *rj = u->r + (size_t)j * D;
            for (int d = 0; d < D; ++d) {
                double acc = 0.0;
                for (int f = 0; f < F; ++f)
                    if (u->assign[f] == j) acc += u->summ[(size_t)f * D + d];
                rj[d] = acc / (double)cnt;
            }
        }
    }
    u->n_lloyd_runs += 1;
}

/* ------------------------------------------------------------------------
 * Self-Adaptive Maintainer (Sec. VI).
 * ------------------------------------------------------------------------ */

/* Switch the maintainer on; call before the first frame.  c_init clusters are
 * built by the initial K-means (default warm-up 2*c_init frames) and splits
 * add clusters up to the table size C.  mode 1 treats every cluster as GPU
 * resident (every invalid cluster is split at once); mode 2 follows Alg. 1
 * with "resident" = selected by the unit's latest retrieval.  The paper gives
 * no values for tau_min, tau_max, N0: they are parameters.  Periodic full
 * re-clustering and the maintainer exclude each other.  Returns 0 or -1. */
int orc_unit_set_maintainer(orc_unit *u, int mode, int c_init, double tau_min,
                            double tau_max, double n0, int split_iters,
                            int buf_max)
{
    if (u->n_frames != 0 || u->recluster_every != 0) return -1;
    if (mode < 1 || mode > 2 || c_init < 1 || c_init > u->C || !(n0 > 0.0) ||
        split_iters < 1 || buf_max < 0) return -1;
    u->maint_mode = mode; u->c_init = c_init; u->n_slots = c_init;
    u->tau_min = tau_min; u->tau_max = tau_max; u->n0 = n0;
    u->split_iters = split_iters; u->buf_max = buf_max;
    u->warmup = u->warmup_arg > 0 ? u->warmup_arg : 2 * c_init;
    u->var = (double *)calloc((size_t)u->C, sizeof(double));
    u->lazy = (int *)calloc((size_t)u->C, sizeof(int));
    u->resident = (int *)calloc((size_t)u->C, sizeof(int));
    u->buf_frame = (int *)calloc((size_t)(buf_max > 0 ? buf_max : 1), sizeof(int));
    u->buf_owner = (int *)calloc((size_t)(buf_max > 0 ? buf_max : 1), sizeof(int));
    u->n_buf = 0;
    return 0;
}

/* "C is in GPU memory" (Alg. 1 line 4) decided outside: with an offloading tier the clusters that
 * are on the GPU are those its working set holds (see oracle/cache_model.py).  After
 * orc_unit_external_residency(u, 1) the retrieval procedure no longer marks its selection as
 * resident; the caller sets the flags with orc_unit_set_resident (flags [C], copied).  A split
 * still hands the parent's flag to the new cluster. */
void orc_unit_external_residency(orc_unit *u, int on) { u->resident_external = on != 0; }
void orc_unit_set_resident(orc_unit *u, const int *flags)
{
    if (u->maint_mode) memcpy(u->resident, flags, (size_t)u->C * sizeof(int));
}

/* Size-adaptive threshold, Eq. 5. */
double orc_tau(double tau_min, double tau_max, double n0, double N)
{
    return tau_min + (tau_max - tau_min) * exp(-N / n0);
}

static double sqdist(const double *a, const double *b, int D)
{
    double s = 0.0;
    for (int d = 0; d < D; ++d) { double t = a[d] - b[d]; s += t * t; }
    return s;
}

/* Size, representative (Eq. 1) and variance (Eq. 2) of cluster j from its
 * member list, members in ascending frame order. */
static void exact_stats(orc_unit *u, int j)
{
    const int D = u->D, F = u->n_frames;
    double *rj = u->r + (size_t)j * D;
    int cnt = 0;
    for (int f = 0; f < F; ++f) cnt += (u->assign[f] == j);
    u->n[j] = cnt;
    if (cnt == 0) { u->var[j] = 0.0; return; }
    for (int d = 0; d < D; ++d) {
        double acc = 0.0;
        for (int f = 0; f < F; ++f)
            if (u->assign[f] == j) acc += u->summ[(size_t)f * D + d];
        rj[d] = acc / (double)cnt;
    }
    double acc = 0.0;
    for (int f = 0; f < F; ++f)
        if (u->assign[f] == j) acc += sqdist(u->summ + (size_t)f * D, rj, D);
    u->var[j] = acc / (double)cnt;
}

/* Split (Alg. 1, lines 5 and 14) -- the paper does not define it.  Reading:
 * two-means under the clustering criterion of Sec. V-B.  Seeds are the two
 * members with the lowest mutual cosine (first such pair in (i, i') order);
 * then split_iters rounds of (each member to the seed representative it is
 * more similar to, equal goes to the first; representatives = means of their
 * sides, a side left empty keeps its representative).  mem[0..m) ascending
 * frames; side[i] = 0 stays, 1 leaves.  Returns the size of side 1 (0 or m
 * means the split is degenerate). */
static int split_members(orc_unit *u, const int *mem, int m, int *side)
{
    const int D = u->D;
    u->split_min_gap = INFINITY;
    if (m < 2) { for (int i = 0; i < m; ++i) side[i] = 0; return 0; }
    int si = 0, sj = 1;
    double best = INFINITY, second = INFINITY;
    for (int i = 0; i < m; ++i)
        for (int k = i + 1; k < m; ++k) {
            double c = cosine(u->summ + (size_t)mem[i] * D, u->summ + (size_t)mem[k] * D, D);
            if (c < best) { second = best; best = c; si = i; sj = k; }
            else if (c < second) second = c;
        }
    if (second < INFINITY) u->split_min_gap = rel_gap(best, second);
    double *ca = (double *)malloc((size_t)D * sizeof(double));
    double *cb = (double *)malloc((size_t)D * sizeof(double));
    memcpy(ca, u->summ + (size_t)mem[si] * D, (size_t)D * sizeof(double));
    memcpy(cb, u->summ + (size_t)mem[sj] * D, (size_t)D * sizeof(double));
    int nb = 0;
    for (int it = 0; it < u->split_iters; ++it) {
        nb = 0;
        for (int i = 0; i < m; ++i) {
            const double *s = u->summ + (size_t)mem[i] * D;
            double a = cosine(s, ca, D), b = cosine(s, cb, D);
            side[i] = b > a;
            nb += side[i];
            double g = rel_gap(a, b);
            if (g < u->split_min_gap) u->split_min_gap = g;
        }
        for (int which = 0; which < 2; ++which) {
            int cnt = which ? nb : m - nb;
            if (cnt == 0) continue;
            double *c = which ? cb : ca;
            for (int d = 0; d < D; ++d) {
                double acc = 0.0;
                for (int i = 0; i < m; ++i)
                    if (side[i] == which) acc += u->summ[(size_t)mem[i] * D + d];
                c[d] = acc / (double)cnt;
            }
        }
    }
    free(ca); free(cb);
    return nb;
}

/* Split cluster a into a (the side of the first seed) and a new cluster id.
 * Returns the new id, or -1 if nothing was split (no free id, fewer than two
 * members, or one side empty); statistics of the touched clusters are then
 * exact (Eq. 1, Eq. 2) when `refresh` is set. */
static int split_cluster(orc_unit *u, int a, int refresh)
{
    const int F = u->n_frames;
    int m = 0, fresh = -1;
    for (int f = 0; f < F; ++f) m += (u->assign[f] == a);
    if (u->n_slots < u->C && m >= 2) {
        int *mem = (int *)malloc((size_t)m * sizeof(int));
        int *side = (int *)malloc((size_t)m * sizeof(int));
        int k = 0;
        for (int f = 0; f < F; ++f) if (u->assign[f] == a) mem[k++] = f;
        int nb = split_members(u, mem, m, side);
        if (nb > 0 && nb < m) {
            fresh = u->n_slots++;
            for (int i = 0; i < m; ++i) if (side[i]) u->assign[mem[i]] = fresh;
            exact_stats(u, a);
            exact_stats(u, fresh);
            u->lazy[a] = u->lazy[fresh] = 0;
            u->resident[fresh] = u->resident[a];
        }
        free(mem); free(side);
    }
    if (fresh < 0 && refresh) exact_stats(u, a);
    return fresh;
}

/* Insertion procedure of Alg. 1 for frame f (summary s) given its cluster a. */
static void maintain_insert(orc_unit *u, int f, const double *s, int a)
{
    const int D = u->D;
    double *ra = u->r + (size_t)a * D;
    const double na = (double)u->n[a];
    for (int d = 0; d < D; ++d)                        /* Eq. 3 */
        ra[d] = (na * ra[d] + s[d]) / (na + 1.0);
    const double var_new = (na * u->var[a] + sqdist(s, ra, D)) / (na + 1.0);   /* Eq. 4 */
    const double tau = orc_tau(u->tau_min, u->tau_max, u->n0, na);  /* size before the insertion (line 2) */
    u->var[a] = var_new;                               /* line 1: statistics always move */
    u->last_var = var_new; u->last_tau = tau;
    const int on_gpu = u->maint_mode == 1 || u->resident[a];
    if (var_new <= tau) {                              /* lines 2-3 */
        u->assign[f] = a; u->n[a] += 1;
        u->last_action = ORC_ACT_ABSORB;
    } else if (on_gpu) {                               /* lines 4-6 */
        u->assign[f] = a; u->n[a] += 1;
        if (split_cluster(u, a, 0) >= 0) { u->n_split_now += 1; u->last_action = ORC_ACT_SPLIT; }
        else { u->n_forced_absorb += 1; u->last_action = ORC_ACT_FORCED_ABSORB; }
    } else if (u->n_buf < u->buf_max) {                /* lines 7-10 */
        u->lazy[a] = 1;
        u->buf_frame[u->n_buf] = f; u->buf_owner[u->n_buf] = a; u->n_buf += 1;
        u->assign[f] = -2 - a;                         /* held in the buffer on behalf of a */
        u->n_deferred += 1; u->last_action = ORC_ACT_DEFER;
    } else {                                           /* buffer full: the paper is silent; absorb */
        u->lazy[a] = 1;
        u->assign[f] = a; u->n[a] += 1;
        u->n_forced_absorb += 1; u->last_action = ORC_ACT_FORCED_ABSORB;
    }
}

/* Retrieval procedure of Alg. 1 (lines 12-17) for one selected cluster: merge
 * its buffered entries, split, refresh the representatives, clear the flag. */
static void materialize(orc_unit *u, int j)
{
    if (!u->lazy[j]) return;
    int w = 0;
    for (int b = 0; b < u->n_buf; ++b) {
        if (u->buf_owner[b] == j) { u->assign[u->buf_frame[b]] = j; continue; }
        u->buf_frame[w] = u->buf_frame[b]; u->buf_owner[w] = u->buf_owner[b]; ++w;
    }
    u->n_buf = w;
    u->lazy[j] = 0;
    if (split_cluster(u, j, 1) >= 0) u->n_split_deferred += 1;
}

/* Query Retrieval with the maintainer on (mode 2): the representative set is
 * the non-empty clusters plus the buffered singletons (a singleton's
 * representative is its own summary, Alg. 1 line 10).  score [C + buf_max];
 * selected ids: cluster j -> j, buffer entry b -> C + b; sorted by (score
 * descending, id ascending); tokens as in the plain gather, a singleton
 * contributing its one frame.  Afterwards the selected clusters count as GPU
 * resident, all others as not, and every selected cluster with a lazy flag
 * has its deferred split materialized (in selection order).  Returns the
 * number of ids; *n_tok tokens are written to tok_idx. */
int orc_unit_retrieve_maintained(orc_unit *u, const double *qbar, int k, int *ids,
                                 double *score, int *tok_idx, int *n_tok,
                                 double *gap_k)
{
    const int C = u->C, D = u->D, R = C + u->n_buf;
    orc_unit_score(u, qbar, score);
    int *live = (int *)calloc((size_t)R, sizeof(int));
    for (int j = 0; j < C; ++j) live[j] = u->n[j];
    for (int b = 0; b < u->n_buf; ++b) {
        const double *sb = u->summ + (size_t)u->buf_frame[b] * D;
        double dp = dot(qbar, sb, D);
        if (u->score_mode == 1) score[C + b] = dp;
        else { double nr = sqrt(dot(sb, sb, D)); score[C + b] = nr == 0.0 ? 0.0 : dp / nr; }
        live[C + b] = 1;
    }
    int kept = orc_select(score, live, R, k, ids, gap_k);
    free(live);
    int m = 0;
    for (int i = 0; i < kept; ++i) {
        if (ids[i] >= C) {
            int f = u->buf_frame[ids[i] - C];
            for (int t = 0; t < u->T; ++t) tok_idx[m++] = f * u->T + t;
        } else {
            for (int f = 0; f < u->n_frames; ++f)
                if (u->assign[f] == ids[i])
                    for (int t = 0; t < u->T; ++t) tok_idx[m++] = f * u->T + t;
        }
    }
    *n_tok = m;
    if (u->maint_mode == 2) {
        if (!u->resident_external) {
            memset(u->resident, 0, (size_t)C * sizeof(int));
            for (int i = 0; i < kept; ++i) if (ids[i] < C) u->resident[ids[i]] = 1;
        }
        for (int i = 0; i < kept; ++i) if (ids[i] < C) materialize(u, ids[i]);
    }
    return kept;
}

/* ------------------------------------------------------------------------
 * Nested visual-semantic hierarchy and two-stage retrieval (Sec. V-B, V-C).
 *
 * The visual level is the same modified K-means, run once per stream on the
 * per-frame visual embeddings (an orc_unit of its own with T = 1 and C = P,
 * see the Python wrapper); it hands every frame a partition id.  This unit,
 * the semantic level of one (layer, KV head), clusters key summaries inside
 * each partition only.  The paper fixes neither how the C cluster ids are
 * shared out nor how a partition's K-means starts; the reading taken: every
 * partition owns Cs = C / P ids, and a partition with np warm-up members
 * starts L = min(Cs, np) clusters from its members floor(j*np/L), j < L (the
 * flat seeding rule applied to the partition's member list); ids that are
 * not started stay empty.  Periodic re-clustering and the maintainer are not
 * combined with the hierarchy.
 * ------------------------------------------------------------------------ */

/* Switch the hierarchy on with P partitions; call before the first frame.
 * Returns 0, or -1 (P < 1, C not a multiple of P, maintainer or periodic
 * re-clustering on, frames already in). */
int orc_unit_set_nested(orc_unit *u, int P)
{
    if (P < 1 || u->C % P != 0 || u->maint_mode || u->recluster_every || u->n_frames > 0) return -1;
    u->n_part = P; u->Cs = u->C / P;
    free(u->part);
    u->part = (int *)malloc((size_t)u->max_frames * sizeof(int));
    for (int f = 0; f < u->max_frames; ++f) u->part[f] = -1;
    return 0;
}

static void seed_nested(orc_unit *u)
{
    const int W = u->warmup, D = u->D, Cs = u->Cs;
    int *mem = (int *)malloc((size_t)W * sizeof(int));
    memset(u->n, 0, (size_t)u->C * sizeof(int));
    memset(u->r, 0, (size_t)u->C * D * sizeof(double));
    for (int p = 0; p < u->n_part; ++p) {
        int np = 0;
        for (int f = 0; f < W; ++f) if (u->part[f] == p) mem[np++] = f;
        const int L = np < Cs ? np : Cs;
        for (int j = 0; j < L; ++j) {
            const int src = mem[(int)(((long long)j * np) / L)];
            memcpy(u->r + (size_t)(p * Cs + j) * D, u->summ + (size_t)src * D, (size_t)D * sizeof(double));
            u->n[p * Cs + j] = 1;          /* started: takes part in the first assignment round */
        }
    }
    free(mem);
}

/* Frame Encoding under the hierarchy: as orc_unit_ingest, with the visual
 * level's frame -> partition map.  part[0..n_frames] must be valid from the
 * frame that completes the warm-up on (the visual level uses the same warm-up
 * length, so it becomes ready on that very frame); before that it is not read. */
int orc_unit_ingest_nested(orc_unit *u, const double *k_frame, const int *part,
                           int force, orc_decision *dec)
{
    if (u->n_part <= 0 || u->n_frames >= u->max_frames) return -1;
    const int f = u->n_frames;
    if (u->ready) u->part[f] = part[f];
    else if (f + 1 == u->warmup) memcpy(u->part, part, (size_t)u->warmup * sizeof(int));
    return orc_unit_ingest(u, k_frame, force, dec);
}

/* What the greedy rule would decide for a frame of partition p (no change of state). */
void orc_unit_peek_nested(const orc_unit *u, const double *k_frame, int p, orc_decision *dec)
{
    double *s = (double *)malloc((size_t)u->D * sizeof(double));
    orc_summary(k_frame, u->T, u->D, s);
    nearest_in(u, s, 0, p * u->Cs, (p + 1) * u->Cs, dec);
    free(s);
}

/* Visual-level representative as this unit's query sees it.  The query lives
 * in the layer's key space, not in the vision encoder's, so the partition is
 * summarized the way every cluster is (Eq. 1): the mean of the key summaries
 * of its frames, in ascending frame order.  rp [D]; returns the frame count. */
int orc_unit_partition_rep(const orc_unit *u, int p, double *rp)
{
    const int D = u->D;
    int cnt = 0;
    for (int d = 0; d < D; ++d) rp[d] = 0.0;
    for (int f = 0; f < u->n_frames; ++f) {
        if (u->part[f] != p) continue;
        for (int d = 0; d < D; ++d) rp[d] += u->summ[(size_t)f * D + d];
        ++cnt;
    }
    if (cnt > 0) for (int d = 0; d < D; ++d) rp[d] /= (double)cnt;
    return cnt;
}

/* Two-Stage Retrieval (Sec. V-C): (1) score the P partition representatives
 * with the query (same relevance as for clusters) and keep the top_p best
 * non-empty partitions; (2) score the non-empty clusters of those partitions
 * only and keep the top k of them.  part_score [P] and score [C] receive the
 * scores (-inf for empty or pruned entries); part_ids [top_p]; ids [k];
 * gap_p / gap_k = relative gap at each cut; *n_cand = clusters scored in
 * stage 2.  Returns the number of clusters kept; *n_part_kept partitions. */
int orc_unit_retrieve_nested(const orc_unit *u, const double *qbar, int top_p, int k,
                             int *part_ids, int *n_part_kept, double *part_score,
                             int *ids, double *score, double *gap_p, double *gap_k,
                             int *n_cand)
{
    const int P = u->n_part, D = u->D, Cs = u->Cs;
    double *rp = (double *)malloc((size_t)D * sizeof(double));
    int *pn = (int *)malloc((size_t)P * sizeof(int));
    for (int p = 0; p < P; ++p) {
        pn[p] = orc_unit_partition_rep(u, p, rp);
        if (pn[p] == 0) { part_score[p] = -INFINITY; continue; }
        double dp = dot(qbar, rp, D);
        if (u->score_mode == 1) { part_score[p] = dp; continue; }
        double nr = sqrt(dot(rp, rp, D));
        part_score[p] = nr == 0.0 ? 0.0 : dp / nr;
    }
    const int kept_p = orc_select(part_score, pn, P, top_p, part_ids, gap_p);
    *n_part_kept = kept_p;
    int *live = (int *)calloc((size_t)u->C, sizeof(int));
    double *full = (double *)malloc((size_t)u->C * sizeof(double));
    orc_unit_score(u, qbar, full);
    int cand = 0;
    for (int j = 0; j < u->C; ++j) score[j] = -INFINITY;
    for (int i = 0; i < kept_p; ++i)
        for (int j = part_ids[i] * Cs; j < (part_ids[i] + 1) * Cs; ++j)
            if (u->n[j] > 0) { live[j] = u->n[j]; score[j] = full[j]; ++cand; }
    if (n_cand) *n_cand = cand;
    const int kept = orc_select(score, live, u->C, k, ids, gap_k);
    free(rp); free(pn); free(live); free(full);
    return kept;
}

/* What the greedy rule would decide for a frame, without changing state.
 * Only meaningful once the unit is ready and no (re-)clustering is due. */
void orc_unit_peek(const orc_unit *u, const double *k_frame, orc_decision *dec)
{
    double *s = (double *)malloc((size_t)u->D * sizeof(double));
    orc_summary(k_frame, u->T, u->D, s);
    nearest_in(u, s, 0, 0, u->n_slots, dec);
    free(s);
}

/* Frame Encoding for one unit (Sec. V-A (1), Sec. VI-A).
 *  - the first `warmup` frames are only buffered; when the warmup-th arrives
 *    the initial clustering runs: seeds r_j = summary of frame floor(j*W/C),
 *    then Lloyd rounds (the paper does not say how K-means starts);
 *  - afterwards every frame is assigned greedily and the representative is
 *    updated by Eq. 3;
 *  - if recluster_every > 0, a full Lloyd run warm-started from the current
 *    representatives follows whenever the frame count reaches a multiple of
 *    it (beyond the warm-up).
 * force >= 0 makes the online step adopt that cluster instead of its own
 * choice (used by the parity harness at documented near-ties only).
 * Returns 0, or -1 if the unit is full.  dec may be NULL. */
int orc_unit_ingest(orc_unit *u, const double *k_frame, int force,
                    orc_decision *dec)
{
    if (u->n_frames >= u->max_frames) return -1;
    const int D = u->D, f = u->n_frames;
    double *s = u->summ + (size_t)f * D;
    orc_summary(k_frame, u->T, D, s);
    orc_decision local;
    local.winner = -1; local.runner_up = -1; local.gap = INFINITY; local.sim = 0.0;
    if (!u->ready) {
        u->n_frames = f + 1;
        if (u->n_frames == u->warmup && u->n_part > 0) {
            seed_nested(u);
            lloyd(u, 0);
            u->ready = 1;
        } else if (u->n_frames == u->warmup) {
            const int W = u->warmup;
            for (int j = 0; j < u->n_slots; ++j) {
                int src = (int)(((long long)j * W) / u->n_slots);
                memcpy(u->r + (size_t)j * D, u->summ + (size_t)src * D,
                       (size_t)D * sizeof(double));
                u->n[j] = 0;
            }
            lloyd(u, 1);
            if (u->maint_mode)                          /* Eq. 2 from the members */
                for (int j = 0; j < u->n_slots; ++j) exact_stats(u, j);
            u->ready = 1;
        }
    } else if (u->maint_mode) {
        nearest(u, f, s, 0, &local);
        u->n_frames = f + 1;                            /* the new state is part of what a split sees */
        maintain_insert(u, f, s, force >= 0 ? force : local.winner);
    } else {
        nearest(u, f, s, 0, &local);
        int a = force >= 0 ? force : local.winner;
        double *ra = u->r + (size_t)a * D;
        double na = (double)u->n[a];
        for (int d = 0; d < D; ++d)                    /* Eq. 3 */
            ra[d] = (na * ra[d] + s[d]) / (na + 1.0);
        u->n[a] += 1;
        u->assign[f] = a;
        u->n_frames = f + 1;
        if (u->recluster_every > 0 && u->n_frames % u->recluster_every == 0)
            lloyd(u, 0);
    }
    if (dec) *dec = local;
    return 0;
}

/* Mean query of the unit: over the Tq question tokens and the G query heads
 * that share KV head h (the paper speaks of "a query"; the mean makes one
 * vector out of several, and a dot product with it equals the mean of the
 * individual dot products).  q is [Tq][Hq][D]. */
void orc_mean_query(const double *q, int Tq, int Hq, int D, int h, int G,
                    double *qbar)
{
    for (int d = 0; d < D; ++d) {
        double acc = 0.0;
        for (int t = 0; t < Tq; ++t)
            for (int g = 0; g < G; ++g)
                acc += q[((size_t)t * Hq + (size_t)h * G + g) * D + d];
        qbar[d] = acc / (double)(Tq * G);
    }
}

/* Query-to-representative relevance (Sec. V-C, second retrieval stage):
 * score_j = (qbar . r_j) / |r_j|, i.e. the cosine up to the factor 1/|qbar|
 * common to all clusters; score_mode 1 is the plain dot product.  Empty
 * clusters score -inf; a zero representative scores 0. */
void orc_unit_score(const orc_unit *u, const double *qbar, double *score)
{
    for (int j = 0; j < u->C; ++j) {
        if (u->n[j] == 0) { score[j] = -INFINITY; continue; }
        const double *rj = u->r + (size_t)j * u->D;
        double dp = dot(qbar, rj, u->D);
        if (u->score_mode == 1) { score[j] = dp; continue; }
        double nr = sqrt(dot(rj, rj, u->D));
        score[j] = nr == 0.0 ? 0.0 : dp / nr;
    }
}

typedef struct { double s; int id; } scored;

static int by_score_desc_id_asc(const void *a, const void *b)
{
    const scored *x = (const scored *)a, *y = (const scored *)b;
    if (x->s > y->s) return -1;
    if (x->s < y->s) return 1;
    return x->id - y->id;
}

/* Top-K clusters (Sec. V-C, Sec. VII-B): full sort of the non-empty clusters
 * by (score descending, id ascending), first min(k, #non-empty) kept.
 * gap_k = relative gap between the last kept and the first dropped score
 * (inf if nothing is dropped).  Returns the number kept. */
int orc_select(const double *score, const int *n, int C, int k, int *ids,
               double *gap_k)
{
    scored *v = (scored *)malloc((size_t)C * sizeof(scored));
    int m = 0;
    for (int j = 0; j < C; ++j)
        if (n[j] > 0) { v[m].s = score[j]; v[m].id = j; ++m; }
    qsort(v, (size_t)m, sizeof(scored), by_score_desc_id_asc);
    int kept = k < m ? k : m;
    for (int i = 0; i < kept; ++i) ids[i] = v[i].id;
    if (gap_k) *gap_k = (kept < m && kept > 0) ? rel_gap(v[kept - 1].s, v[kept].s)
                                               : INFINITY;
    free(v);
    return kept;
}

/* Cluster-granular gather (Sec. V-C: clusters are the retrieval units): for
 * each selected cluster in selection order, each member frame in ascending
 * order, all T tokens of the frame; token index = f*T + t.  Returns the
 * number of tokens written. */
int orc_unit_gather(const orc_unit *u, const int *ids, int n_ids, int *tok_idx)
{
    int m = 0;
    for (int i = 0; i < n_ids; ++i)
        for (int f = 0; f < u->n_frames; ++f)
            if (u->assign[f] == ids[i])
                for (int t = 0; t < u->T; ++t) tok_idx[m++] = f * u->T + t;
    return m;
}

/* Attention of the question tokens over the retrieved KV (Sec. V-A (2)):
 * softmax(q K^T / sqrt(D)) V restricted to tok_idx, for the G query heads of
 * KV head h; no mask (everything retrieved lies in the past).
 * q [Tq][Hq][D]; K,V [N][D] of this unit (token-major);
 * out [Tq][G][D]; lse [Tq][G] = log sum exp of the scaled logits. */
void orc_attend(const double *q, int Tq, int Hq, int D, int h, int G,
                const double *K, const double *V, const int *tok_idx, int n_tok,
                double *out, double *lse)
{
    const double scale = 1.0 / sqrt((double)D);
    double *logit = (double *)malloc((size_t)(n_tok > 0 ? n_tok : 1) * sizeof(double));
    for (int t = 0; t < Tq; ++t)
        for (int g = 0; g < G; ++g) {
            const double *qv = q + ((size_t)t * Hq + (size_t)h * G + g) * D;
            double *o = out + ((size_t)t * G + g) * D;
            double mx = -INFINITY;
            for (int i = 0; i < n_tok; ++i) {
                logit[i] = dot(qv, K + (size_t)tok_idx[i] * D, D) * scale;
                if (logit[i] > mx) mx = logit[i];
            }
            double den = 0.0;
            for (int d = 0; d < D; ++d) o[d] = 0.0;
            for (int i = 0; i < n_tok; ++i) {
                double p = exp(logit[i] - mx);
                den += p;
                const double *vv = V + (size_t)tok_idx[i] * D;
                for (int d = 0; d < D; ++d) o[d] += p * vv[d];
            }
            if (n_tok > 0) {
                for (int d = 0; d < D; ++d) o[d] /= den;
                lse[(size_t)t * G + g] = mx + log(den);
            } else {
                lse[(size_t)t * G + g] = -INFINITY;
            }
        }
    free(logit);
}

/* Accessors for the Python wrapper. */
int orc_unit_n_frames(const orc_unit *u) { return u->n_frames; }
int orc_unit_ready(const orc_unit *u) { return u->ready; }
int orc_unit_n_lloyd_runs(const orc_unit *u) { return u->n_lloyd_runs; }
double orc_unit_lloyd_min_gap(const orc_unit *u) { return u->lloyd_min_gap; }
const double *orc_unit_centroids(const orc_unit *u) { return u->r; }
const int *orc_unit_sizes(const orc_unit *u) { return u->n; }
const int *orc_unit_assign(const orc_unit *u) { return u->assign; }
const double *orc_unit_summaries(const orc_unit *u) { return u->summ; }
int orc_unit_n_slots(const orc_unit *u) { return u->n_slots; }
int orc_unit_n_buf(const orc_unit *u) { return u->n_buf; }
int orc_unit_last_action(const orc_unit *u) { return u->last_action; }
double orc_unit_last_var(const orc_unit *u) { return u->last_var; }
double orc_unit_last_tau(const orc_unit *u) { return u->last_tau; }
double orc_unit_split_min_gap(const orc_unit *u) { return u->split_min_gap; }
long orc_unit_n_split_now(const orc_unit *u) { return u->n_split_now; }
long orc_unit_n_split_deferred(const orc_unit *u) { return u->n_split_deferred; }
long orc_unit_n_deferred(const orc_unit *u) { return u->n_deferred; }
long orc_unit_n_forced_absorb(const orc_unit *u) { return u->n_forced_absorb; }
const double *orc_unit_var(const orc_unit *u) { return u->var; }
const int *orc_unit_lazy(const orc_unit *u) { return u->lazy; }
const int *orc_unit_resident(const orc_unit *u) { return u->resident; }
const int *orc_unit_buf_frame(const orc_unit *u) { return u->buf_frame; }
const int *orc_unit_buf_owner(const orc_unit *u) { return u->buf_owner; }
const int *orc_unit_part(const orc_unit *u) { return u->part; }
