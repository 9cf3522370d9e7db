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
} orc_unit;

typedef struct {
    int winner;     /* chosen cluster */
    int runner_up;  /* second best, -1 if there is none */
    double gap;     /* |a-b| / max(|a|,|b|,1e-30) of their similarities */
    double sim;     /* similarity of the winner */
} orc_decision;

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
    free(u->summ); free(u->r); free(u->n); free(u->assign); free(u);
}

void orc_unit_reset(orc_unit *u)
{
    u->n_frames = 0; u->ready = 0; u->n_lloyd_runs = 0;
    u->lloyd_min_gap = INFINITY;
    memset(u->r, 0, (size_t)u->C * u->D * sizeof(double));
    memset(u->n, 0, (size_t)u->C * sizeof(int));
    for (int f = 0; f < u->max_frames; ++f) u->assign[f] = -1;
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
static void nearest(const orc_unit *u, const double *s, int all_live,
                    orc_decision *dec)
{
    int best = -1, second = -1;
    double bs = -INFINITY, ss = -INFINITY;
    for (int j = 0; j < u->C; ++j) {
        if (!all_live && u->n[j] == 0) continue;
        double c = cosine(s, u->r + (size_t)j * u->D, u->D);
        if (best < 0 || c > bs) { second = best; ss = bs; best = j; bs = c; }
        else if (second < 0 || c > ss) { second = j; ss = c; }
    }
    if (best < 0) { best = 0; bs = 0.0; }      /* no live cluster at all */
    dec->winner = best; dec->runner_up = second; dec->sim = bs;
    dec->gap = second >= 0 ? rel_gap(bs, ss) : INFINITY;
}

/* Modified K-means of Sec. V-B: `iters` rounds of (assign every stored summary
 * by the greedy cosine rule, then set each representative to the mean of its
 * members, Eq. 1).  A cluster left without members keeps its previous
 * representative and is skipped by later assignments.  Members are summed in
 * ascending frame order. */
static void lloyd(orc_unit *u, int first_all_live)
{
    const int F = u->n_frames, C = u->C, D = u->D;
    u->lloyd_min_gap = INFINITY;
    for (int it = 0; it < u->lloyd_iters; ++it) {
        int all_live = first_all_live && it == 0;
        for (int f = 0; f < F; ++f) {
            orc_decision dec;
            nearest(u, u->summ + (size_t)f * D, all_live, &dec);
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

/* What the greedy rule would decide for a frame, without changing state.
 * Only meaningful once the unit is ready and no (re-)clustering is due. */
void orc_unit_peek(const orc_unit *u, const double *k_frame, orc_decision *dec)
{
    double *s = (double *)malloc((size_t)u->D * sizeof(double));
    orc_summary(k_frame, u->T, u->D, s);
    nearest(u, s, 0, dec);
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
        if (u->n_frames == u->warmup) {
            const int W = u->warmup;
            for (int j = 0; j < u->C; ++j) {
                int src = (int)(((long long)j * W) / u->C);
                memcpy(u->r + (size_t)j * D, u->summ + (size_t)src * D,
                       (size_t)D * sizeof(double));
                u->n[j] = 0;
            }
            lloyd(u, 1);
            u->ready = 1;
        }
    } else {
        nearest(u, s, 0, &local);
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
