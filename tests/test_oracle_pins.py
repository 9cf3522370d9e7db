"""Pins for the CPU oracle: closed forms, brute force, invariants, special cases
that reduce to library routines, and hand-worked fixtures.  No GPU needed.

Each test names the passage of the paper whose reading it pins.  The brute
forces below are written with numpy/scipy whole-array routines, not with the
oracle's loops, so an index, sign or transposition mistake in the oracle shows.
"""
import os

import numpy as np
import pytest
from scipy.special import logsumexp, softmax

from oracle import mosaic_oracle as orc
from paper_2604_10060_amd import inputs

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


def _cos_matrix(S, R):
    """Exhaustive cosine table with whole-array numpy (Sec. V-B criterion)."""
    Sn = S / np.linalg.norm(S, axis=1, keepdims=True)
    Rn = R / np.linalg.norm(R, axis=1, keepdims=True)
    return Sn @ Rn.T


def _stream(F, T, D, n_scenes, seed, noise=0.3):
    """Small scene-structured key stream [F][T][D] and its scene labels."""
    r = _rng(seed)
    centres = r.normal(size=(n_scenes, D))
    labels = np.sort(r.integers(0, n_scenes, size=F))
    K = centres[labels][:, None, :] + noise * r.normal(size=(F, T, D))
    return K, labels


# --------------------------------------------------------------------------
# O1: per-frame key summary
# --------------------------------------------------------------------------
def test_summary_is_token_mean():
    K = _rng(1).normal(size=(7, 13))
    np.testing.assert_allclose(orc.summary(K), K.mean(axis=0), rtol=1e-14, atol=1e-15)
    # a transposed read would give a vector of the wrong length or values
    assert orc.summary(K).shape == (13,)


# --------------------------------------------------------------------------
# Eq. 3 vs Eq. 1, hand-worked fixture
# --------------------------------------------------------------------------
def test_eq3_hand_worked_fixture():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "eq3_running_mean.txt"))
            if l.strip() and not l.startswith("#")]
    # one cluster, one token per frame: the frame summary is the state itself
    u = orc.OracleUnit(1, 2, 1, 8, warmup_frames=1, lloyd_iters=1)
    for step, x, y, rx, ry, n in rows:
        u.ingest(np.array([[float(x), float(y)]]))
        np.testing.assert_allclose(u.centroids()[0], [float(rx), float(ry)], atol=1e-15)
        assert u.sizes()[0] == int(n)


# --------------------------------------------------------------------------
# O3/O4: greedy online assignment = exhaustive search; Eq. 3 = Eq. 1
# --------------------------------------------------------------------------
@pytest.mark.parametrize("seed,C,D,T,F", [(3, 4, 8, 3, 60), (4, 6, 16, 5, 90), (5, 3, 5, 1, 40)])
def test_online_assignment_is_exhaustive_argmax_and_running_mean(seed, C, D, T, F):
    K, _ = _stream(F, T, D, C, seed)
    u = orc.OracleUnit(C, D, T, F, warmup_frames=2 * C, lloyd_iters=4)
    for f in range(F):
        if u.ready:
            R, n = u.centroids(), u.sizes()
            s = K[f].mean(axis=0)
            cos = _cos_matrix(s[None, :], np.where(n[:, None] > 0, R, 1.0))[0]
            cos[n == 0] = -np.inf
            want = int(np.argmax(cos))          # numpy argmax: first maximum = lowest id
            dec = u.ingest(K[f])
            assert dec.winner == want
            assert u.assignments()[f] == want
            order = np.sort(cos)[::-1]
            if len(order) > 1 and np.isfinite(order[1]):
                gap = abs(order[0] - order[1]) / max(abs(order[0]), abs(order[1]), 1e-30)
                assert dec.gap == pytest.approx(gap, rel=1e-6, abs=1e-12)
        else:
            u.ingest(K[f])
    a, n, R = u.assignments(), u.sizes(), u.centroids()
    # partition: every frame in exactly one cluster (Sec. VI-A, greedy rule)
    assert a.min() >= 0 and a.max() < C
    np.testing.assert_array_equal(np.bincount(a, minlength=C), n)
    assert n.sum() == F
    S = K.mean(axis=1)
    for j in range(C):
        if n[j]:
            # Eq. 3 after any insert sequence == Eq. 1 batch mean of the members
            np.testing.assert_allclose(R[j], S[a == j].mean(axis=0), rtol=1e-12, atol=1e-13)
            # equal tokens per frame: also the mean of all member token keys
            np.testing.assert_allclose(R[j], K[a == j].reshape(-1, D).mean(axis=0),
                                       rtol=1e-12, atol=1e-13)


def test_single_cluster_takes_everything():
    K, _ = _stream(20, 2, 4, 3, 9)
    u = orc.OracleUnit(1, 4, 2, 20, warmup_frames=2, lloyd_iters=2)
    for f in range(20):
        u.ingest(K[f])
    assert (u.assignments() == 0).all() and u.sizes()[0] == 20


def test_forced_decision_is_adopted():
    K, _ = _stream(30, 2, 6, 3, 11)
    u = orc.OracleUnit(3, 6, 2, 30, warmup_frames=6, lloyd_iters=3)
    for f in range(29):
        u.ingest(K[f])
    peek = u.peek(K[29])
    other = (peek.winner + 1) % 3
    n_before = u.sizes()
    dec = u.ingest(K[29], force=other)
    assert dec.winner == peek.winner and dec.gap == peek.gap   # the record stays the oracle's own
    assert u.assignments()[29] == other
    assert u.sizes()[other] == n_before[other] + 1


# --------------------------------------------------------------------------
# O2/O5: Lloyd rounds vs a whole-array brute force
# --------------------------------------------------------------------------
def _lloyd_brute(S, R, n, iters, first_all_live):
    R, n = R.copy(), n.copy()
    a = None
    for it in range(iters):
        live = np.ones(len(n), bool) if (first_all_live and it == 0) else n > 0
        cos = _cos_matrix(S, np.where(live[:, None], R, 1.0))
        cos[:, ~live] = -np.inf
        a = np.argmax(cos, axis=1)
        n = np.bincount(a, minlength=len(n))
        for j in np.nonzero(n)[0]:
            R[j] = S[a == j].mean(axis=0)
    return a, R, n


@pytest.mark.parametrize("seed,C,D,T", [(21, 4, 8, 2), (22, 5, 12, 3)])
def test_init_lloyd_matches_brute_force(seed, C, D, T):
    W = 2 * C + 3
    K, _ = _stream(W, T, D, C, seed, noise=0.6)
    u = orc.OracleUnit(C, D, T, W, warmup_frames=W, lloyd_iters=5)
    for f in range(W):
        assert not u.ready
        u.ingest(K[f])
    assert u.ready and u.n_lloyd_runs == 1
    S = K.mean(axis=1)
    seeds = S[[(j * W) // C for j in range(C)]]
    a, R, n = _lloyd_brute(S, seeds, np.zeros(C, int), 5, True)
    np.testing.assert_array_equal(u.assignments(), a)
    np.testing.assert_array_equal(u.sizes(), n)
    live = n > 0
    np.testing.assert_allclose(u.centroids()[live], R[live], rtol=1e-12, atol=1e-13)


def test_recluster_warm_start_matches_brute_force():
    C, D, T, W, every, F = 3, 6, 2, 6, 8, 24
    K, _ = _stream(F, T, D, 4, 31, noise=0.8)
    u = orc.OracleUnit(C, D, T, F, warmup_frames=W, lloyd_iters=3, recluster_every=every)
    runs = 1
    for f in range(F):
        if u.ready and (f + 1) % every == 0:
            # state right before the frame that triggers the re-clustering
            R0, n0, a0 = u.centroids(), u.sizes(), u.assignments()
            dec = u.ingest(K[f])
            # replay: Eq. 3 for this frame, then warm-started rounds over all frames
            S = K[: f + 1].mean(axis=1)
            R1, n1 = R0.copy(), n0.copy()
            R1[dec.winner] = (n0[dec.winner] * R0[dec.winner] + S[f]) / (n0[dec.winner] + 1)
            n1[dec.winner] += 1
            a, R, n = _lloyd_brute(S, R1, n1, 3, False)
            runs += 1
            np.testing.assert_array_equal(u.assignments(), a)
            np.testing.assert_array_equal(u.sizes(), n)
            np.testing.assert_allclose(u.centroids()[n > 0], R[n > 0], rtol=1e-12, atol=1e-13)
        else:
            u.ingest(K[f])
    assert u.n_lloyd_runs == runs == 4      # init + re-clusterings at frames 8, 16, 24


def test_empty_cluster_keeps_representative_and_is_skipped():
    # two identical seeds: the second can never win (ties go to the lowest id)
    D, T = 4, 1
    x = np.array([1.0, 0.0, 0.0, 0.0])
    y = np.array([0.0, 1.0, 0.0, 0.0])
    frames = [x, x, y, y]             # W = 4, C = 3 -> seeds = frames 0, 1, 2
    u = orc.OracleUnit(3, D, T, 16, warmup_frames=4, lloyd_iters=2)
    for s in frames:
        u.ingest(s[None, :])
    np.testing.assert_array_equal(u.sizes(), [2, 0, 2])
    np.testing.assert_allclose(u.centroids()[1], x)     # kept its previous value
    # a new frame identical to the empty cluster's representative goes to cluster 0
    assert u.ingest(x[None, :]).winner == 0
    assert u.sizes()[1] == 0


def test_well_separated_scenes_recover_generator_labels():
    # C = number of scenes, tiny noise: clusters must coincide with the scenes
    wl = inputs.CONFIGS[0].scaled(n_frames=96, n_scenes=4, n_clusters=4, noise=0.02,
                                  drift=0.0, seed=77, warmup_frames=0)
    st = inputs.SceneStream(wl)
    by_scene = [list(np.nonzero(st.scene_of_frame == s)[0]) for s in range(4)]
    assert min(len(b) for b in by_scene) >= 2
    # warm-up of 8 frames = two per scene, so the strided seeds (frames 0,2,4,6) see
    # every scene once; the remaining frames follow in stream order
    order = [b.pop(0) for b in by_scene for _ in range(2)]
    order += sorted(f for b in by_scene for f in b)
    Kf = [inputs.unit_pages(st.frame(int(f))[0][None], 0, 0)[0] for f in order]
    u = orc.OracleUnit(4, wl.head_dim, wl.tokens_per_frame, len(order), lloyd_iters=4)
    for k in Kf:
        u.ingest(k)
    a = u.assignments()
    lab = st.scene_of_frame[np.array(order)]
    for s in range(4):
        assert len(set(a[lab == s])) == 1
    assert len(set(a)) == 4


# --------------------------------------------------------------------------
# O6: scoring
# --------------------------------------------------------------------------
def _filled_unit(seed=41, C=5, D=8, T=3, F=50, score_mode=0):
    K, _ = _stream(F, T, D, C, seed)
    u = orc.OracleUnit(C, D, T, F, lloyd_iters=4, score_mode=score_mode)
    for f in range(F):
        u.ingest(K[f])
    return u, K


def test_mean_query_is_mean_over_tokens_and_group():
    q = _rng(5).normal(size=(3, 6, 4))          # Tq=3, Hq=6, D=4; G=2
    for h in range(3):
        np.testing.assert_allclose(orc.mean_query(q, h, 2),
                                   q[:, 2 * h:2 * h + 2, :].reshape(-1, 4).mean(axis=0),
                                   rtol=1e-14, atol=1e-15)


def test_dot_score_is_mean_member_logit():
    u, K = _filled_unit(score_mode=1)
    qbar = _rng(6).normal(size=8)
    sc = u.score(qbar)
    a, S = u.assignments(), K.mean(axis=1)
    for j in range(u.C):
        if u.sizes()[j]:
            assert sc[j] == pytest.approx((S[a == j] @ qbar).mean(), rel=1e-11, abs=1e-12)


def test_cosine_score_matches_numpy_and_scale_invariance():
    u, _ = _filled_unit()
    qbar = _rng(7).normal(size=8)
    R, n = u.centroids(), u.sizes()
    want = (R @ qbar) / np.linalg.norm(R, axis=1)
    sc = u.score(qbar)
    np.testing.assert_allclose(sc[n > 0], want[n > 0], rtol=1e-12)
    # rescaling the query rescales all scores alike: the ranking cannot change
    ids1, _ = orc.select(sc, n, 3)
    ids2, _ = orc.select(u.score(3.7 * qbar), n, 3)
    np.testing.assert_array_equal(ids1, ids2)


def test_empty_cluster_scores_minus_inf():
    u = orc.OracleUnit(3, 4, 1, 16, warmup_frames=4, lloyd_iters=2)
    x = np.array([1.0, 0, 0, 0]); y = np.array([0, 1.0, 0, 0])
    for s in (x, x, y, y):
        u.ingest(s[None, :])
    sc = u.score(x)
    assert sc[1] == -np.inf and np.isfinite(sc[0]) and np.isfinite(sc[2])


# --------------------------------------------------------------------------
# O7: top-k selection vs full sort
# --------------------------------------------------------------------------
@pytest.mark.parametrize("seed", range(6))
def test_select_matches_full_lexsort(seed):
    r = _rng(100 + seed)
    C = 40
    score = np.round(r.normal(size=C), 1)        # rounding makes exact ties common
    sizes = r.integers(0, 3, size=C).astype(np.int32)
    for k in (1, 5, C, C + 7):
        ids, gap = orc.select(score, sizes, k)
        live = np.nonzero(sizes > 0)[0]
        order = live[np.lexsort((live, -score[live]))]      # score desc, id asc
        want = order[: min(k, len(live))]
        np.testing.assert_array_equal(ids, want)
        rest = np.setdiff1d(live, ids)
        if len(rest) and len(ids):
            assert score[rest].max() <= score[ids].min()
            a, b = score[ids[-1]], score[order[len(ids)]]
            assert gap == pytest.approx(abs(a - b) / max(abs(a), abs(b), 1e-30))
        else:
            assert gap == np.inf


# --------------------------------------------------------------------------
# O8: gather invariants
# --------------------------------------------------------------------------
def test_gather_is_union_of_whole_clusters_in_order():
    u, K = _filled_unit(C=6, F=70)
    a, n, T = u.assignments(), u.sizes(), u.T
    ids = np.array([4, 1, 3], dtype=np.int32)
    tok = u.gather(ids)
    assert len(tok) == T * n[ids].sum()
    assert len(np.unique(tok)) == len(tok) and tok.max() < 70 * T
    frames = tok.reshape(-1, T)
    np.testing.assert_array_equal(frames[:, 1:] - frames[:, :-1], 1)   # whole frames
    fr = frames[:, 0] // T
    want = np.concatenate([np.nonzero(a == j)[0] for j in ids])        # ids order, frames ascending
    np.testing.assert_array_equal(fr, want)
    # k = C: the retrieved set is every token exactly once
    allc = np.arange(6, dtype=np.int32)
    np.testing.assert_array_equal(np.sort(u.gather(allc)), np.arange(70 * T))


# --------------------------------------------------------------------------
# O9: attention
# --------------------------------------------------------------------------
def _dense_attention(q, K, V, h, G):
    """Textbook softmax attention over all tokens with scipy routines."""
    D = q.shape[-1]
    qq = q[:, h * G:(h + 1) * G, :]                       # [Tq][G][D]
    logits = np.einsum("tgd,nd->tgn", qq, K) / np.sqrt(D)
    return np.einsum("tgn,nd->tgd", softmax(logits, axis=-1), V), logsumexp(logits, axis=-1)


def test_attention_hand_worked_fixture():
    vals = {l.split()[0]: [float(x) for x in l.split()[1:]]
            for l in open(os.path.join(GOLDEN, "softmax_two_tokens.txt"))
            if l.strip() and not l.startswith("#")}
    q = np.array([[[2.0, 0, 0, 0]]])
    K = np.array([[1.0, 0, 0, 0], [0, 1.0, 0, 0]])
    V = np.array([[1.0, 0, 0, 0], [0, 0, 0, 3.0]])
    out, lse = orc.attend(q, K, V, np.array([0, 1]), 0, 1)
    np.testing.assert_allclose(out[0, 0], vals["out"], rtol=1e-15, atol=1e-16)
    np.testing.assert_allclose(lse[0, 0], vals["lse"][0], rtol=1e-15)


def test_full_selection_equals_dense_attention():
    u, K = _filled_unit(C=5, D=8, T=3, F=50)
    r = _rng(8)
    V = r.normal(size=(50, 3, 8))
    q = r.normal(size=(4, 6, 8))                          # Tq=4, Hq=6 -> Hkv=3, G=2
    ids, sc, tok, gap = u.retrieve(q, h=1, G=2, top_k=5)
    assert gap == np.inf and len(ids) == (u.sizes() > 0).sum()
    out, lse = orc.attend(q, K.reshape(-1, 8), V.reshape(-1, 8), tok, 1, 2)
    want, want_lse = _dense_attention(q, K.reshape(-1, 8), V.reshape(-1, 8), 1, 2)
    np.testing.assert_allclose(out, want, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(lse, want_lse, rtol=1e-12)


def test_attention_special_cases():
    r = _rng(9)
    N, D = 37, 8
    K, V = r.normal(size=(N, D)), r.normal(size=(N, D))
    q = r.normal(size=(2, 4, D))
    # one retrieved token: output is that token's value, lse its logit
    out, lse = orc.attend(q, K, V, np.array([5]), 1, 2)
    np.testing.assert_allclose(out, np.broadcast_to(V[5], out.shape), rtol=1e-14)
    np.testing.assert_allclose(lse, q[:, 2:4, :] @ K[5] / np.sqrt(D), rtol=1e-13)
    # a subset is attention over the subset only (checked with the dense routine)
    idx = np.array([3, 30, 7, 11, 19])
    out, lse = orc.attend(q, K, V, idx, 0, 2)
    want, wl_ = _dense_attention(q, K[idx], V[idx], 0, 2)
    np.testing.assert_allclose(out, want, rtol=1e-12, atol=1e-13)
    # order of the retrieved tokens does not matter
    out_p, lse_p = orc.attend(q, K, V, idx[::-1].copy(), 0, 2)
    np.testing.assert_allclose(out_p, out, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(lse_p, lse, rtol=1e-13)
    # log-sum-exp merge of two disjoint halves equals attention over the union
    a, b = idx[:2], idx[2:]
    oa, la = orc.attend(q, K, V, a, 0, 2)
    ob, lb = orc.attend(q, K, V, b, 0, 2)
    l = np.logaddexp(la, lb)
    merged = oa * np.exp(la - l)[..., None] + ob * np.exp(lb - l)[..., None]
    np.testing.assert_allclose(merged, out, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(l, lse, rtol=1e-13)
    # nothing retrieved
    out, lse = orc.attend(q, K, V, np.zeros(0, np.int32), 0, 2)
    assert (out == 0).all() and (lse == -np.inf).all()


def test_gqa_head_mapping():
    # query head hq reads KV head hq // G: give each KV head a distinct constant V
    r = _rng(10)
    N, D, G, Hkv = 9, 4, 3, 2
    K = r.normal(size=(N, D))
    q = r.normal(size=(1, G * Hkv, D))
    for h in range(Hkv):
        V = np.full((N, D), float(h + 1))
        out, _ = orc.attend(q, K, V, np.arange(N), h, G)
        np.testing.assert_allclose(out, h + 1.0, rtol=1e-14)
        # and the logits of head h*G+g use q[:, h*G+g]
        _, lse = orc.attend(q, K, V, np.arange(N), h, G)
        want = logsumexp(q[0, h * G:(h + 1) * G] @ K.T / np.sqrt(D), axis=-1)
        np.testing.assert_allclose(lse[0], want, rtol=1e-13)


# --------------------------------------------------------------------------
# whole pipeline on the tiny workload: invariants only (no printed values exist)
# --------------------------------------------------------------------------
def test_cfg0_pipeline_invariants():
    wl = inputs.CONFIGS[0]
    st = inputs.SceneStream(wl)
    Kall, Vall = st.frames(0, wl.n_frames)
    scene = st.draw_scene()
    q = st.question(scene, wl.question_tokens, tag=0)[0].to("cpu").double().numpy()
    for h in range(wl.n_kv_heads):
        K = inputs.unit_pages(Kall, 0, h)
        V = inputs.unit_pages(Vall, 0, h)
        u = orc.OracleUnit(wl.n_clusters, wl.head_dim, wl.tokens_per_frame, wl.n_frames)
        for f in range(wl.n_frames):
            u.ingest(K[f])
        assert u.sizes().sum() == wl.n_frames
        ids, sc, tok, gap = u.retrieve(q, h, wl.group, wl.top_k)
        assert len(ids) == wl.top_k and len(set(ids)) == wl.top_k
        assert len(tok) == wl.tokens_per_frame * u.sizes()[ids].sum()
        out, lse = orc.attend(q, K.reshape(-1, wl.head_dim), V.reshape(-1, wl.head_dim),
                              tok, h, wl.group)
        assert np.isfinite(out).all() and np.isfinite(lse).all()
        # attention output is a convex combination of the retrieved values
        Vs = V.reshape(-1, wl.head_dim)[tok]
        assert (out <= Vs.max(axis=0) + 1e-12).all() and (out >= Vs.min(axis=0) - 1e-12).all()


# --------------------------------------------------------------------------
# Self-adaptive maintainer (Sec. VI): Eq. 2, Eq. 4, Eq. 5, Split, Alg. 1
# --------------------------------------------------------------------------
BIG = 1e300


def _maint(mode=1, c_init=1, tau_min=BIG, tau_max=BIG, n0=8.0, split_iters=4, buf_max=8):
    return dict(mode=mode, c_init=c_init, tau_min=tau_min, tau_max=tau_max, n0=n0,
                split_iters=split_iters, buf_max=buf_max)


def test_eq4_hand_worked_fixture():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "eq4_running_variance.txt"))
            if l.strip() and not l.startswith("#")]
    u = orc.OracleUnit(2, 1, 1, 16, warmup_frames=2, lloyd_iters=2, maintainer=_maint())
    u.ingest(np.array([[1.0]]))
    u.ingest(np.array([[3.0]]))
    assert u.ready and u.sizes()[0] == 2
    np.testing.assert_allclose(u.centroids()[0], [2.0], atol=1e-15)
    np.testing.assert_allclose(u.variances()[0], 1.0, atol=1e-15)          # Eq. 2
    for x, r, var, n in rows:
        u.ingest(np.array([[float(x)]]))
        np.testing.assert_allclose(u.centroids()[0], [float(r)], rtol=1e-15)
        np.testing.assert_allclose(u.variances()[0], float(var), rtol=1e-14)
        assert u.sizes()[0] == int(n) and u.last_action == orc.ACT_ABSORB


def test_eq5_threshold_closed_forms():
    lo, hi, n0 = 0.7, 5.2, 12.0
    assert orc.tau(lo, hi, n0, 0.0) == hi                                   # empty cluster: tau_max
    np.testing.assert_allclose(orc.tau(lo, hi, n0, n0), lo + (hi - lo) / np.e, rtol=1e-15)
    np.testing.assert_allclose(orc.tau(lo, hi, n0, 2 * n0), lo + (hi - lo) / np.e ** 2, rtol=1e-15)
    assert abs(orc.tau(lo, hi, n0, 1e6) - lo) < 1e-300 or orc.tau(lo, hi, n0, 1e6) == lo
    vals = [orc.tau(lo, hi, n0, n) for n in range(0, 200)]
    assert all(a > b for a, b in zip(vals, vals[1:]))                       # relaxes towards tau_min as N grows
    # halving the distance to tau_min takes n0 * ln 2 members
    np.testing.assert_allclose(orc.tau(lo, hi, n0, n0 * np.log(2.0)) - lo, (hi - lo) / 2, rtol=1e-14)


def test_eq5_threshold_is_evaluated_at_the_size_before_the_insertion():
    """Alg. 1 tests the threshold (line 2) before the union (line 3): tau takes the cluster size
    without the new state.  Hand-worked fixture with tau_min != tau_max whose first row is absorbed
    at tau(|C|) and would be invalid at tau(|C| + 1)."""
    import math
    rows = [l.split() for l in open(os.path.join(GOLDEN, "eq5_threshold_before_insertion.txt"))
            if l.strip() and not l.startswith("#")]
    lo, hi, n0 = 1.0, 5.0, 2.0
    u = orc.OracleUnit(2, 1, 1, 16, warmup_frames=2, lloyd_iters=2,
                       maintainer=_maint(tau_min=lo, tau_max=hi, n0=n0))
    u.ingest(np.array([[1.0]]))
    u.ingest(np.array([[3.0]]))
    flips = 0
    for x, n_before, var, tau_n, tau_n1, verdict in rows:
        assert u.sizes()[0] == int(n_before)
        u.ingest(np.array([[float(x)]]))
        got_var, got_tau = u.last_threshold_test
        np.testing.assert_allclose(got_var, float(var), rtol=1e-14)
        np.testing.assert_allclose(got_tau, float(tau_n), rtol=1e-15)
        np.testing.assert_allclose(got_tau, lo + (hi - lo) * math.exp(-int(n_before) / n0), rtol=1e-15)
        assert (u.last_action == orc.ACT_ABSORB) == (verdict == "absorb")
        assert (float(var) <= float(tau_n)) == (verdict == "absorb")
        flips += (float(var) <= float(tau_n)) != (float(var) <= float(tau_n1))
        assert u.sizes()[0] == int(n_before) + 1      # (a 1-D cluster cannot be split: absorbed either way)
    assert flips >= 1                                  # the fixture does tell the two readings apart
    assert u.counters()["forced_absorb"] == 1


def test_deferred_insertion_moves_the_owners_statistics_but_not_its_size():
    """Alg. 1 line 1 runs before the case analysis: representative (Eq. 3) and variance (Eq. 4) of
    the assigned cluster move also when the state is then buffered (lines 7-10); membership and
    size do not.  Two deferred insertions in a row, compared with Eq. 3 / Eq. 4 in numpy."""
    r = _rng(30)
    u, K, ca, cb = _deferred_unit(r, n_a=10, n_b=0)
    S = u.summaries()
    n = 10
    rep = S.mean(axis=0)
    np.testing.assert_allclose(u.centroids()[0], rep, rtol=1e-13)
    var = u.variances()[0]            # Eq. 2 at the warm-up, Eq. 4 since (pinned by the Eq. 4 fixture)
    assert 0.0 < var < 2.0 and u.lazy_flags()[0] == 0
    for i in range(2):
        k_new = cb[None, :] + 0.2 * r.normal(size=(2, 8))
        s = k_new.mean(axis=0)
        u.ingest(k_new)
        assert u.last_action == orc.ACT_DEFER and u.n_buf == i + 1
        rep = (n * rep + s) / (n + 1)                                  # Eq. 3 with the size of the members
        var = (n * var + ((s - rep) ** 2).sum()) / (n + 1)             # Eq. 4
        np.testing.assert_allclose(u.centroids()[0], rep, rtol=1e-13, atol=1e-15)
        np.testing.assert_allclose(u.variances()[0], var, rtol=1e-13)
        got_var, got_tau = u.last_threshold_test
        np.testing.assert_allclose(got_var, var, rtol=1e-13)
        assert got_var > got_tau == 2.0
        assert u.sizes()[0] == n and u.assignments()[10 + i] == -2 and u.lazy_flags()[0] == 1
    # the owner's moved representative is what the next query scores
    q = r.normal(size=(1, 1, 8))
    ids, sc, tok, _ = u.retrieve_maintained(q, 0, 1, 3)
    np.testing.assert_allclose(sc[0], q[0, 0] @ rep / np.linalg.norm(rep), rtol=1e-13)


@pytest.mark.parametrize("score_mode", [0, 1])
def test_buffered_singletons_are_scored_like_clusters(score_mode):
    """Alg. 1 line 10 registers a buffered state as a singleton cluster: its representative is its
    own summary and its relevance follows the cluster formula -- (q . s)/|s|, or the plain dot
    product in score_mode 1 -- so that clusters and singletons rank on one scale (numpy)."""
    r = _rng(31 + score_mode)
    D, T, C = 8, 2, 6
    ca, cb = r.normal(size=D) * 3, r.normal(size=D) * 3
    K = np.stack([ca] * 10 + [cb] * 4)[:, None, :] + 0.2 * r.normal(size=(14, T, D))
    u = orc.OracleUnit(C, D, T, 64, warmup_frames=6, lloyd_iters=2, score_mode=score_mode,
                       maintainer=_maint(mode=2, c_init=1, tau_min=2.0, tau_max=2.0, buf_max=8))
    for f in range(14):
        u.ingest(K[f])
    assert u.n_buf == 4
    S, R = u.summaries(), u.centroids()
    q = r.normal(size=(3, 2, D))                        # 3 tokens, G = 2 heads on this KV head
    qbar = q.reshape(-1, D).mean(axis=0)
    fr, _ = u.buffer()
    want_single = S[fr] @ qbar
    want_cluster = R[0] @ qbar
    if score_mode == 0:
        want_single = want_single / np.linalg.norm(S[fr], axis=1)
        want_cluster = want_cluster / np.linalg.norm(R[0])
    k = 3
    ids, sc, tok, gap = u.retrieve_maintained(q, 0, 2, k)
    assert sc.shape == (C + 4,)
    np.testing.assert_allclose(sc[C:], want_single, rtol=1e-13)
    np.testing.assert_allclose(sc[0], want_cluster, rtol=1e-13)
    assert np.all(np.isneginf(sc[1:C]))
    # ranking over clusters and singletons together: full numpy sort, ties to the lower id
    cand = np.array([0] + [C + b for b in range(4)])
    val = np.concatenate([[want_cluster], want_single])
    order = cand[np.lexsort((cand, -val))][:k]
    np.testing.assert_array_equal(ids, order)
    # the two score modes differ by the norms only: a scaled copy of a state ranks differently
    if score_mode == 1:
        assert not np.allclose(want_single, want_single / np.linalg.norm(S[fr], axis=1))


def test_reset_and_reingest_equals_a_fresh_unit():
    """orc_unit_reset forgets frames, clusters and maintainer state: the same stream through a
    reset unit gives exactly the state of a new one (flat, maintainer in both modes, nested)."""
    K, _ = _stream(120, 2, 8, 6, seed=32, noise=0.4)
    part = (np.arange(120) // 7 % 3).astype(np.int32)
    variants = [dict(), dict(recluster_every=40),
                dict(maintainer=_maint(mode=1, c_init=3, tau_min=1.0, tau_max=3.0, n0=10.0)),
                dict(maintainer=_maint(mode=2, c_init=3, tau_min=1.0, tau_max=3.0, n0=10.0, buf_max=6)),
                dict(nested=3)]
    for kw in variants:
        def run(u):
            rq = _rng(33)
            for f in range(120):
                if kw.get("nested"):
                    u.ingest_nested(K[f], part)
                else:
                    u.ingest(K[f])
                if kw.get("maintainer", {}).get("mode") == 2 and f >= 6 and f % 25 == 0:
                    u.retrieve_maintained(rq.normal(size=(1, 1, 8)), 0, 1, 3)
            st = dict(a=u.assignments(), n=u.sizes(), r=u.centroids(), s=u.summaries(), runs=u.n_lloyd_runs)
            if kw.get("maintainer"):
                st.update(v=u.variances(), lz=u.lazy_flags(), res=u.resident_flags(), nb=u.n_buf,
                          ns=u.n_slots, buf=np.concatenate(u.buffer()), cnt=tuple(u.counters().values()))
            return st
        C = 12
        used = orc.OracleUnit(C, 8, 2, 120, lloyd_iters=3, **kw)
        first = run(used)
        used.reset()
        assert used.n_frames == 0 and not used.ready and used.sizes().sum() == 0
        again = run(used)
        fresh = run(orc.OracleUnit(C, 8, 2, 120, lloyd_iters=3, **kw))
        for key in fresh:
            np.testing.assert_array_equal(again[key], fresh[key], err_msg=f"{kw}: {key} after reset")
            np.testing.assert_array_equal(first[key], fresh[key], err_msg=f"{kw}: {key}")


def test_maintainer_with_unreachable_threshold_is_the_plain_online_rule():
    """With tau = 1e300 nothing is ever invalid: assignments, sizes and representatives must be
    those of the plain greedy rule with C = c_init (Sec. VI-A without refinement)."""
    K, _ = _stream(160, 3, 8, 5, seed=21)
    a = orc.OracleUnit(12, 8, 3, 160, lloyd_iters=4, maintainer=_maint(c_init=5))
    b = orc.OracleUnit(5, 8, 3, 160, lloyd_iters=4)
    for f in range(160):
        a.ingest(K[f]); b.ingest(K[f])
    assert a.n_slots == 5 and a.counters() == {"split_now": 0, "split_deferred": 0, "deferred": 0, "forced_absorb": 0}
    np.testing.assert_array_equal(a.assignments(), b.assignments())
    np.testing.assert_array_equal(a.sizes()[:5], b.sizes())
    np.testing.assert_array_equal(a.centroids()[:5], b.centroids())
    assert np.all(a.sizes()[5:] == 0)


def test_eq2_exact_variance_after_initial_clustering():
    K, _ = _stream(24, 4, 6, 3, seed=22)
    u = orc.OracleUnit(8, 6, 4, 24, warmup_frames=24, lloyd_iters=5, maintainer=_maint(c_init=3))
    for f in range(24):
        u.ingest(K[f])
    S, A, R = u.summaries(), u.assignments(), u.centroids()
    for j in range(3):
        mem = S[A == j]
        assert len(mem) == u.sizes()[j] > 0
        np.testing.assert_allclose(u.variances()[j], ((mem - R[j]) ** 2).sum(axis=1).mean(), rtol=1e-13)


def _split_brute_force(S, iters):
    """Two-means with cosine, seeds = the pair with the lowest mutual cosine (numpy)."""
    Cm = _cos_matrix(S, S)
    iu = np.triu_indices(len(S), 1)
    p = np.argmin(Cm[iu])                       # first minimum in (i, i') order
    ca, cb = S[iu[0][p]].copy(), S[iu[1][p]].copy()
    for _ in range(iters):
        side = (_cos_matrix(S, cb[None])[:, 0] > _cos_matrix(S, ca[None])[:, 0]).astype(int)
        if (side == 0).any():
            ca = S[side == 0].mean(axis=0)
        if (side == 1).any():
            cb = S[side == 1].mean(axis=0)
    return side


def test_split_matches_brute_force_two_means():
    """One cluster, the threshold trips on the first frame after warm-up: the members are then
    split; compare sides, sizes, Eq. 1 and Eq. 2 of both halves with numpy."""
    r = _rng(23)
    D, T, W = 6, 2, 14
    cent = r.normal(size=(2, D)) * 2.0
    K = cent[r.integers(0, 2, size=W + 1)][:, None, :] + 0.4 * r.normal(size=(W + 1, T, D))
    u = orc.OracleUnit(4, D, T, 32, warmup_frames=W, lloyd_iters=2,
                       maintainer=_maint(c_init=1, tau_min=1e-9, tau_max=1e-9, split_iters=3))
    for f in range(W + 1):
        u.ingest(K[f])
    assert u.last_action == orc.ACT_SPLIT and u.n_slots == 2 and u.counters()["split_now"] == 1
    S = u.summaries()
    side = _split_brute_force(S, 3)
    assert 0 < side.sum() < len(S)
    np.testing.assert_array_equal(u.assignments(), side)       # first seed's side keeps id 0
    for j in (0, 1):
        mem = S[side == j]
        assert u.sizes()[j] == len(mem)
        np.testing.assert_allclose(u.centroids()[j], mem.mean(axis=0), rtol=1e-13, atol=1e-15)
        np.testing.assert_allclose(u.variances()[j], ((mem - mem.mean(axis=0)) ** 2).sum(axis=1).mean(), rtol=1e-12)
    assert u.split_min_gap > 1e-6


def test_split_separates_two_scenes_and_followers_join_their_scene():
    r = _rng(24)
    D, T = 8, 3
    ca, cb = r.normal(size=D) * 3, r.normal(size=D) * 3
    frames = [ca] * 12 + [cb] * 10 + [ca] * 5
    K = np.stack(frames)[:, None, :] + 0.2 * r.normal(size=(len(frames), T, D))
    u = orc.OracleUnit(6, D, T, 64, warmup_frames=8, lloyd_iters=2,
                       maintainer=_maint(c_init=1, tau_min=2.0, tau_max=2.0))
    for f in range(len(frames)):
        u.ingest(K[f])
    A = u.assignments()
    assert u.n_slots == 2 and u.counters()["split_now"] == 1
    assert len(set(A[:12])) == 1 and len(set(A[12:22])) == 1 and A[0] != A[12]
    np.testing.assert_array_equal(A[22:], A[0])                # scene A returns: old cluster
    assert u.sizes()[A[0]] == 17 and u.sizes()[A[12]] == 10


def test_full_cluster_table_forces_absorption():
    K, _ = _stream(80, 2, 6, 8, seed=25, noise=0.5)
    u = orc.OracleUnit(3, 6, 2, 80, warmup_frames=4, lloyd_iters=2,
                       maintainer=_maint(c_init=2, tau_min=1e-9, tau_max=1e-9))
    for f in range(80):
        u.ingest(K[f])
    c = u.counters()
    assert u.n_slots == 3 and c["split_now"] == 1 and c["forced_absorb"] > 0
    A = u.assignments()
    assert A.min() >= 0 and A.max() <= 2 and u.sizes().sum() == 80


def _deferred_unit(r, n_a=10, n_b=4, buf_max=8, k_table=6):
    D, T = 8, 2
    ca, cb = r.normal(size=D) * 3, r.normal(size=D) * 3
    K = np.stack([ca] * n_a + [cb] * n_b)[:, None, :] + 0.2 * r.normal(size=(n_a + n_b, T, D))
    u = orc.OracleUnit(k_table, D, T, 64, warmup_frames=6, lloyd_iters=2,
                       maintainer=_maint(mode=2, c_init=1, tau_min=2.0, tau_max=2.0, buf_max=buf_max))
    for f in range(n_a + n_b):
        u.ingest(K[f])
    return u, K, ca, cb


def test_deferred_split_buffers_singletons_until_the_cluster_is_retrieved():
    """Alg. 1: nothing is resident before the first retrieval, so invalid insertions are buffered
    (lines 7-10), stay visible to retrieval as singletons, and the split happens when the flagged
    cluster is retrieved (lines 12-17)."""
    r = _rng(26)
    u, K, ca, cb = _deferred_unit(r)
    c = u.counters()
    assert c["split_now"] == 0 and c["split_deferred"] == 0 and c["deferred"] == 4 and u.n_buf == 4
    A = u.assignments()
    np.testing.assert_array_equal(A[:10], 0)
    np.testing.assert_array_equal(A[10:], -2)                  # -2 - owner: buffered on behalf of cluster 0
    assert u.lazy_flags()[0] == 1 and u.sizes()[0] == 10 and u.sizes()[0] + u.n_buf == 14
    fr, ow = u.buffer()
    np.testing.assert_array_equal(fr, [10, 11, 12, 13]); np.testing.assert_array_equal(ow, 0)
    # a query along a buffered state ranks that singleton first; k = 1 returns just its frame
    T, D, C = 2, 8, 6
    q = u.summaries()[11][None, None, :]
    ids, sc, tok, _ = u.retrieve_maintained(q, 0, 1, 1)
    np.testing.assert_array_equal(ids, [C + 1]); np.testing.assert_array_equal(tok, [11 * T, 11 * T + 1])
    assert u.n_buf == 4 and u.lazy_flags()[0] == 1              # owner not retrieved: still deferred
    # retrieving the flagged cluster materializes the split
    q = ca[None, None, :]
    ids, sc, tok, _ = u.retrieve_maintained(q, 0, 1, 1)
    np.testing.assert_array_equal(ids, [0])
    np.testing.assert_array_equal(tok, np.arange(10 * T))       # the query sees the cluster as it was
    assert u.n_buf == 0 and u.lazy_flags()[0] == 0 and u.counters()["split_deferred"] == 1 and u.n_slots == 2
    A = u.assignments()
    np.testing.assert_array_equal(A[:10], 0); np.testing.assert_array_equal(A[10:], 1)
    S = u.summaries()
    np.testing.assert_allclose(u.centroids()[1], S[10:].mean(axis=0), rtol=1e-13)
    np.testing.assert_allclose(u.variances()[1], ((S[10:] - S[10:].mean(axis=0)) ** 2).sum(axis=1).mean(), rtol=1e-12)
    # both halves are now resident: the next invalid insertion splits at once
    assert u.resident_flags()[0] == 1 and u.resident_flags()[1] == 1
    cc = r.normal(size=8) * 3
    for i in range(3):
        u.ingest(cc[None, :] + 0.2 * r.normal(size=(2, 8)))
    assert u.counters()["split_now"] == 1 and u.n_slots == 3


def test_deferred_buffer_overflow_is_absorbed():
    u, K, ca, cb = _deferred_unit(_rng(27), n_a=10, n_b=6, buf_max=2)
    c = u.counters()
    assert u.n_buf == 2 and c["deferred"] == 2 and c["forced_absorb"] == 4
    assert u.sizes()[0] == 14 and u.sizes()[0] + u.n_buf == 16


def test_maintainer_conserves_frames():
    K, _ = _stream(300, 2, 8, 9, seed=28, noise=0.4)
    for mode in (1, 2):
        u = orc.OracleUnit(24, 8, 2, 300, lloyd_iters=3,
                           maintainer=_maint(mode=mode, c_init=3, tau_min=1.5, tau_max=4.0, n0=10.0, buf_max=16))
        r = _rng(29)
        for f in range(300):
            u.ingest(K[f])
            if mode == 2 and f >= 6 and f % 37 == 0:
                u.retrieve_maintained(r.normal(size=(1, 1, 8)), 0, 1, 4)
            if u.ready:
                A = u.assignments()
                assert np.array_equal(np.bincount(A[A >= 0], minlength=24), u.sizes())
                assert (A < 0).sum() == u.n_buf and u.sizes().sum() + u.n_buf == f + 1
                assert np.all(u.sizes()[u.n_slots:] == 0)
        assert u.n_slots > 3


# --------------------------------------------------------------------------
# Retrieval augmentation (Sec. V-C): global representatives + local window
# --------------------------------------------------------------------------
def _aug_unit(seed, F=40, T=3, D=8, C=5):
    r = _rng(seed)
    K, _ = _stream(F, T, D, 4, seed=seed)
    V = r.normal(size=(F, T, D))
    u = orc.OracleUnit(C, D, T, F, lloyd_iters=3)
    for f in range(F):
        u.ingest(K[f])
    return u, K, V, r


def test_window_covering_the_stream_is_dense_attention():
    u, K, V, r = _aug_unit(31)
    F, T, D = 40, 3, 8
    q = r.normal(size=(2, 2, D))
    ids, _, _, _ = u.retrieve(q, 0, 2, 2)
    tok, Kx, Vx = orc.augmented_context(u, K, V, ids, window_frames=F + 5, global_reps=False)
    np.testing.assert_array_equal(tok, np.arange(F * T))       # every token once, nothing from the clusters
    out, lse = orc.attend(q, Kx, Vx, tok, 0, 2)
    logits = np.einsum("tgd,nd->tgn", q, K.reshape(-1, D)) / np.sqrt(D)
    np.testing.assert_allclose(out, np.einsum("tgn,nd->tgd", softmax(logits, axis=-1), V.reshape(-1, D)), rtol=1e-12)
    np.testing.assert_allclose(lse, logsumexp(logits, axis=-1), rtol=1e-12)


def test_window_frames_are_listed_once_and_last():
    u, K, V, r = _aug_unit(32)
    F, T, W = 40, 3, 6
    A = u.assignments()
    ids = np.array([A[F - 1], A[0]], dtype=np.int32) if A[F - 1] != A[0] else np.array([A[0]], dtype=np.int32)
    tok, _, _ = orc.augmented_context(u, K, V, ids, window_frames=W, global_reps=False)
    assert len(set(tok.tolist())) == len(tok)                   # no token twice
    np.testing.assert_array_equal(tok[-W * T:], np.arange((F - W) * T, F * T))
    want_frames = sorted(set(np.nonzero(np.isin(A[: F - W], ids))[0].tolist()) | set(range(F - W, F)))
    assert sorted(set((tok // T).tolist())) == want_frames
    plain = u.gather(ids)                                        # without the window: whole clusters
    assert set(plain.tolist()) <= set(tok.tolist())


def test_global_representatives_are_cluster_means_and_merge_by_lse():
    u, K, V, r = _aug_unit(33)
    F, T, D = 40, 3, 8
    q = r.normal(size=(3, 2, D))
    ids, _, tok_plain, _ = u.retrieve(q, 1, 1, 2)
    tok, Kx, Vx = orc.augmented_context(u, K, V, ids, window_frames=0, global_reps=True)
    A, n = u.assignments(), u.sizes()
    live = np.nonzero(n > 0)[0]
    P = len(live)
    np.testing.assert_array_equal(tok[: len(tok_plain)], tok_plain)
    np.testing.assert_array_equal(tok[len(tok_plain):], F * T + np.arange(P))
    for i, j in enumerate(live):
        np.testing.assert_allclose(Kx[F * T + i], K[A == j].reshape(-1, D).mean(axis=0), rtol=1e-12)   # Eq. 1 over member tokens
        np.testing.assert_allclose(Vx[F * T + i], V[A == j].reshape(-1, D).mean(axis=0), rtol=1e-12)
    # one softmax over the union == log-sum-exp merge of the two parts computed separately
    out, lse = orc.attend(q, Kx, Vx, tok, 1, 1)
    o1, l1 = orc.attend(q, Kx, Vx, tok[: len(tok_plain)], 1, 1)
    o2, l2 = orc.attend(q, Kx, Vx, tok[len(tok_plain):], 1, 1)
    w1, w2 = np.exp(l1 - np.logaddexp(l1, l2)), np.exp(l2 - np.logaddexp(l1, l2))
    np.testing.assert_allclose(out, o1 * w1[..., None] + o2 * w2[..., None], rtol=1e-12)
    np.testing.assert_allclose(lse, np.logaddexp(l1, l2), rtol=1e-12)


# --------------------------------------------------------------------------
# Nested visual-semantic hierarchy and two-stage retrieval (Sec. V-B, V-C)
# --------------------------------------------------------------------------
def _nested_stream(seed, F=96, T=2, D=8, Dv=6, n_visual=3, n_scenes=9):
    """Scene-structured keys plus visual embeddings whose classes group the scenes."""
    r = _rng(seed)
    K, labels = _stream(F, T, D, n_scenes, seed)
    r.shuffle(labels)                      # scenes interleaved in time: partitions are not contiguous runs
    centres = r.normal(size=(n_scenes, D))
    K = centres[labels][:, None, :] + 0.3 * r.normal(size=(F, T, D))
    cls = r.integers(0, n_visual, size=n_scenes)
    vc = 3.0 * r.normal(size=(n_visual, Dv))
    E = vc[cls[labels]] + 0.2 * r.normal(size=(F, Dv))
    return K, E, labels, cls[labels]


def _run_nested(K, E, P, C, W, iters=4, score_mode=0):
    F, T, D = K.shape
    vis = orc.OracleUnit(P, E.shape[1], 1, F, warmup_frames=W, lloyd_iters=iters)
    sem = orc.OracleUnit(C, D, T, F, warmup_frames=W, lloyd_iters=iters, score_mode=score_mode, nested=P)
    part = np.full(F, -1, dtype=np.int32)
    for f in range(F):
        vis.ingest(E[f][None, :])
        if vis.ready:
            part[: f + 1] = vis.assignments()
        sem.ingest_nested(K[f], part)
    return vis, sem


def test_nested_with_one_partition_is_the_flat_index():
    # special case: P = 1 puts every frame into the same partition, so seeding, K-means,
    # online assignment and the two-stage selection must reduce to the flat path
    K, E, _, _ = _nested_stream(61)
    F, T, D = K.shape
    flat = orc.OracleUnit(6, D, T, F, warmup_frames=18, lloyd_iters=4)
    for f in range(F):
        flat.ingest(K[f])
    _, sem = _run_nested(K, E, 1, 6, 18)
    np.testing.assert_array_equal(sem.assignments(), flat.assignments())
    np.testing.assert_array_equal(sem.centroids(), flat.centroids())
    q = _rng(62).normal(size=(3, 4, D))
    a = sem.retrieve_nested(q, 1, 2, 1, 3)
    ids, sc, tok, _ = flat.retrieve(q, 1, 2, 3)
    np.testing.assert_array_equal(a["ids"], ids)
    np.testing.assert_array_equal(a["scores"], sc)
    np.testing.assert_array_equal(a["tok_idx"], tok)


def test_nested_clusters_stay_inside_their_visual_partition():
    K, E, _, _ = _nested_stream(63)
    P, Cs = 3, 4
    vis, sem = _run_nested(K, E, P, P * Cs, 24)
    part, A = vis.assignments(), sem.assignments()
    np.testing.assert_array_equal(sem.partitions(), part)
    np.testing.assert_array_equal(A // Cs, part)                  # the nesting itself
    # sizes count the members, every frame is in exactly one cluster
    np.testing.assert_array_equal(sem.sizes(), np.bincount(A, minlength=P * Cs))


def test_nested_seeds_follow_the_partition_member_lists():
    # zero K-means rounds leave the seeds in place: slot j of partition p holds the summary of
    # the partition's member floor(j * np / L), L = min(Cs, np); slots beyond L stay empty
    K, E, _, _ = _nested_stream(64, F=40)
    F, T, D = K.shape
    P, Cs, W = 3, 5, 12
    vis = orc.OracleUnit(P, E.shape[1], 1, F, warmup_frames=W, lloyd_iters=4)
    for f in range(W):
        vis.ingest(E[f][None, :])
    part = vis.assignments().astype(np.int32)
    sem = orc.OracleUnit(P * Cs, D, T, F, warmup_frames=W, lloyd_iters=0, nested=P)
    for f in range(W):
        sem.ingest_nested(K[f], np.concatenate([part, [-1] * (F - W)]).astype(np.int32))
    assert sem.ready
    S = K[:W].mean(axis=1)
    R, n = sem.centroids(), sem.sizes()
    saw_short = False
    for p in range(P):
        mem = np.flatnonzero(part == p)
        L = min(Cs, len(mem))
        saw_short |= L < Cs
        for j in range(Cs):
            if j < L:
                np.testing.assert_allclose(R[p * Cs + j], S[mem[(j * len(mem)) // L]], rtol=0, atol=1e-15)
                assert n[p * Cs + j] == 1
            else:
                assert n[p * Cs + j] == 0
    assert saw_short        # the case of a partition with fewer members than ids is exercised


@pytest.mark.parametrize("seed", [65, 66])
def test_nested_online_assignment_is_argmax_over_the_partition_only(seed):
    K, E, _, _ = _nested_stream(seed)
    F, T, D = K.shape
    P, Cs, W = 3, 3, 18
    vis = orc.OracleUnit(P, E.shape[1], 1, F, warmup_frames=W, lloyd_iters=4)
    sem = orc.OracleUnit(P * Cs, D, T, F, warmup_frames=W, lloyd_iters=4, nested=P)
    part = np.full(F, -1, dtype=np.int32)
    crossed = 0
    for f in range(F):
        vis.ingest(E[f][None, :])
        if vis.ready:
            part[: f + 1] = vis.assignments()
        if sem.ready:
            R, n = sem.centroids(), sem.sizes()
            s = K[f].mean(axis=0)
            cos = _cos_matrix(s[None, :], np.where(n[:, None] > 0, R, 1.0))[0]
            cos[n == 0] = -np.inf
            inside = np.full_like(cos, -np.inf)
            lo = part[f] * Cs
            inside[lo: lo + Cs] = cos[lo: lo + Cs]
            want = int(np.argmax(inside))
            crossed += int(np.argmax(cos)) != want       # the restriction changes some decisions
            n_before = n[want]
            dec = sem.ingest_nested(K[f], part)
            assert dec.winner == want and sem.assignments()[f] == want
            # Eq. 3 on the winner, nothing else moves
            R2 = sem.centroids()
            np.testing.assert_allclose(R2[want], (n_before * R[want] + s) / (n_before + 1), rtol=1e-14)
            mask = np.arange(P * Cs) != want
            np.testing.assert_array_equal(R2[mask], R[mask])
        else:
            sem.ingest_nested(K[f], part)
    assert crossed > 0


def test_nested_lloyd_matches_brute_force_inside_each_partition():
    # the initial clustering equals an independent brute-force K-means run on each partition's
    # members alone (that is what "constrained within each visual cluster" means)
    K, E, _, _ = _nested_stream(67, F=60)
    F, T, D = K.shape
    P, Cs, W, iters = 3, 3, 36, 3
    vis, sem = _run_nested(K[:W], E[:W], P, P * Cs, W, iters=iters)
    part = vis.assignments()
    S = K[:W].mean(axis=1)
    for p in range(P):
        mem = np.flatnonzero(part == p)
        L = min(Cs, len(mem))
        R0 = np.stack([S[mem[(j * len(mem)) // L]] for j in range(L)])
        A, R, n = _lloyd_brute(S[mem], R0, np.ones(L, dtype=np.int64), iters, False)
        np.testing.assert_array_equal(sem.assignments()[mem] - p * Cs, A)
        np.testing.assert_allclose(sem.centroids()[p * Cs: p * Cs + L][n > 0], R[n > 0], rtol=1e-13)


def test_partition_representative_is_member_mean_and_weighted_centroid_mean():
    K, E, _, _ = _nested_stream(68)
    P, Cs = 3, 4
    vis, sem = _run_nested(K, E, P, P * Cs, 24)
    part = vis.assignments()
    S = K.mean(axis=1)
    R, n = sem.centroids(), sem.sizes()
    for p in range(P):
        rp, cnt = sem.partition_rep(p)
        assert cnt == int((part == p).sum())
        np.testing.assert_allclose(rp, S[part == p].mean(axis=0), rtol=1e-13)
        # Eq. 1 one level up: the partition's mean is the size-weighted mean of its clusters' means
        w = n[p * Cs:(p + 1) * Cs].astype(np.float64)
        np.testing.assert_allclose(rp, (w[:, None] * R[p * Cs:(p + 1) * Cs]).sum(axis=0) / w.sum(), rtol=1e-12)


@pytest.mark.parametrize("seed,score_mode", [(69, 0), (70, 1), (71, 0)])
def test_two_stage_retrieval_matches_brute_force(seed, score_mode):
    K, E, _, _ = _nested_stream(seed)
    F, T, D = K.shape
    P, Cs, top_p, k = 3, 4, 2, 3
    vis, sem = _run_nested(K, E, P, P * Cs, 24, score_mode=score_mode)
    part, A = vis.assignments(), sem.assignments()
    S = K.mean(axis=1)
    R, n = sem.centroids(), sem.sizes()
    q = _rng(seed + 100).normal(size=(2, 4, D))
    h, G = 1, 2
    qbar = q[:, h * G:(h + 1) * G].reshape(-1, D).mean(axis=0)
    # stage 1 with whole-array numpy
    PR = np.stack([S[part == p].mean(axis=0) for p in range(P)])
    ps = PR @ qbar if score_mode == 1 else (PR @ qbar) / np.linalg.norm(PR, axis=1)
    want_parts = np.lexsort((np.arange(P), -ps))[:top_p]
    # stage 2 over the clusters of those partitions
    cs = R @ qbar if score_mode == 1 else (R @ qbar) / np.where(n > 0, np.linalg.norm(R, axis=1), 1.0)
    cand = np.array([j for j in range(P * Cs) if n[j] > 0 and j // Cs in want_parts])
    order = cand[np.lexsort((cand, -cs[cand]))][:k]
    got = sem.retrieve_nested(q, h, G, top_p, k)
    np.testing.assert_array_equal(got["part_ids"], want_parts)
    np.testing.assert_allclose(got["part_scores"], ps, rtol=1e-12)
    np.testing.assert_array_equal(got["ids"], order)
    assert got["n_candidates"] == len(cand)
    assert set(np.flatnonzero(np.isfinite(got["scores"]))) == set(cand)
    np.testing.assert_allclose(got["scores"][cand], cs[cand], rtol=1e-12)
    # the gather is the members of the chosen clusters, clusters in selection order
    want_tok = np.concatenate([(np.flatnonzero(A == j)[:, None] * T + np.arange(T)).ravel() for j in order])
    np.testing.assert_array_equal(got["tok_idx"], want_tok)


def test_two_stage_with_all_partitions_is_the_flat_selection():
    K, E, _, _ = _nested_stream(72)
    P, Cs = 3, 4
    _, sem = _run_nested(K, E, P, P * Cs, 24)
    q = _rng(73).normal(size=(2, 4, K.shape[2]))
    got = sem.retrieve_nested(q, 0, 2, P, 5)
    ids, sc, tok, gap = sem.retrieve(q, 0, 2, 5)
    np.testing.assert_array_equal(got["ids"], ids)
    np.testing.assert_array_equal(got["scores"], sc)
    np.testing.assert_array_equal(got["tok_idx"], tok)
    assert got["gap_k"] == gap


def test_nested_hierarchy_rejects_bad_parameters():
    with pytest.raises(ValueError):
        orc.OracleUnit(10, 8, 2, 32, nested=3)            # C not a multiple of P
    with pytest.raises(ValueError):
        orc.OracleUnit(8, 8, 2, 32, recluster_every=8, nested=2)


def test_synthetic_visual_embeddings_group_scenes_by_class():
    wl = inputs.CONFIGS[0].scaled(visual_dim=16, n_visual=3, visual_noise=0.1)
    st = inputs.SceneStream(wl)
    E = st.embeddings(0, wl.n_frames).numpy().astype(np.float64)
    cls = st.visual_class_of_scene[st.scene_of_frame]
    C = _cos_matrix(E, E)
    same = cls[:, None] == cls[None, :]
    assert C[same].mean() > C[~same].mean() + 0.3
    # the K/V stream does not depend on the visual draws
    k0, _ = inputs.SceneStream(inputs.CONFIGS[0]).frame(5)
    k1, _ = st.frame(5)
    assert (k0 == k1).all()
