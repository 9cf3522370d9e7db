"""Pins for the CPU model of the offloading tier's GPU working set and of the overlap-aware
prefetch (oracle/cache_model.py): a hand-worked access trace, invariants under random traces,
and the predict / verify / complete steps of Sec. VII-B on a small clustered stream."""
import os

import numpy as np
import pytest

from oracle import cache_model as cm
from oracle import mosaic_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _pairs(text):
    return {} if text.strip() in ("-", "refused") else {int(a): int(b) for a, b in (x.split(":") for x in text.split())}


def test_hand_worked_lru_trace():
    sizes = {0: 4, 1: 3, 2: 5, 3: 2, 4: 6}
    m = cm.ClusterCacheModel(capacity_pages=10, max_clusters=3)
    for line in open(os.path.join(GOLDEN, "lru_cluster_cache_trace.txt")):
        if not line.strip() or line.startswith("#"):
            continue
        head, moved, counts, resident = [x.strip() for x in line.split("|")]
        step, op, ids = head.split()
        ids = [int(x) for x in ids.split(",")]
        if step == "6":
            sizes[2] = 6
        mem = cm.membership_from_sizes(sizes)
        if moved == "refused":
            before = (set(m.cached), dict(m.fstamp), m.hits, m.misses, m.evictions, m.pages_moved)
            with pytest.raises(cm.CapacityError):
                m.access(ids, mem, prefetch=(op == "prefetch"))
            assert before == (set(m.cached), dict(m.fstamp), m.hits, m.misses, m.evictions, m.pages_moved)
        else:
            got = m.access(ids, mem, prefetch=(op == "prefetch"))
            assert dict(got) == _pairs(moved), f"step {step}: moved {got}"
        want = [int(x) for x in counts.split()]
        assert [m.hits, m.misses, m.evictions, m.prefetch_fetched, m.prefetch_useful, m.pages_moved] == want, f"step {step}"
        assert m.directory(mem) == _pairs(resident), f"step {step}: resident {m.directory(mem)}"


@pytest.mark.parametrize("seed", range(4))
def test_cache_model_invariants_on_random_traces(seed):
    r = np.random.Generator(np.random.PCG64(100 + seed))
    C, cap, maxc, k = 12, 40, 5, 3
    sizes = r.integers(1, 9, size=C)
    m = cm.ClusterCacheModel(cap, maxc)
    calls = 0
    for step in range(300):
        if step % 17 == 0:
            sizes[r.integers(0, C)] += 1                   # the stream keeps growing
        ids = [int(x) for x in r.choice(C, size=k, replace=False)]
        pre = r.random() < 0.3
        before_moved = m.pages_moved
        mem = cm.membership_from_sizes(sizes)
        try:
            moved = m.access(ids, mem, prefetch=pre)
        except cm.CapacityError:
            assert sum(sizes[c] for c in ids) > cap
            continue
        calls += not pre
        d = m.directory(mem)
        assert m.used() <= cap and len(d) <= maxc and m.used() == sum(d.values())
        assert all(d[c] == sizes[c] for c in ids)          # what was asked for is resident, in full
        assert m.pages_moved - before_moved == sum(p for _, p in moved)
        assert all(d[c] <= sizes[c] for c in d)
    assert m.hits + m.misses == calls * k
    assert m.prefetch_useful <= m.prefetch_fetched
    assert m.evictions > 0 and m.hits > 0


def _unit(seed=7, F=90, T=2, D=8, C=6):
    r = np.random.Generator(np.random.PCG64(seed))
    centres = r.normal(size=(5, D)) * 2
    labels = np.sort(r.integers(0, 5, size=F))
    K = centres[labels][:, None, :] + 0.3 * r.normal(size=(F, T, D))
    u = orc.OracleUnit(C, D, T, F, lloyd_iters=4)
    for f in range(F):
        u.ingest(K[f])
    return u, centres, r


def test_prefetch_round_predicts_verifies_and_completes():
    """Sec. VII-B: predicted = top-K under the proxy query; whatever of the actual top-K is still
    missing afterwards is the completion set; a perfect proxy leaves nothing to complete and every
    prefetched cluster is then used; no proxy means every actual cluster is fetched on demand."""
    u, centres, r = _unit()
    sizes = u.sizes()
    k = 3
    q_a = centres[1][None, None, :] + 0.1 * r.normal(size=(1, 1, 8))
    q_far = -centres[1][None, None, :]
    # perfect proxy
    c1 = cm.ClusterCacheModel(int(sizes.sum()), 6)
    out = cm.prefetch_round(u, c1, q_a, q_a, 0, 1, k)
    assert out["predicted"] == out["actual"] and out["completion"] == []
    assert [c for c, _ in out["prefetched"]] == out["actual"]
    assert c1.prefetch_fetched == k == c1.prefetch_useful and c1.hits == k and c1.misses == 0
    # no proxy: all on demand
    c2 = cm.ClusterCacheModel(int(sizes.sum()), 6)
    out2 = cm.prefetch_round(u, c2, None, q_a, 0, 1, k)
    assert out2["predicted"] == [] and [c for c, _ in out2["completion"]] == out2["actual"] == out["actual"]
    assert c2.misses == k and c2.prefetch_fetched == 0
    # an unrelated proxy: completion = actual minus predicted, set arithmetic on the oracle's selections
    c3 = cm.ClusterCacheModel(int(sizes.sum()), 6)
    out3 = cm.prefetch_round(u, c3, q_far, q_a, 0, 1, k)
    ids_far = [int(c) for c in u.retrieve(q_far, 0, 1, k)[0]]
    assert out3["predicted"] == ids_far
    assert [c for c, _ in out3["completion"]] == [c for c in out3["actual"] if c not in ids_far]
    assert c3.prefetch_useful == len(set(ids_far) & set(out3["actual"]))
    assert c3.pages_moved == sum(int(sizes[c]) for c in set(ids_far) | set(out3["actual"]))
    # only the best prefetch_top_k predictions are fetched ahead
    c4 = cm.ClusterCacheModel(int(sizes.sum()), 6)
    out4 = cm.prefetch_round(u, c4, q_a, q_a, 0, 1, k, prefetch_top_k=1)
    assert out4["predicted"] == out["actual"][:1] and [c for c, _ in out4["completion"]] == out["actual"][1:]


def test_a_split_hands_residency_and_recency_to_both_halves():
    """Membership changes under the cache (Sec. VI splits): the model's state is per frame, so the
    halves of a split cluster are resident as far as their frames are, inherit the parent's time of
    last use (the lower id goes first when both are the oldest), and a half that received an uncached
    frame is incomplete: a miss that moves only that frame."""
    m = cm.ClusterCacheModel(capacity_pages=12, max_clusters=4)
    mem = {0: [0, 1, 2, 3, 4, 5], 1: [10, 11, 12], 2: [20, 21]}
    m.access([0], mem); m.access([1], mem); m.access([2], mem)           # times 1, 2, 3; 11 pages
    assert m.directory(mem) == {0: 6, 1: 3, 2: 2}
    # cluster 0 splits into 0 = {0, 1, 2} and 3 = {3, 4, 5, 30}; frame 30 is new and not cached
    mem = {0: [0, 1, 2], 1: [10, 11, 12], 2: [20, 21], 3: [3, 4, 5, 30]}
    assert m.directory(mem) == {0: 3, 1: 3, 2: 2, 3: 3}
    assert m.stamp(mem[0]) == m.stamp(mem[3]) == 1
    moved = m.access([3], mem)                                           # incomplete: one page moves, a miss
    assert moved == [(3, 1)] and m.misses == 4 and m.hits == 0 and m.used() == 12
    # a new cluster of 4 frames: 4 clusters are resident and no page is free, the oldest goes: that is
    # cluster 0 (time 1); then 1 (time 2) for the space
    mem[4] = [40, 41, 42, 43]
    moved = m.access([4], mem)
    assert moved == [(4, 4)] and m.evictions == 2
    assert m.directory(mem) == {2: 2, 3: 4, 4: 4}
