"""CPU model of the offloading tier's GPU working set and of the overlap-aware
prefetch (test infrastructure, like the rest of oracle/).

The paper keeps every cluster in CPU memory, moves whole clusters to the GPU when a
query selects them (Sec. V-A "Setup", Sec. V-C "Cluster Indexing") and keeps "only a
small working set" on the GPU; it does not name the replacement policy.  Reading
taken: least recently used at cluster granularity, the clusters of the call being
served never evicted, capacity counted in frame pages and in clusters.

The self-adaptive maintainer (Sec. VI) changes cluster membership under the cache:
a split hands part of a cached cluster's frames to a new cluster id.  The model
therefore keeps its state per FRAME (cached or not, time of last use, fetched ahead
or not) and derives everything cluster-level from the membership it is given at each
call: a cluster is resident if any of its frames is cached, complete if all are, and
its time of last use is the latest of its cached frames' -- so both halves of a split
cluster inherit the parent's recency without the model knowing about the split.
Equal times (the halves of a split) evict the lower cluster id first.

Sec. VII-B ("Overlap-Aware Prefetch"): while layer l runs, its query predicts the
top-K clusters of layer l+1 and they are fetched ahead; at layer l+1 the actual query
verifies the prediction and whatever is still missing is fetched on demand (the
completion step).  `prefetch_round` below is those three steps on top of the cache
model and an OracleUnit's scoring / selection.

Plain Python, no arithmetic of the method beyond set bookkeeping; pinned by a
hand-worked access trace (tests/golden/lru_cluster_cache_trace.txt) and invariants.
"""
from __future__ import annotations

from dataclasses import dataclass, field


class CapacityError(Exception):
    """The clusters of one call cannot be resident together."""


def membership_from_sizes(sizes) -> dict:
    """Clusters with the given frame counts as disjoint frame lists (cluster c owns frames
    1000*c .. 1000*c + sizes[c] - 1): enough when membership never changes except by growth."""
    items = sizes.items() if isinstance(sizes, dict) else enumerate(sizes)
    return {int(c): [1000 * int(c) + i for i in range(int(n))] for c, n in items}


def membership_from_assignments(assign, buf_frames=(), n_clusters=None) -> dict:
    """Cluster -> ascending frame list from a frame -> cluster array (negative = in no cluster);
    buffered singletons (Alg. 1, line 10) are entries n_clusters + b holding their one frame."""
    mem: dict = {}
    for f, c in enumerate(assign):
        if c >= 0:
            mem.setdefault(int(c), []).append(f)
    for b, f in enumerate(buf_frames):
        mem[int(n_clusters) + b] = [int(f)]
    return mem


@dataclass
class ClusterCacheModel:
    capacity_pages: int
    max_clusters: int
    cached: set = field(default_factory=set)         # frames whose page is in the GPU cache
    fstamp: dict = field(default_factory=dict)       # frame -> time of last use
    ahead: set = field(default_factory=set)          # frames fetched by a prefetch and not used since
    clock: int = 0
    hits: int = 0
    misses: int = 0
    evictions: int = 0
    pages_moved: int = 0
    prefetch_fetched: int = 0
    prefetch_useful: int = 0

    # -- cluster-level views of the per-frame state -----------------------------------
    def have(self, frames) -> int:
        return sum(1 for f in frames if f in self.cached)

    def directory(self, membership) -> dict:
        """cluster -> frames of it that are cached, for the clusters that have any"""
        out = {}
        for c, frames in membership.items():
            h = self.have(frames)
            if h:
                out[c] = h
        return out

    def stamp(self, frames) -> int:
        return max((self.fstamp.get(f, 0) for f in frames if f in self.cached), default=0)

    def used(self) -> int:
        return len(self.cached)

    def access(self, ids, membership, prefetch: bool = False):
        """Make clusters `ids` (in this order) resident.  membership: cluster -> frame list of
        EVERY cluster of the unit as it is now (what may be evicted is decided over all of them).
        Returns [(cluster, pages moved host-to-device), ...] for the clusters that needed data.
        A retrieval counts a hit for a cluster found complete and a miss otherwise; a prefetch
        counts neither, only what it had to fetch.  Raises CapacityError, leaving everything as
        it was, if the clusters of the call cannot be resident together."""
        ids = [int(c) for c in ids]
        if sum(len(membership[c]) for c in ids) > self.capacity_pages or len(ids) > max(self.max_clusters, 1):
            raise CapacityError(ids)
        moved = []
        for c in ids:
            frames = membership[c]
            want, have = len(frames), self.have(frames)
            done = have == want
            if prefetch:
                if not done:
                    self.prefetch_fetched += 1
                    self.ahead.update(frames)
            else:
                if done:
                    self.hits += 1
                    self.prefetch_useful += any(f in self.ahead for f in frames)
                else:
                    self.misses += 1
                self.ahead.difference_update(frames)
            while self.capacity_pages - len(self.cached) < want - have or \
                    (have == 0 and len(self.directory(membership)) >= self.max_clusters):
                victims = [j for j in sorted(membership) if j not in ids and self.have(membership[j]) > 0]
                victim = min(victims, key=lambda j: self.stamp(membership[j]))      # first lowest: lowest id on ties
                self.cached.difference_update(membership[victim])
                self.ahead.difference_update(membership[victim])
                self.evictions += 1
            self.clock += 1
            for f in frames:
                self.cached.add(f)
                self.fstamp[f] = self.clock
            self.pages_moved += want - have
            if want > have:
                moved.append((c, want - have))
            have = want
        return moved


def prefetch_round(unit, cache: ClusterCacheModel, q_proxy, q_actual, h: int, G: int, top_k: int,
                   prefetch_top_k: int = 0):
    """One layer transition of the overlap-aware prefetch (Sec. VII-B) for one unit.

    unit: the OracleUnit of (layer l+1, KV head h); q_proxy: layer l's query [Tq][Hq][D] (None: no
    prediction is made); q_actual: layer l+1's query.  Steps: (1) predicted = top-K of the unit's
    clusters under the proxy query (the best prefetch_top_k of them if that is > 0), fetched ahead;
    (2) actual = top-K under the actual query; (3) completion = the actual clusters that are not
    complete in the cache after (1), fetched on demand.  Returns dict(predicted, prefetched,
    actual, completion): id lists, `prefetched` / `completion` as [(cluster, pages)]."""
    membership = membership_from_assignments(unit.assignments())
    predicted, prefetched = [], []
    if q_proxy is not None:
        ids_p, _, _, _ = unit.retrieve(q_proxy, h, G, top_k)
        predicted = [int(c) for c in (ids_p[:prefetch_top_k] if prefetch_top_k > 0 else ids_p)]
        prefetched = cache.access(predicted, membership, prefetch=True)
    ids_a, _, _, _ = unit.retrieve(q_actual, h, G, top_k)
    actual = [int(c) for c in ids_a]
    completion = cache.access(actual, membership, prefetch=False)
    return dict(predicted=predicted, prefetched=prefetched, actual=actual, completion=completion)
