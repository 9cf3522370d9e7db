"""CPU model of the offloading tier's GPU working set and of the overlap-aware
prefetch (test infrastructure, like the rest of oracle/).

The paper keeps every cluster in CPU memory, moves whole clusters to the GPU when a
query selects them (Sec. V-A "Setup", Sec. V-C "Cluster Indexing") and keeps "only a
small working set" on the GPU; it does not name the replacement policy.  Reading
taken: least recently used at cluster granularity, the clusters of the call being
served never evicted, capacity counted in frame pages and in clusters.

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


@dataclass
class ClusterCacheModel:
    capacity_pages: int
    max_clusters: int
    pages: dict = field(default_factory=dict)        # cluster -> pages resident
    stamp: dict = field(default_factory=dict)        # cluster -> time of last use
    by_prefetch: dict = field(default_factory=dict)  # cluster -> fetched ahead and not used yet
    clock: int = 0
    hits: int = 0
    misses: int = 0
    evictions: int = 0
    pages_moved: int = 0
    prefetch_fetched: int = 0
    prefetch_useful: int = 0

    def used(self) -> int:
        return sum(self.pages.values())

    def complete(self, c: int, sizes) -> bool:
        return c in self.pages and self.pages[c] == int(sizes[c])

    def access(self, ids, sizes, prefetch: bool = False):
        """Make clusters `ids` (in this order) resident; sizes[c] = frames of cluster c now.
        Returns [(cluster, pages moved host-to-device), ...] for the clusters that needed data.
        A retrieval counts a hit for a cluster found complete and a miss otherwise; a prefetch
        counts neither, only what it had to fetch.  Raises CapacityError, leaving everything as
        it was, if the clusters of the call cannot be resident together."""
        ids = [int(c) for c in ids]
        if sum(int(sizes[c]) for c in ids) > self.capacity_pages or len(ids) > max(self.max_clusters, 1):
            raise CapacityError(ids)
        moved = []
        for c in ids:
            want = int(sizes[c])
            have = self.pages.get(c, 0)
            done = c in self.pages and have == want
            if prefetch:
                if not done:
                    self.prefetch_fetched += 1
                    self.by_prefetch[c] = True
            else:
                if done:
                    self.hits += 1
                    self.prefetch_useful += bool(self.by_prefetch.get(c))
                else:
                    self.misses += 1
                self.by_prefetch[c] = False
            while self.capacity_pages - self.used() < want - have or \
                    (c not in self.pages and len(self.pages) >= self.max_clusters):
                victim = min((j for j in self.pages if j not in ids), key=lambda j: self.stamp[j])
                del self.pages[victim]
                self.by_prefetch[victim] = False
                self.evictions += 1
            self.pages[c] = want
            self.clock += 1
            self.stamp[c] = self.clock
            self.pages_moved += want - have
            if want > have:
                moved.append((c, want - have))
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
    sizes = unit.sizes()
    predicted, prefetched = [], []
    if q_proxy is not None:
        ids_p, _, _, _ = unit.retrieve(q_proxy, h, G, top_k)
        predicted = [int(c) for c in (ids_p[:prefetch_top_k] if prefetch_top_k > 0 else ids_p)]
        prefetched = cache.access(predicted, sizes, prefetch=True)
    ids_a, _, _, _ = unit.retrieve(q_actual, h, G, top_k)
    actual = [int(c) for c in ids_a]
    completion = cache.access(actual, sizes, prefetch=False)
    return dict(predicted=predicted, prefetched=prefetched, actual=actual, completion=completion)
