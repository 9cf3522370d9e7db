"""ctypes wrapper around the fp64 CPU oracle (test infrastructure).

Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this.  It never imports the HIP package.  The C source beside this file is
compiled with gcc on first use if no built library is present.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mosaic_oracle.c")
_LIB = os.path.join(_HERE, "libmosaic_oracle.so")


_LIB_SAN = os.path.join(_HERE, "libmosaic_oracle_san.so")


def build(force: bool = False, sanitize: bool = False) -> str:
    """Compile the oracle with gcc (-O2, strict IEEE: no fast-math, no FMA
    contraction) and return the library path.  sanitize=True builds a second
    library with AddressSanitizer and UndefinedBehaviorSanitizer (host code only),
    which lib() loads when MOSAIC_ORACLE_SANITIZED=1 is set in the environment."""
    out = _LIB_SAN if sanitize else _LIB
    if force or not os.path.exists(out) or os.path.getmtime(out) < os.path.getmtime(_SRC):
        extra = ["-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                 "-fno-omit-frame-pointer"] if sanitize else []
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fPIC", "-shared", *extra,
             "-o", out, _SRC, "-lm"])
    return out


def sanitizer_runtime() -> str | None:
    """Path of gcc's libasan.so (a process that loads the sanitized oracle needs it preloaded), or None."""
    try:
        p = subprocess.check_output(["gcc", "-print-file-name=libasan.so"], text=True).strip()
    except (OSError, subprocess.CalledProcessError):
        return None
    return p if os.path.isabs(p) and os.path.exists(p) else None


class _Decision(C.Structure):
    _fields_ = [("winner", C.c_int), ("runner_up", C.c_int),
                ("gap", C.c_double), ("sim", C.c_double)]


@dataclass
class Decision:
    winner: int
    runner_up: int
    gap: float
    sim: float


_lib = None
_dp = C.POINTER(C.c_double)
_ip = C.POINTER(C.c_int)


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build(sanitize=os.environ.get("MOSAIC_ORACLE_SANITIZED") == "1"))
        L.orc_unit_new.restype = C.c_void_p
        L.orc_unit_new.argtypes = [C.c_int] * 8
        L.orc_unit_free.argtypes = [C.c_void_p]
        L.orc_unit_reset.argtypes = [C.c_void_p]
        L.orc_summary.argtypes = [_dp, C.c_int, C.c_int, _dp]
        L.orc_unit_peek.argtypes = [C.c_void_p, _dp, C.POINTER(_Decision)]
        L.orc_unit_ingest.restype = C.c_int
        L.orc_unit_ingest.argtypes = [C.c_void_p, _dp, C.c_int, C.POINTER(_Decision)]
        L.orc_mean_query.argtypes = [_dp, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, _dp]
        L.orc_unit_score.argtypes = [C.c_void_p, _dp, _dp]
        L.orc_select.restype = C.c_int
        L.orc_select.argtypes = [_dp, _ip, C.c_int, C.c_int, _ip, _dp]
        L.orc_unit_gather.restype = C.c_int
        L.orc_unit_gather.argtypes = [C.c_void_p, _ip, C.c_int, _ip]
        L.orc_attend.argtypes = [_dp, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                 _dp, _dp, _ip, C.c_int, _dp, _dp]
        L.orc_unit_set_maintainer.restype = C.c_int
        L.orc_unit_set_maintainer.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_double, C.c_double,
                                              C.c_double, C.c_int, C.c_int]
        L.orc_unit_external_residency.argtypes = [C.c_void_p, C.c_int]
        L.orc_unit_set_resident.argtypes = [C.c_void_p, _ip]
        L.orc_tau.restype = C.c_double
        L.orc_tau.argtypes = [C.c_double] * 4
        L.orc_unit_retrieve_maintained.restype = C.c_int
        L.orc_unit_retrieve_maintained.argtypes = [C.c_void_p, _dp, C.c_int, _ip, _dp, _ip, _ip, _dp]
        L.orc_unit_set_nested.restype = C.c_int
        L.orc_unit_set_nested.argtypes = [C.c_void_p, C.c_int]
        L.orc_unit_ingest_nested.restype = C.c_int
        L.orc_unit_ingest_nested.argtypes = [C.c_void_p, _dp, _ip, C.c_int, C.POINTER(_Decision)]
        L.orc_unit_peek_nested.argtypes = [C.c_void_p, _dp, C.c_int, C.POINTER(_Decision)]
        L.orc_unit_partition_rep.restype = C.c_int
        L.orc_unit_partition_rep.argtypes = [C.c_void_p, C.c_int, _dp]
        L.orc_unit_retrieve_nested.restype = C.c_int
        L.orc_unit_retrieve_nested.argtypes = [C.c_void_p, _dp, C.c_int, C.c_int, _ip, _ip, _dp, _ip, _dp,
                                               _dp, _dp, _ip]
        L.orc_unit_part.restype = _ip
        L.orc_unit_part.argtypes = [C.c_void_p]
        for name, rt in (("orc_unit_n_slots", C.c_int), ("orc_unit_n_buf", C.c_int),
                         ("orc_unit_last_action", C.c_int), ("orc_unit_last_var", C.c_double),
                         ("orc_unit_last_tau", C.c_double), ("orc_unit_split_min_gap", C.c_double),
                         ("orc_unit_n_split_now", C.c_long), ("orc_unit_n_split_deferred", C.c_long),
                         ("orc_unit_n_deferred", C.c_long), ("orc_unit_n_forced_absorb", C.c_long),
                         ("orc_unit_var", _dp), ("orc_unit_lazy", _ip), ("orc_unit_resident", _ip),
                         ("orc_unit_buf_frame", _ip), ("orc_unit_buf_owner", _ip)):
            fn = getattr(L, name)
            fn.restype = rt
            fn.argtypes = [C.c_void_p]
        for name, rt in (("orc_unit_n_frames", C.c_int), ("orc_unit_ready", C.c_int),
                         ("orc_unit_n_lloyd_runs", C.c_int),
                         ("orc_unit_lloyd_min_gap", C.c_double),
                         ("orc_unit_centroids", _dp), ("orc_unit_sizes", _ip),
                         ("orc_unit_assign", _ip), ("orc_unit_summaries", _dp)):
            fn = getattr(L, name)
            fn.restype = rt
            fn.argtypes = [C.c_void_p]
        _lib = L
    return _lib


def _d(a: np.ndarray):
    assert a.dtype == np.float64 and a.flags.c_contiguous
    return a.ctypes.data_as(_dp)


def _i(a: np.ndarray):
    assert a.dtype == np.int32 and a.flags.c_contiguous
    return a.ctypes.data_as(_ip)


def f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def summary(k_frame: np.ndarray) -> np.ndarray:
    k_frame = f64(k_frame)
    T, D = k_frame.shape
    s = np.empty(D, dtype=np.float64)
    lib().orc_summary(_d(k_frame), T, D, _d(s))
    return s


def mean_query(q: np.ndarray, h: int, G: int) -> np.ndarray:
    q = f64(q)
    Tq, Hq, D = q.shape
    out = np.empty(D, dtype=np.float64)
    lib().orc_mean_query(_d(q), Tq, Hq, D, h, G, _d(out))
    return out


def select(score: np.ndarray, sizes: np.ndarray, k: int):
    """-> (ids kept, relative gap between last kept and first dropped)."""
    score = f64(score)
    sizes = np.ascontiguousarray(sizes, dtype=np.int32)
    Cn = score.shape[0]
    ids = np.empty(max(k, 1), dtype=np.int32)
    gap = C.c_double()
    m = lib().orc_select(_d(score), _i(sizes), Cn, k, _i(ids), C.byref(gap))
    return ids[:m].copy(), gap.value


def attend(q: np.ndarray, K: np.ndarray, V: np.ndarray, tok_idx: np.ndarray,
           h: int, G: int):
    """q [Tq][Hq][D], K/V [N][D] -> (out [Tq][G][D], lse [Tq][G])."""
    q, K, V = f64(q), f64(K), f64(V)
    tok_idx = np.ascontiguousarray(tok_idx, dtype=np.int32)
    Tq, Hq, D = q.shape
    out = np.empty((Tq, G, D), dtype=np.float64)
    lse = np.empty((Tq, G), dtype=np.float64)
    lib().orc_attend(_d(q), Tq, Hq, D, h, G, _d(K), _d(V), _i(tok_idx),
                     int(tok_idx.shape[0]), _d(out), _d(lse))
    return out, lse


ACT_NONE, ACT_ABSORB, ACT_SPLIT, ACT_DEFER, ACT_FORCED_ABSORB = range(5)


def tau(tau_min: float, tau_max: float, n0: float, size: float) -> float:
    """Size-adaptive threshold (Eq. 5)."""
    return lib().orc_tau(tau_min, tau_max, n0, size)


class OracleUnit:
    """Clustering state of one (layer, KV head).

    maintainer = dict(mode=1|2, c_init=.., tau_min=.., tau_max=.., n0=..,
    split_iters=.., buf_max=..) switches the self-adaptive maintainer on
    (Sec. VI): n_clusters is then the size of the cluster table, c_init the
    number of clusters the initial K-means builds.

    nested = P switches the nested visual-semantic hierarchy on (Sec. V-B):
    the C cluster ids are shared out over P visual partitions and every frame
    is ingested with the visual level's frame -> partition map (ingest_nested)."""

    def __init__(self, n_clusters: int, head_dim: int, tokens_per_frame: int,
                 max_frames: int, warmup_frames: int = 0, lloyd_iters: int = 8,
                 recluster_every: int = 0, score_mode: int = 0, maintainer: dict | None = None,
                 nested: int = 0):
        self.C, self.D, self.T = n_clusters, head_dim, tokens_per_frame
        self.max_frames = max_frames
        self._L = lib()
        self._u = self._L.orc_unit_new(n_clusters, head_dim, tokens_per_frame,
                                       max_frames, warmup_frames, lloyd_iters,
                                       recluster_every, score_mode)
        self.maintainer = maintainer
        self.buf_max = 0
        if maintainer:
            m = maintainer
            self.buf_max = int(m.get("buf_max", 0))
            rc = self._L.orc_unit_set_maintainer(self._u, int(m["mode"]), int(m["c_init"]),
                                                 float(m["tau_min"]), float(m["tau_max"]), float(m["n0"]),
                                                 int(m.get("split_iters", 4)), self.buf_max)
            if rc != 0:
                raise ValueError("bad maintainer parameters")
        self.n_part = int(nested)
        if self.n_part:
            if self._L.orc_unit_set_nested(self._u, self.n_part) != 0:
                raise ValueError("bad nested-hierarchy parameters")

    def __del__(self):
        if getattr(self, "_u", None):
            self._L.orc_unit_free(self._u)
            self._u = None

    def reset(self):
        self._L.orc_unit_reset(self._u)

    def peek(self, k_frame: np.ndarray) -> Decision:
        k_frame = f64(k_frame)
        d = _Decision()
        self._L.orc_unit_peek(self._u, _d(k_frame), C.byref(d))
        return Decision(d.winner, d.runner_up, d.gap, d.sim)

    def ingest(self, k_frame: np.ndarray, force: int = -1) -> Decision:
        k_frame = f64(k_frame)
        assert k_frame.shape == (self.T, self.D)
        d = _Decision()
        rc = self._L.orc_unit_ingest(self._u, _d(k_frame), force, C.byref(d))
        if rc != 0:
            raise RuntimeError("oracle unit is full")
        return Decision(d.winner, d.runner_up, d.gap, d.sim)

    @property
    def n_frames(self) -> int:
        return self._L.orc_unit_n_frames(self._u)

    @property
    def ready(self) -> bool:
        return bool(self._L.orc_unit_ready(self._u))

    @property
    def n_lloyd_runs(self) -> int:
        return self._L.orc_unit_n_lloyd_runs(self._u)

    @property
    def lloyd_min_gap(self) -> float:
        return self._L.orc_unit_lloyd_min_gap(self._u)

    def centroids(self) -> np.ndarray:
        p = self._L.orc_unit_centroids(self._u)
        return np.ctypeslib.as_array(p, shape=(self.C, self.D)).copy()

    def sizes(self) -> np.ndarray:
        p = self._L.orc_unit_sizes(self._u)
        return np.ctypeslib.as_array(p, shape=(self.C,)).copy()

    def assignments(self) -> np.ndarray:
        p = self._L.orc_unit_assign(self._u)
        return np.ctypeslib.as_array(p, shape=(self.max_frames,))[: self.n_frames].copy()

    def summaries(self) -> np.ndarray:
        p = self._L.orc_unit_summaries(self._u)
        return np.ctypeslib.as_array(p, shape=(self.max_frames, self.D))[: self.n_frames].copy()

    def score(self, qbar: np.ndarray) -> np.ndarray:
        qbar = f64(qbar)
        out = np.empty(self.C, dtype=np.float64)
        self._L.orc_unit_score(self._u, _d(qbar), _d(out))
        return out

    def gather(self, ids: np.ndarray) -> np.ndarray:
        ids = np.ascontiguousarray(ids, dtype=np.int32)
        out = np.empty(max(self.n_frames * self.T, 1), dtype=np.int32)
        m = self._L.orc_unit_gather(self._u, _i(ids), int(ids.shape[0]), _i(out))
        return out[:m].copy()

    # -- self-adaptive maintainer ------------------------------------------
    @property
    def n_slots(self) -> int:
        return self._L.orc_unit_n_slots(self._u)

    @property
    def n_buf(self) -> int:
        return self._L.orc_unit_n_buf(self._u)

    @property
    def last_action(self) -> int:
        return self._L.orc_unit_last_action(self._u)

    @property
    def last_threshold_test(self):
        """(variance after the update, threshold it was compared with)"""
        return self._L.orc_unit_last_var(self._u), self._L.orc_unit_last_tau(self._u)

    @property
    def split_min_gap(self) -> float:
        return self._L.orc_unit_split_min_gap(self._u)

    def counters(self) -> dict:
        L, u = self._L, self._u
        return {"split_now": L.orc_unit_n_split_now(u), "split_deferred": L.orc_unit_n_split_deferred(u),
                "deferred": L.orc_unit_n_deferred(u), "forced_absorb": L.orc_unit_n_forced_absorb(u)}

    def variances(self) -> np.ndarray:
        return np.ctypeslib.as_array(self._L.orc_unit_var(self._u), shape=(self.C,)).copy()

    def lazy_flags(self) -> np.ndarray:
        return np.ctypeslib.as_array(self._L.orc_unit_lazy(self._u), shape=(self.C,)).copy()

    def resident_flags(self) -> np.ndarray:
        return np.ctypeslib.as_array(self._L.orc_unit_resident(self._u), shape=(self.C,)).copy()

    def external_residency(self, on: bool = True):
        """The caller decides which clusters are "in GPU memory" (Alg. 1 line 4), e.g. from a cache model."""
        self._L.orc_unit_external_residency(self._u, int(on))

    def set_resident(self, flags):
        flags = np.ascontiguousarray(flags, dtype=np.int32)
        assert flags.shape == (self.C,)
        self._L.orc_unit_set_resident(self._u, _i(flags))

    def buffer(self):
        """-> (frames, owning clusters) of the buffered singletons"""
        nb = self.n_buf
        if nb == 0:
            return np.empty(0, np.int32), np.empty(0, np.int32)
        fr = np.ctypeslib.as_array(self._L.orc_unit_buf_frame(self._u), shape=(max(self.buf_max, 1),))
        ow = np.ctypeslib.as_array(self._L.orc_unit_buf_owner(self._u), shape=(max(self.buf_max, 1),))
        return fr[:nb].copy(), ow[:nb].copy()

    def retrieve_maintained(self, q: np.ndarray, h: int, G: int, top_k: int):
        """Retrieval with singletons visible and deferred splits materialized
        (Alg. 1): q [Tq][Hq][D] -> (ids, scores [C + n_buf], tok_idx, gap_k).
        Changes the unit's state in mode 2."""
        qbar = mean_query(q, h, G)
        nb = self.n_buf
        sc = np.full(self.C + max(self.buf_max, 1), -np.inf, dtype=np.float64)
        ids = np.empty(max(top_k, 1), dtype=np.int32)
        tok = np.empty(max(self.n_frames * self.T, 1), dtype=np.int32)
        n_tok = C.c_int()
        gap = C.c_double()
        m = self._L.orc_unit_retrieve_maintained(self._u, _d(qbar), top_k, _i(ids), _d(sc), _i(tok),
                                                 C.byref(n_tok), C.byref(gap))
        return ids[:m].copy(), sc[: self.C + nb].copy(), tok[: n_tok.value].copy(), gap.value

    # -- nested visual-semantic hierarchy ----------------------------------
    def ingest_nested(self, k_frame: np.ndarray, part: np.ndarray, force: int = -1) -> Decision:
        """part: the visual level's frame -> partition map, valid for frames
        0..n_frames once the warm-up completes (not read before)."""
        k_frame = f64(k_frame)
        assert k_frame.shape == (self.T, self.D)
        part = np.ascontiguousarray(part, dtype=np.int32)
        assert part.shape[0] > self.n_frames
        d = _Decision()
        rc = self._L.orc_unit_ingest_nested(self._u, _d(k_frame), _i(part), force, C.byref(d))
        if rc != 0:
            raise RuntimeError("oracle unit is full or not nested")
        return Decision(d.winner, d.runner_up, d.gap, d.sim)

    def peek_nested(self, k_frame: np.ndarray, p: int) -> Decision:
        k_frame = f64(k_frame)
        d = _Decision()
        self._L.orc_unit_peek_nested(self._u, _d(k_frame), int(p), C.byref(d))
        return Decision(d.winner, d.runner_up, d.gap, d.sim)

    def partitions(self) -> np.ndarray:
        p = self._L.orc_unit_part(self._u)
        return np.ctypeslib.as_array(p, shape=(self.max_frames,))[: self.n_frames].copy()

    def partition_rep(self, p: int):
        """-> (mean key summary of partition p's frames, frame count)"""
        rp = np.empty(self.D, dtype=np.float64)
        cnt = self._L.orc_unit_partition_rep(self._u, int(p), _d(rp))
        return rp, cnt

    def retrieve_nested(self, q: np.ndarray, h: int, G: int, top_p: int, top_k: int):
        """Two-stage retrieval (Sec. V-C): q [Tq][Hq][D] -> dict(part_ids, part_scores [P], gap_p,
        ids, scores [C] (-inf for empty or pruned clusters), gap_k, n_candidates, tok_idx)."""
        qbar = mean_query(q, h, G)
        P = self.n_part
        part_ids = np.empty(max(top_p, 1), dtype=np.int32)
        part_sc = np.empty(P, dtype=np.float64)
        ids = np.empty(max(top_k, 1), dtype=np.int32)
        sc = np.empty(self.C, dtype=np.float64)
        n_pk, n_cand = C.c_int(), C.c_int()
        gap_p, gap_k = C.c_double(), C.c_double()
        m = self._L.orc_unit_retrieve_nested(self._u, _d(qbar), top_p, top_k, _i(part_ids), C.byref(n_pk),
                                             _d(part_sc), _i(ids), _d(sc), C.byref(gap_p), C.byref(gap_k),
                                             C.byref(n_cand))
        ids = ids[:m].copy()
        return dict(part_ids=part_ids[: n_pk.value].copy(), part_scores=part_sc, gap_p=gap_p.value,
                    ids=ids, scores=sc, gap_k=gap_k.value, n_candidates=n_cand.value,
                    tok_idx=self.gather(ids))

    # -- the whole query side for this unit --------------------------------
    def retrieve(self, q: np.ndarray, h: int, G: int, top_k: int):
        """q [Tq][Hq][D] -> (ids, scores, tok_idx, gap_k)."""
        qbar = mean_query(q, h, G)
        sc = self.score(qbar)
        ids, gap = select(sc, self.sizes(), top_k)
        return ids, sc, self.gather(ids), gap


def augmented_context(unit: "OracleUnit", K_unit: np.ndarray, V_unit: np.ndarray, ids: np.ndarray,
                      window_frames: int, global_reps: bool):
    """Retrieval augmentation (Sec. V-C): what attention runs over besides the retrieved clusters.

    K_unit, V_unit [F][T][D] of this unit.  Returns (tok_idx, K_ext, V_ext): token indices into
    K_ext / V_ext [N + P][D], the unit's N = F*T real tokens followed by P pseudo tokens.
      * local window: all tokens of the `window_frames` most recent frames, after the clusters,
        ascending; a window frame that belongs to a selected cluster is listed with the window only,
        so every real token is attended once (the paper does not say how overlaps are treated);
      * global representatives: one pseudo token per non-empty cluster, in cluster order: key = the
        cluster's representative (Eq. 1), value = the mean of its members' value vectors (the paper
        keeps "the representatives of all clusters"; values follow the keys' frame->cluster map).
    Plain numpy: the definition written out."""
    K_unit, V_unit = f64(K_unit), f64(V_unit)
    F, T, D = unit.n_frames, unit.T, unit.D
    A = unit.assignments()
    w0 = max(0, F - int(window_frames))
    tok = []
    for j in ids:
        for f in range(w0):
            if A[f] == j:
                tok.extend(range(f * T, (f + 1) * T))
    for f in range(w0, F):
        tok.extend(range(f * T, (f + 1) * T))
    Kx, Vx = K_unit[:F].reshape(F * T, D), V_unit[:F].reshape(F * T, D)
    if global_reps:
        R, n = unit.centroids(), unit.sizes()
        keys, vals = [], []
        for j in range(unit.C):
            if n[j] > 0:
                keys.append(R[j])
                vals.append(V_unit[:F][A == j].reshape(-1, D).mean(axis=0))
        P = len(keys)
        if P:
            Kx = np.concatenate([Kx, np.stack(keys)])
            Vx = np.concatenate([Vx, np.stack(vals)])
            tok.extend(range(F * T, F * T + P))
    return np.asarray(tok, dtype=np.int32), Kx, Vx
