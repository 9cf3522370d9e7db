"""Thin ctypes binding of libmosaic (argument marshalling only).

Every step of the path runs in the HIP kernels behind the C ABI declared in
include/mosaic.h; PyTorch supplies device memory (the arena, inputs, outputs)
and the stream.  There is no CPU fallback: if the built library is missing the
import of the library fails with an error that says how to build it.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmosaic.so")

OK, EINVAL, ENOMEM, ECAPACITY, ENOTREADY, EHIP = 0, -1, -2, -3, -4, -5
FP32, BF16 = 0, 1
TIER_HBM, TIER_HOST = 0, 1
ATTEND_AUTO, ATTEND_VALU, ATTEND_MFMA = 0, 1, 2
MAINT_OFF, MAINT_EAGER, MAINT_DEFERRED = 0, 1, 2
_STATUS = {0: "OK", -1: "EINVAL", -2: "ENOMEM", -3: "ECAPACITY", -4: "ENOTREADY", -5: "EHIP"}

EXPORTS = (
    "mosaic_host_alloc", "mosaic_host_free", "mosaic_workspace_size", "mosaic_create", "mosaic_destroy", "mosaic_reset",
    "mosaic_ingest_frame", "mosaic_retrieve", "mosaic_prefetch", "mosaic_attend", "mosaic_attend_static",
    "mosaic_get_assignments", "mosaic_get_centroids", "mosaic_get_summaries", "mosaic_get_maintainer",
    "mosaic_decode_step", "mosaic_ingest_frame_visual", "mosaic_ingest_join", "mosaic_get_partitions", "mosaic_get_partition_selection",
    "mosaic_get_selection", "mosaic_get_stats", "mosaic_get_cache_directory", "mosaic_profile_enable",
    "mosaic_profile_read", "mosaic_calibration_copy", "mosaic_last_error",
)


class MosaicError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"{_STATUS.get(code, code)}: {text}")
        self.code = code


class Config(C.Structure):
    _fields_ = [
        ("n_layers", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
        ("head_dim", C.c_int32), ("tokens_per_frame", C.c_int32), ("max_frames", C.c_int32),
        ("n_clusters", C.c_int32), ("top_k", C.c_int32), ("kv_dtype", C.c_int32),
        ("warmup_frames", C.c_int32), ("lloyd_iters", C.c_int32),
        ("recluster_every", C.c_int32), ("score_mode", C.c_int32),
        ("max_q_tokens", C.c_int32), ("attend_impl", C.c_int32), ("tier", C.c_int32),
        ("dev_arena", C.c_void_p), ("dev_arena_bytes", C.c_size_t), ("stream", C.c_void_p),
        ("slab_frames", C.c_int32), ("cache_pages_per_unit", C.c_int32),
        ("cache_fraction", C.c_float), ("decode_fused_max_mib", C.c_int32),
        ("host_arena", C.c_void_p), ("host_arena_bytes", C.c_size_t),
        ("maint_mode", C.c_int32), ("init_clusters", C.c_int32), ("split_iters", C.c_int32),
        ("buffer_max", C.c_int32), ("tau_min", C.c_double), ("tau_max", C.c_double),
        ("tau_n0", C.c_double),
        ("aug_global_reps", C.c_int32), ("aug_window_frames", C.c_int32),
        ("prefetch_top_k", C.c_int32), ("n_partitions", C.c_int32),
        ("visual_dim", C.c_int32), ("top_partitions", C.c_int32),
        ("ingest_overlap", C.c_int32),
    ]


class Stats(C.Structure):
    _fields_ = [
        ("frames_ingested", C.c_int64), ("lloyd_runs", C.c_int64),
        ("retrieve_calls", C.c_int64), ("attend_calls", C.c_int64),
        ("kv_bytes_stored", C.c_int64), ("ready", C.c_int32), ("attend_impl", C.c_int32),
        ("last_n_splits", C.c_int32), ("last_decode_fused", C.c_int32),
        ("cache_hits", C.c_int64), ("cache_misses", C.c_int64),
        ("h2d_bytes", C.c_int64), ("h2d_copies", C.c_int64), ("h2d_busy_ms", C.c_double),
        ("prefetch_calls", C.c_int64), ("prefetch_fetched", C.c_int64), ("prefetch_useful", C.c_int64),
        ("splits_immediate", C.c_int64), ("splits_deferred", C.c_int64),
        ("deferred_inserts", C.c_int64), ("forced_absorbs", C.c_int64), ("sync_timeouts", C.c_int64),
    ]


_lib = None


def load_library():
    """dlopen the in-tree libmosaic.so; fails loudly when it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2604_10060_amd.build` "
            "(hipcc, gfx950).  There is no fallback path.")
    L = C.CDLL(LIB_PATH)
    vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
    L.mosaic_host_alloc.argtypes = [sz, C.POINTER(vp)]
    L.mosaic_host_free.argtypes = [vp]
    L.mosaic_workspace_size.argtypes = [C.POINTER(Config), C.POINTER(sz), C.POINTER(sz)]
    L.mosaic_create.argtypes = [C.POINTER(Config), C.POINTER(vp)]
    L.mosaic_destroy.argtypes = [vp]
    L.mosaic_reset.argtypes = [vp]
    L.mosaic_ingest_frame.argtypes = [vp, vp, vp, i32]
    L.mosaic_ingest_frame_visual.argtypes = [vp, vp, vp, vp, i32]
    L.mosaic_ingest_join.argtypes = [vp]
    L.mosaic_get_partitions.argtypes = [vp, vp, vp, vp, vp, vp]
    L.mosaic_get_partition_selection.argtypes = [vp, i32, vp, vp, vp]
    L.mosaic_retrieve.argtypes = [vp, i32, vp, i32]
    L.mosaic_attend.argtypes = [vp, i32, vp, i32, vp, vp]
    L.mosaic_attend_static.argtypes = [vp, i32, vp, i32, vp, vp]
    L.mosaic_prefetch.argtypes = [vp, i32, vp, i32]
    L.mosaic_decode_step.argtypes = [vp, i32, vp, i32, vp, vp]
    L.mosaic_get_assignments.argtypes = [vp, vp]
    L.mosaic_get_centroids.argtypes = [vp, vp, vp]
    L.mosaic_get_summaries.argtypes = [vp, vp]
    L.mosaic_get_maintainer.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp]
    L.mosaic_get_selection.argtypes = [vp, i32, vp, vp, vp, vp, C.c_int64, vp]
    L.mosaic_get_stats.argtypes = [vp, C.POINTER(Stats)]
    L.mosaic_get_cache_directory.argtypes = [vp, vp]
    L.mosaic_profile_enable.argtypes = [vp, i32]
    L.mosaic_profile_read.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
    L.mosaic_calibration_copy.argtypes = [vp, vp, sz, vp]
    L.mosaic_last_error.argtypes = [vp]
    L.mosaic_last_error.restype = C.c_char_p
    for name in EXPORTS:
        if name != "mosaic_last_error":
            getattr(L, name).restype = i32
    _lib = L
    return L


def make_config(*, n_layers, n_q_heads, n_kv_heads, head_dim, tokens_per_frame, max_frames,
                n_clusters, top_k, kv_dtype, warmup_frames=0, lloyd_iters=0, recluster_every=0,
                score_mode=0, max_q_tokens=0, attend_impl=ATTEND_AUTO, tier=TIER_HBM,
                slab_frames=0, cache_pages_per_unit=0, cache_fraction=0.0,
                maint_mode=MAINT_OFF, init_clusters=0, split_iters=0, buffer_max=0,
                tau_min=0.0, tau_max=0.0, tau_n0=1.0, aug_global_reps=0, aug_window_frames=0,
                prefetch_top_k=0, n_partitions=0, visual_dim=0, top_partitions=0, decode_fused_max_mib=0,
                ingest_overlap=0) -> Config:
    c = Config()
    c.n_layers, c.n_q_heads, c.n_kv_heads = n_layers, n_q_heads, n_kv_heads
    c.head_dim, c.tokens_per_frame, c.max_frames = head_dim, tokens_per_frame, max_frames
    c.n_clusters, c.top_k = n_clusters, top_k
    c.kv_dtype = {"fp32": FP32, "bf16": BF16}.get(kv_dtype, kv_dtype)
    c.warmup_frames, c.lloyd_iters, c.recluster_every = warmup_frames, lloyd_iters, recluster_every
    c.score_mode, c.max_q_tokens, c.attend_impl = score_mode, max_q_tokens, attend_impl
    c.tier, c.slab_frames, c.cache_pages_per_unit = tier, slab_frames, cache_pages_per_unit
    c.cache_fraction = cache_fraction
    c.maint_mode, c.init_clusters, c.split_iters, c.buffer_max = maint_mode, init_clusters, split_iters, buffer_max
    c.tau_min, c.tau_max, c.tau_n0 = tau_min, tau_max, tau_n0
    c.aug_global_reps, c.aug_window_frames = aug_global_reps, aug_window_frames
    c.prefetch_top_k = prefetch_top_k
    c.decode_fused_max_mib = decode_fused_max_mib
    c.n_partitions, c.visual_dim, c.top_partitions = n_partitions, visual_dim, top_partitions
    c.ingest_overlap = ingest_overlap
    return c


def workspace_sizes(cfg: Config):
    """-> (device arena bytes, pinned host arena bytes)"""
    L = load_library()
    n, h = C.c_size_t(), C.c_size_t()
    rc = L.mosaic_workspace_size(C.byref(cfg), C.byref(n), C.byref(h))
    if rc != OK:
        raise MosaicError(rc, L.mosaic_last_error(None).decode())
    return n.value, h.value


def workspace_size(cfg: Config) -> int:
    return workspace_sizes(cfg)[0]


def _ptr(t) -> int:
    return 0 if t is None else t.data_ptr()


class PinnedArena:
    """Pinned, device-mapped host memory of an exact size (mosaic_host_alloc: hipHostMalloc in the HIP
    runtime the library uses).  torch's own pinned allocator rounds requests up to a power of two,
    which on a box that grants about 64 GB of pinned memory in all turns a 40 GB arena into a refused
    64 GB one."""

    def __init__(self, nbytes: int):
        self._L = load_library()
        p = C.c_void_p()
        rc = self._L.mosaic_host_alloc(nbytes, C.byref(p))
        if rc != OK or not p.value:
            raise MosaicError(rc, self._L.mosaic_last_error(None).decode())
        self.ptr, self.nbytes = p.value, nbytes

    def free(self):
        if getattr(self, "ptr", None):
            self._L.mosaic_host_free(C.c_void_p(self.ptr))
            self.ptr = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


class Mosaic:
    """One video stream's context.  Tensors are torch CUDA tensors; the
    observers return numpy arrays."""

    def __init__(self, cfg: Config, device="cuda:0", stream=None):
        import torch
        self._torch = torch
        self._L = load_library()
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self.cfg = cfg
        nbytes, hbytes = workspace_sizes(cfg)
        # the arena: uninitialised device memory owned here, borrowed by the library
        self.arena = torch.empty(nbytes + 256, dtype=torch.uint8, device=self.device)
        base = (self.arena.data_ptr() + 255) // 256 * 256
        cfg.dev_arena = base
        cfg.dev_arena_bytes = nbytes
        self.host_arena = None
        if hbytes:
            # pinned (hipHostMalloc) host memory for the host tier's cluster slabs
            torch.cuda.current_stream(self.device)            # (the HIP runtime is up before the raw call)
            self.host_arena = PinnedArena(hbytes + 256)
            cfg.host_arena = (self.host_arena.ptr + 255) // 256 * 256
            cfg.host_arena_bytes = hbytes
        self.stream = stream if stream is not None else torch.cuda.current_stream(self.device)
        cfg.stream = self.stream.cuda_stream
        h = C.c_void_p()
        rc = self._L.mosaic_create(C.byref(cfg), C.byref(h))
        if rc != OK:
            raise MosaicError(rc, self._L.mosaic_last_error(None).decode())
        self._h = h
        self.U = cfg.n_layers * cfg.n_kv_heads
        self.dtype = torch.float32 if cfg.kv_dtype == FP32 else torch.bfloat16
        # score columns beyond n_clusters: the buffered singletons of the deferred-split maintainer
        self.buffer_max = (cfg.buffer_max or 32) if cfg.maint_mode == MAINT_DEFERRED else 0

    def close(self):
        if getattr(self, "_h", None):
            self._L.mosaic_destroy(self._h)
            self._h = None
        if getattr(self, "host_arena", None) is not None:
            self.host_arena.free()
            self.host_arena = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc: int):
        if rc != OK:
            raise MosaicError(rc, self._L.mosaic_last_error(self._h).decode())

    def _check_tensor(self, t, shape, name):
        if t.device != self.device or t.dtype != self.dtype or not t.is_contiguous():
            raise ValueError(f"{name}: need a contiguous {self.dtype} tensor on {self.device}")
        if tuple(t.shape) != tuple(shape):
            raise ValueError(f"{name}: shape {tuple(t.shape)} != expected {tuple(shape)}")

    # -- the four calls ------------------------------------------------------
    def reset(self):
        self._check(self._L.mosaic_reset(self._h))

    def ingest_frame(self, k, v):
        """k, v: [n_frames][L][Hkv][T][D]"""
        c = self.cfg
        n = k.shape[0]
        shape = (n, c.n_layers, c.n_kv_heads, c.tokens_per_frame, c.head_dim)
        self._check_tensor(k, shape, "k")
        self._check_tensor(v, shape, "v")
        self._check(self._L.mosaic_ingest_frame(self._h, _ptr(k), _ptr(v), n))

    def ingest_join(self):
        """ingest_overlap = 1: make the context's stream wait for the ingest work on the library's own stream"""
        self._check(self._L.mosaic_ingest_join(self._h))

    def ingest_frame_visual(self, k, v, e):
        """Nested hierarchy: k, v as for ingest_frame; e: fp32 [n_frames][visual_dim]"""
        c = self.cfg
        n = k.shape[0]
        shape = (n, c.n_layers, c.n_kv_heads, c.tokens_per_frame, c.head_dim)
        self._check_tensor(k, shape, "k")
        self._check_tensor(v, shape, "v")
        if c.n_partitions > 0 and (e.device != self.device or e.dtype != self._torch.float32
                                   or not e.is_contiguous() or tuple(e.shape) != (n, c.visual_dim)):
            raise ValueError(f"e: need a contiguous float32 [{n}][{c.visual_dim}] tensor on {self.device}")
        self._check(self._L.mosaic_ingest_frame_visual(self._h, _ptr(k), _ptr(v), _ptr(e), n))

    def _q_shape(self, layer, q):
        c = self.cfg
        tq = q.shape[-3]
        lead = (c.n_layers,) if layer < 0 else ()
        return lead + (tq, c.n_q_heads, c.head_dim), tq

    def retrieve(self, layer: int, q):
        """q: [Tq][Hq][D] (layer >= 0) or [L][Tq][Hq][D] (layer == -1)"""
        shape, tq = self._q_shape(layer, q)
        self._check_tensor(q, shape, "q")
        self._check(self._L.mosaic_retrieve(self._h, layer, _ptr(q), tq))

    def prefetch(self, layer: int, q_proxy):
        """Host tier: predict `layer`'s clusters with a proxy query [Tq][Hq][D] and start fetching them."""
        shape, tq = self._q_shape(max(layer, 0), q_proxy)
        self._check_tensor(q_proxy, shape, "q_proxy")
        self._check(self._L.mosaic_prefetch(self._h, layer, _ptr(q_proxy), tq))

    def prefetch_raw(self, layer: int, q_ptr: int, n_q_tokens: int):
        rc = self._L.mosaic_prefetch(self._h, layer, q_ptr, n_q_tokens)
        if rc != OK:
            self._check(rc)

    def attend(self, layer: int, q, out=None, lse=None):
        torch = self._torch
        shape, tq = self._q_shape(layer, q)
        self._check_tensor(q, shape, "q")
        if out is None:
            out = torch.empty(shape, dtype=self.dtype, device=self.device)
        if lse is None:
            lse = torch.empty(shape[:-1], dtype=torch.float32, device=self.device)
        self._check(self._L.mosaic_attend(self._h, layer, _ptr(q), tq, _ptr(out), _ptr(lse)))
        return out, lse

    def attend_static(self, layer: int, q, out, lse):
        """mosaic_attend with its partials in the library's static buffer; out and lse are the
        caller's (the call itself allocates nothing)."""
        shape, tq = self._q_shape(layer, q)
        self._check_tensor(q, shape, "q")
        self._check_tensor(out, shape, "out")
        self._check(self._L.mosaic_attend_static(self._h, layer, _ptr(q), tq, _ptr(out), _ptr(lse)))
        return out, lse

    def decode_step(self, layer: int, q, out=None, lse=None):
        """retrieve + attend in one call (one fused kernel where it applies)"""
        torch = self._torch
        shape, tq = self._q_shape(layer, q)
        self._check_tensor(q, shape, "q")
        if out is None:
            out = torch.empty(shape, dtype=self.dtype, device=self.device)
        if lse is None:
            lse = torch.empty(shape[:-1], dtype=torch.float32, device=self.device)
        self._check(self._L.mosaic_decode_step(self._h, layer, _ptr(q), tq, _ptr(out), _ptr(lse)))
        return out, lse

    # -- unchecked variants for timed loops: raw device addresses, same C calls --
    def decode_step_raw(self, layer: int, q_ptr: int, n_q_tokens: int, out_ptr: int, lse_ptr: int):
        rc = self._L.mosaic_decode_step(self._h, layer, q_ptr, n_q_tokens, out_ptr, lse_ptr)
        if rc != OK:
            self._check(rc)

    def retrieve_raw(self, layer: int, q_ptr: int, n_q_tokens: int):
        rc = self._L.mosaic_retrieve(self._h, layer, q_ptr, n_q_tokens)
        if rc != OK:
            self._check(rc)

    def attend_raw(self, layer: int, q_ptr: int, n_q_tokens: int, out_ptr: int, lse_ptr: int):
        rc = self._L.mosaic_attend(self._h, layer, q_ptr, n_q_tokens, out_ptr, lse_ptr)
        if rc != OK:
            self._check(rc)

    # -- observers -------------------------------------------------------------
    def stats(self) -> Stats:
        s = Stats()
        self._check(self._L.mosaic_get_stats(self._h, C.byref(s)))
        return s

    def cache_directory(self) -> np.ndarray:
        """Host tier: [U][C] frames of each cluster resident in the GPU cluster cache, -1 = not resident"""
        d = np.empty((self.U, self.cfg.n_clusters), dtype=np.int32)
        self._check(self._L.mosaic_get_cache_directory(self._h, d.ctypes.data))
        return d

    def assignments(self) -> np.ndarray:
        nf = self.stats().frames_ingested
        a = np.empty((self.U, nf), dtype=np.int32)
        self._check(self._L.mosaic_get_assignments(self._h, a.ctypes.data))
        return a

    def centroids(self):
        c = self.cfg
        r = np.empty((self.U, c.n_clusters, c.head_dim), dtype=np.float64)
        n = np.empty((self.U, c.n_clusters), dtype=np.int32)
        self._check(self._L.mosaic_get_centroids(self._h, r.ctypes.data, n.ctypes.data))
        return r, n

    def summaries(self) -> np.ndarray:
        nf = self.stats().frames_ingested
        s = np.empty((self.U, nf, self.cfg.head_dim), dtype=np.float64)
        self._check(self._L.mosaic_get_summaries(self._h, s.ctypes.data))
        return s

    def selection(self, layer: int, with_tokens: bool = True):
        """-> ids [Hkv][k], n_ids [Hkv], scores [Hkv][C], list of tok_idx arrays per head"""
        c = self.cfg
        H = c.n_kv_heads
        ids = np.empty((H, c.top_k), dtype=np.int32)
        n_ids = np.empty(H, dtype=np.int32)
        scores = np.empty((H, c.n_clusters + self.buffer_max), dtype=np.float64)
        n_tok = np.empty(H, dtype=np.int32)
        self._check(self._L.mosaic_get_selection(self._h, layer, ids.ctypes.data, n_ids.ctypes.data,
                                                 scores.ctypes.data, None, 0, n_tok.ctypes.data))
        toks = None
        if with_tokens:
            cap = max(int(n_tok.max()), 1)
            buf = np.empty((H, cap), dtype=np.int32)
            self._check(self._L.mosaic_get_selection(self._h, layer, None, None, None,
                                                     buf.ctypes.data, cap, None))
            toks = [buf[h, : n_tok[h]].copy() for h in range(H)]
        return ids, n_ids, scores, toks

    def partitions(self) -> dict:
        """Nested hierarchy: frame_to_partition [n_frames]; visual_r [P][Dv], visual_n [P];
        part_r [U][P][D], part_n [U][P]."""
        c = self.cfg
        F = int(self.stats().frames_ingested)
        U, P = c.n_layers * c.n_kv_heads, c.n_partitions
        out = {"frame_to_partition": np.empty(max(F, 1), np.int32),
               "visual_r": np.empty((P, c.visual_dim), np.float64), "visual_n": np.empty(P, np.int32),
               "part_r": np.empty((U, P, c.head_dim), np.float64), "part_n": np.empty((U, P), np.int32)}
        self._check(self._L.mosaic_get_partitions(
            self._h, out["frame_to_partition"].ctypes.data, out["visual_r"].ctypes.data,
            out["visual_n"].ctypes.data, out["part_r"].ctypes.data, out["part_n"].ctypes.data))
        out["frame_to_partition"] = out["frame_to_partition"][:F]
        return out

    def partition_selection(self, layer: int):
        """First stage of the latest two-stage selection: part_ids [Hkv][top_partitions],
        n_part_ids [Hkv], part_scores [Hkv][P]."""
        c = self.cfg
        H = c.n_kv_heads
        tp = c.top_partitions or max(1, c.n_partitions // 4)
        ids = np.empty((H, tp), dtype=np.int32)
        n_ids = np.empty(H, dtype=np.int32)
        sc = np.empty((H, c.n_partitions), dtype=np.float64)
        self._check(self._L.mosaic_get_partition_selection(self._h, layer, ids.ctypes.data,
                                                           n_ids.ctypes.data, sc.ctypes.data))
        return ids, n_ids, sc

    def maintainer(self) -> dict:
        """State of the self-adaptive maintainer: var, lazy, resident [U][C]; n_slots, n_buf [U];
        buf_frame, buf_owner [U][buffer_max]."""
        c = self.cfg
        U, Cn, B = c.n_layers * c.n_kv_heads, c.n_clusters, self.buffer_max
        out = {"var": np.empty((U, Cn), np.float64), "lazy": np.empty((U, Cn), np.int32),
               "resident": np.empty((U, Cn), np.int32), "n_slots": np.empty(U, np.int32),
               "n_buf": np.empty(U, np.int32), "buf_frame": np.zeros((U, max(B, 1)), np.int32),
               "buf_owner": np.zeros((U, max(B, 1)), np.int32)}
        self._check(self._L.mosaic_get_maintainer(
            self._h, out["var"].ctypes.data, out["lazy"].ctypes.data, out["resident"].ctypes.data,
            out["n_slots"].ctypes.data, out["n_buf"].ctypes.data,
            out["buf_frame"].ctypes.data if B else None, out["buf_owner"].ctypes.data if B else None))
        return out

    def profile_enable(self, on: bool = True):
        self._check(self._L.mosaic_profile_enable(self._h, 1 if on else 0))

    def profile_read(self):
        ms, n = C.c_double(), C.c_int64()
        self._check(self._L.mosaic_profile_read(self._h, C.byref(ms), C.byref(n)))
        return ms.value, n.value


def config_for(wl, **overrides) -> Config:
    """Config of a paper_2604_10060_amd.inputs.Workload."""
    kw = dict(n_layers=wl.n_layers, n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads,
              head_dim=wl.head_dim, tokens_per_frame=wl.tokens_per_frame,
              max_frames=wl.n_frames, n_clusters=wl.n_clusters, top_k=wl.top_k,
              kv_dtype=wl.kv_dtype, warmup_frames=wl.warmup_frames,
              lloyd_iters=wl.lloyd_iters, recluster_every=wl.recluster_every,
              max_q_tokens=max(wl.question_tokens, 1))
    kw.update(overrides)
    return make_config(**kw)
