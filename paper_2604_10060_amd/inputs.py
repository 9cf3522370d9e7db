"""Seeded synthetic video-KV streams and questions.

This module only draws random inputs; it contains none of the method's
arithmetic (no summaries, similarities, clustering, selection or attention),
so both the CPU oracle's tests and the HIP path's tests may use it.

The streams stand in for the key/value caches a 28-layer, 28-query-head /
4-KV-head, head_dim-128 decoder would produce on the public long-video
benchmarks the paper evaluates on (Sec. VIII-A, Table II); those datasets and
model weights are not available here.  What is reproduced is the structure the
paper attributes to such streams: temporally contiguous, visually coherent
scene segments whose keys form groups (Sec. III-A), and, for live streams,
frequent scene changes (Sec. VIII, real-world dataset paragraph).

Recipe (per layer l and KV head h independently):
  scene centre   c[s,l,h]  ~ N(0, I_D)         (keys and values: independent)
  drift          d[s,l,h]  ~ N(0, I_D)/sqrt(D)
  token          x = c[s] + drift * i * d[s] + noise * N(0, I_D)
                 with i = index of the frame inside its scene segment
  outliers       each token independently, with probability outlier_frac,
                 is replaced by N(0, 2 I_D) in both K and V
  question       q[l,t,hq] = cK[s*, l, hq // G] + 0.5 * N(0, I_D)
Scene segmentation:
  'dirichlet'  n_scenes segments, lengths 1 + floor(w_s (F - S)), w ~ Dir(1),
               remainder handed to the largest fractional parts
  'geometric'  i.i.d. Geometric(1/mean_scene_len) lengths until F is filled
  'rapid'      i.i.d. Uniform{1,2,3} lengths (low visual coherence)
Values are generated in fp32 and rounded (RNE) to the workload's KV dtype.

Visual embeddings (visual_dim > 0; a stand-in for the vision encoder's pooled
per-frame output, which the nested visual-semantic hierarchy of Sec. V-B
clusters first): every scene belongs to one of n_visual appearance classes,
  class centre   a[v]  ~ N(0, I_Dv),  scene offset  o[s] ~ N(0, I_Dv)
  embedding      e_f = a[class(s)] + 0.3 * o[s] + visual_noise * N(0, I_Dv)   (fp32)
so scenes of one class look alike while their key states differ.  With
visual_key_corr = a > 0 the scenes of a class also share a part of their key
centre, cK[s] <- a * bK[class(s)] + sqrt(1 - a^2) * cK[s] with bK ~ N(0, I_D) per
layer and head (the cross-modal regularity of Sec. III-A: visually similar
content tends to be retrieved together); a = 0 leaves the K/V stream untouched.
"""
from __future__ import annotations

import dataclasses
from dataclasses import dataclass
from typing import Optional

import numpy as np
import torch


@dataclass(frozen=True)
class Workload:
    name: str
    n_layers: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    tokens_per_frame: int
    n_frames: int
    n_clusters: int
    top_k: int
    kv_dtype: str                 # "fp32" | "bf16"
    scene_model: str              # "dirichlet" | "geometric" | "rapid"
    n_scenes: int = 0             # dirichlet only
    mean_scene_len: float = 80.0  # geometric only
    noise: float = 0.3
    drift: float = 0.05
    outlier_frac: float = 0.0
    layer_corr: float = 0.0       # correlation of adjacent layers' scene centres and question noise (0 = independent)
    visual_dim: int = 0           # > 0: per-frame visual embeddings of this size are generated as well
    n_visual: int = 8             # appearance classes the scenes are drawn from
    visual_noise: float = 0.3
    visual_key_corr: float = 0.0  # share of a scene's key centre that it has in common with its appearance class
    warmup_frames: int = 0        # 0 -> 2 * n_clusters
    lloyd_iters: int = 8
    recluster_every: int = 0
    question_tokens: int = 16
    decode_steps: int = 0
    seed: int = 1000

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def units(self) -> int:
        return self.n_layers * self.n_kv_heads

    @property
    def warmup(self) -> int:
        return self.warmup_frames if self.warmup_frames > 0 else 2 * self.n_clusters

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.float32 if self.kv_dtype == "fp32" else torch.bfloat16

    def scaled(self, **kw) -> "Workload":
        return dataclasses.replace(self, **kw)


# The five workloads named by the benchmark definition (index = config number).
CONFIGS = (
    Workload("cfg0_tiny", 1, 4, 2, 64, 16, 128, 16, 4, "fp32", "dirichlet",
             n_scenes=8, question_tokens=16, decode_steps=0, seed=1000),
    Workload("cfg1_single_layer_hbm", 1, 28, 4, 128, 64, 1024, 64, 8, "bf16",
             "dirichlet", n_scenes=40, question_tokens=32, decode_steps=256,
             seed=1001),
    Workload("cfg2_full_stack_hbm", 28, 28, 4, 128, 64, 4096, 128, 16, "bf16",
             "geometric", mean_scene_len=80.0, outlier_frac=0.05,
             recluster_every=256, question_tokens=32, decode_steps=64,
             seed=1002),
    Workload("cfg3_host_offload", 28, 28, 4, 128, 196, 16384, 512, 32, "bf16",
             "geometric", mean_scene_len=80.0, question_tokens=32,
             decode_steps=128, seed=1003),
    Workload("cfg4_prefill_stream", 1, 28, 4, 128, 64, 2048, 256, 32, "bf16",
             "dirichlet", n_scenes=64, question_tokens=256, decode_steps=0,
             seed=1004),
)


def cfg4_stream(stream_id: int) -> Workload:
    """Stream `stream_id` (0..7) of the 8-stream prefill workload: streams 0-3
    are scene-coherent, 4-7 change scene every 1-3 frames with noise 1.0."""
    base = CONFIGS[4]
    seed = base.seed + 17 * stream_id
    if stream_id < 4:
        return base.scaled(name=f"cfg4_s{stream_id}", seed=seed)
    return base.scaled(name=f"cfg4_s{stream_id}", seed=seed, scene_model="rapid",
                       noise=1.0, drift=0.0)


def _segment_lengths(wl: Workload, rng: np.random.Generator) -> np.ndarray:
    F = wl.n_frames
    if wl.scene_model == "dirichlet":
        S = min(wl.n_scenes, F)
        w = rng.dirichlet(np.ones(S))
        raw = w * (F - S)
        base = np.floor(raw).astype(np.int64)
        rem = int(F - S - base.sum())
        order = np.argsort(-(raw - base), kind="stable")
        base[order[:rem]] += 1
        return base + 1
    lens = []
    total = 0
    while total < F:
        if wl.scene_model == "geometric":
            n = int(rng.geometric(1.0 / wl.mean_scene_len))
        elif wl.scene_model == "rapid":
            n = int(rng.integers(1, 4))
        else:
            raise ValueError(f"unknown scene_model {wl.scene_model!r}")
        n = min(n, F - total)
        lens.append(n)
        total += n
    return np.asarray(lens, dtype=np.int64)


class SceneStream:
    """A seeded stream of per-frame K and V pages plus questions about it.

    Frame f is a pure function of (workload.seed, f, device type), so any
    frame can be regenerated on its own and frames can be produced in chunks
    of any size with identical results on one device type.
    """

    def __init__(self, wl: Workload, device: str | torch.device = "cpu"):
        self.wl = wl
        self.device = torch.device(device)
        rng = np.random.Generator(np.random.PCG64(wl.seed))
        lens = _segment_lengths(wl, rng)
        assert int(lens.sum()) == wl.n_frames
        self.segment_lengths = lens
        self.scene_of_frame = np.repeat(np.arange(len(lens)), lens)
        starts = np.concatenate([[0], np.cumsum(lens)[:-1]])
        self.index_in_scene = np.arange(wl.n_frames) - np.repeat(starts, lens)
        self.n_scenes = len(lens)
        g = torch.Generator(device=self.device)
        g.manual_seed(wl.seed * 7919 + 1)
        shape = (self.n_scenes, wl.n_layers, wl.n_kv_heads, wl.head_dim)
        rn = lambda: torch.randn(shape, generator=g, device=self.device,
                                 dtype=torch.float32)
        self.centre_k = rn()
        self.centre_v = rn()
        if wl.layer_corr > 0.0:
            # adjacent layers see similar states (residual connections, paper Sec. VII-B): an AR(1)
            # chain over the layer index with unit variance, built from the same draws
            rho, mix = float(wl.layer_corr), float(np.sqrt(1.0 - wl.layer_corr ** 2))
            for c in (self.centre_k, self.centre_v):
                for l in range(1, wl.n_layers):
                    c[:, l] = rho * c[:, l - 1] + mix * c[:, l]
        inv = 1.0 / float(np.sqrt(wl.head_dim))
        self.drift_k = rn() * inv
        self.drift_v = rn() * inv
        self._gen = torch.Generator(device=self.device)
        self._qrng = np.random.Generator(np.random.PCG64(wl.seed + 500_000))
        if wl.visual_dim > 0:      # draws of their own: the K/V stream does not depend on them
            vr = np.random.Generator(np.random.PCG64(wl.seed + 900_000))
            self.visual_class_of_scene = vr.integers(0, wl.n_visual, size=self.n_scenes)
            gv = torch.Generator(device=self.device)
            gv.manual_seed(wl.seed * 7919 + 3)
            self.visual_centre = torch.randn((wl.n_visual, wl.visual_dim), generator=gv,
                                             device=self.device, dtype=torch.float32)
            self.visual_offset = torch.randn((self.n_scenes, wl.visual_dim), generator=gv,
                                             device=self.device, dtype=torch.float32)
            if wl.visual_key_corr > 0.0:
                a = float(wl.visual_key_corr)
                bk = torch.randn((wl.n_visual,) + shape[1:], generator=gv, device=self.device,
                                 dtype=torch.float32)
                cls = torch.as_tensor(self.visual_class_of_scene, device=self.device)
                self.centre_k = a * bk[cls] + float(np.sqrt(1.0 - a * a)) * self.centre_k

    # -- frames ------------------------------------------------------------
    def frame(self, f: int) -> tuple[torch.Tensor, torch.Tensor]:
        """K and V of frame f, each [L][Hkv][T][D] in the workload's KV dtype."""
        wl = self.wl
        s = int(self.scene_of_frame[f])
        i = float(self.index_in_scene[f])
        g = self._gen
        g.manual_seed(wl.seed * 1_000_003 + 17 * f + 5)
        shape = (wl.n_layers, wl.n_kv_heads, wl.tokens_per_frame, wl.head_dim)
        out = []
        mask = None
        if wl.outlier_frac > 0.0:
            u = torch.rand(shape[:-1], generator=g, device=self.device)
            mask = (u < wl.outlier_frac).unsqueeze(-1)
        for centre, drift in ((self.centre_k, self.drift_k),
                              (self.centre_v, self.drift_v)):
            base = centre[s] + (wl.drift * i) * drift[s]          # [L][Hkv][D]
            x = torch.randn(shape, generator=g, device=self.device,
                            dtype=torch.float32)
            x = base.unsqueeze(2) + wl.noise * x
            if mask is not None:
                o = torch.randn(shape, generator=g, device=self.device,
                                dtype=torch.float32) * float(np.sqrt(2.0))
                x = torch.where(mask, o, x)
            out.append(x.to(wl.torch_dtype))
        return out[0], out[1]

    def frames(self, f0: int, f1: int) -> tuple[torch.Tensor, torch.Tensor]:
        """K and V of frames f0..f1-1, each [f1-f0][L][Hkv][T][D]."""
        ks, vs = zip(*(self.frame(f) for f in range(f0, f1)))
        return torch.stack(ks), torch.stack(vs)

    # -- visual embeddings -------------------------------------------------
    def embedding(self, f: int) -> torch.Tensor:
        """Visual embedding of frame f, fp32 [Dv]."""
        wl = self.wl
        assert wl.visual_dim > 0
        s = int(self.scene_of_frame[f])
        g = self._gen
        g.manual_seed(wl.seed * 3_000_017 + 13 * f + 7)
        x = torch.randn((wl.visual_dim,), generator=g, device=self.device, dtype=torch.float32)
        return self.visual_centre[int(self.visual_class_of_scene[s])] + 0.3 * self.visual_offset[s] \
            + wl.visual_noise * x

    def embeddings(self, f0: int, f1: int) -> torch.Tensor:
        """Visual embeddings of frames f0..f1-1, fp32 [f1-f0][Dv]."""
        return torch.stack([self.embedding(f) for f in range(f0, f1)])

    # -- questions ---------------------------------------------------------
    def draw_scene(self) -> int:
        """Uniformly drawn scene a question is about (advances the question RNG)."""
        return int(self._qrng.integers(0, self.n_scenes))

    def question(self, scene: int, n_tokens: int, tag: int) -> torch.Tensor:
        """Query states [L][Tq][Hq][D] around scene `scene`'s key centres."""
        wl = self.wl
        g = self._gen
        g.manual_seed(wl.seed * 2_000_003 + 31 * tag + 11)
        c = self.centre_k[scene]                                   # [L][Hkv][D]
        c = c.repeat_interleave(wl.group, dim=1)                   # [L][Hq][D]
        x = torch.randn((wl.n_layers, n_tokens, wl.n_q_heads, wl.head_dim),
                        generator=g, device=self.device, dtype=torch.float32)
        if wl.layer_corr > 0.0:
            rho, mix = float(wl.layer_corr), float(np.sqrt(1.0 - wl.layer_corr ** 2))
            for l in range(1, wl.n_layers):
                x[l] = rho * x[l - 1] + mix * x[l]
        q = c.unsqueeze(1) + 0.5 * x
        return q.to(wl.torch_dtype)


def unit_pages(x: torch.Tensor, layer: int, head: int) -> np.ndarray:
    """[F][L][Hkv][T][D] tensor -> float64 numpy [F][T][D] of one (layer, head)."""
    return x[:, layer, head].to(torch.float32).cpu().numpy().astype(np.float64)
