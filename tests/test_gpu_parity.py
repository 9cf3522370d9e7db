"""GPU parity tests: the HIP library, called through its C ABI, against the
fp64 CPU oracle on the same seeded streams.  Bars are stated in tests/harness.py.
"""
import numpy as np
import pytest
import torch

from oracle import cache_model
from paper_2604_10060_amd import binding, inputs
from tests import harness

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _small(**kw):
    """A reduced single-layer bf16 workload with the realistic head shape."""
    base = dict(name="small_bf16", n_frames=160, n_scenes=8, n_clusters=12, top_k=4,
                question_tokens=4)
    base.update(kw)
    return inputs.CONFIGS[1].scaled(**base)


def _report(rep):
    print(f"  decisions {rep.online_decisions} forced {rep.forced_near_ties} lloyd {rep.lloyd_runs} "
          f"topk-ties {rep.topk_near_ties} out {rep.max_out_err:.2e} lse {rep.max_lse_err:.2e} "
          f"centroid {rep.max_centroid_rel:.1e}", flush=True)


def test_cfg0_fp32_full():
    rep = harness.run_workload(inputs.CONFIGS[0])
    _report(rep)
    assert rep.max_out_err <= 1e-4


def test_small_bf16_mfma_prefill_and_decode():
    rep = harness.run_workload(_small(), decode_steps=3)
    _report(rep)
    assert rep.max_out_err <= 2e-2


def test_small_bf16_valu_kernel():
    rep = harness.run_workload(_small(), decode_steps=2, attend_impl=binding.ATTEND_VALU)
    _report(rep)


def test_all_layers_in_one_call():
    wl = _small(n_layers=3, n_frames=96, n_clusters=8, top_k=3)
    rep = harness.run_workload(wl, decode_steps=2, layer_mode="all")
    _report(rep)


@pytest.mark.parametrize("kw", [
    dict(tokens_per_frame=5, n_clusters=7, top_k=7),            # ragged page, k = C (dense attention)
    dict(tokens_per_frame=13, top_k=1),                         # k = 1
    dict(tokens_per_frame=1, n_frames=300, n_clusters=20, top_k=6),   # one token per frame: a page is 1/32 of a chunk
    dict(tokens_per_frame=196, n_frames=64, n_clusters=6, top_k=2, n_scenes=4),   # 7 chunks per page, last ragged
    dict(tokens_per_frame=40, question_tokens=3),               # 21 query rows: two row tiles
    dict(n_q_heads=4, n_kv_heads=4, question_tokens=5),         # G = 1
    dict(n_q_heads=8, n_kv_heads=4, head_dim=64, question_tokens=9),   # G = 2, D = 64, 18 rows
    dict(n_q_heads=32, n_kv_heads=2, question_tokens=1),        # G = 16: exactly one full tile
])
def test_shapes_bf16(kw):
    rep = harness.run_workload(_small(**kw), decode_steps=1)
    _report(rep)


@pytest.mark.parametrize("kw", [
    dict(tokens_per_frame=3, n_clusters=5, top_k=5),
    dict(tokens_per_frame=33, head_dim=128, n_q_heads=6, n_kv_heads=2, question_tokens=7),
])
def test_shapes_fp32(kw):
    wl = inputs.CONFIGS[0].scaled(name="odd_fp32", **kw)
    rep = harness.run_workload(wl, decode_steps=1)
    _report(rep)


@pytest.mark.parametrize("tq,kw", [
    (256, dict(n_frames=128, n_clusters=8, top_k=3)),          # 1792 rows: 7 full 256-row workgroups
    (41, dict(tokens_per_frame=50, n_frames=96)),              # 287 rows: 18 tiles, ragged last workgroup and tile
    (19, dict(n_q_heads=8, n_kv_heads=4, head_dim=64)),        # G = 2, D = 64, 38 rows
    (64, dict(tokens_per_frame=196, n_frames=64, n_clusters=6, top_k=2)),   # 7 chunks per page, the last with 4 tokens
    (70, dict(n_q_heads=8, n_kv_heads=4, head_dim=64, tokens_per_frame=40)),   # D = 64, 140 rows (two row blocks), ragged pages
])
def test_long_question_prefill_bf16(tq, kw):
    rep = harness.run_workload(_small(question_tokens=tq, **kw))
    _report(rep)


def test_recluster_parity():
    wl = _small(n_frames=200, recluster_every=48, n_clusters=10, warmup_frames=24, lloyd_iters=3)
    rep = harness.run_workload(wl, decode_steps=1)
    _report(rep)
    assert rep.lloyd_runs >= 4 * 4      # init + 4 re-clusterings (48..192, 96 etc.), per unit


@pytest.mark.parametrize("kw", [
    # weakly structured keys (a scene every 1-3 frames, noise as large as the scene centres): many frames keep
    # moving between clusters for all twelve rounds, so rows of frames pass and fail the bound test of the later
    # rounds side by side
    dict(n_frames=700, scene_model="rapid", noise=1.0, drift=0.0, n_clusters=24, warmup_frames=48,
         recluster_every=128, lloyd_iters=12),
    # more frames than one workgroup of the bound test covers, cluster count not a multiple of the tile
    dict(n_frames=1200, n_scenes=30, n_clusters=40, warmup_frames=80, recluster_every=400, lloyd_iters=8),
    # head size 64, clusters that run empty (more clusters than scenes, few frames)
    dict(n_frames=300, head_dim=64, n_scenes=5, n_clusters=48, warmup_frames=96, recluster_every=100, lloyd_iters=6),
])
def test_recluster_rounds_with_skipped_frames_parity(kw):
    """The K-means rounds after the first skip frames whose assignment cannot change and clusters whose members
    did not change: assignments, sizes and representatives must still be the oracle's, which does neither."""
    wl = _small(**kw)
    rep = harness.run_workload(wl, decode_steps=1)
    _report(rep)
    assert rep.lloyd_runs >= 2 * 4


def test_low_coherence_stream():
    wl = inputs.cfg4_stream(5).scaled(n_frames=192, n_clusters=16, top_k=5, question_tokens=8)
    rep = harness.run_workload(wl)
    _report(rep)


def _ingest_all(wl, K, V, pattern, **over):
    m = binding.Mosaic(binding.config_for(wl, **over), device=DEV)
    f = 0
    i = 0
    while f < wl.n_frames:
        nb = min(pattern[i % len(pattern)], wl.n_frames - f)
        i += 1
        m.ingest_frame(K[f:f + nb].contiguous(), V[f:f + nb].contiguous())
        f += nb
    return m


def test_batched_ingest_equals_single_frame_calls_bitwise():
    # batches that straddle the warm-up boundary and re-clustering points
    wl = _small(n_frames=150, recluster_every=40, warmup_frames=24, lloyd_iters=2)
    st = inputs.SceneStream(wl)
    K, V = [x.to(DEV) for x in st.frames(0, wl.n_frames)]
    q = st.question(0, 2, 0).to(DEV)
    res = []
    for pattern in ((1,), (37, 5, 64), (150,)):
        m = _ingest_all(wl, K, V, pattern)
        m.retrieve(0, q[0].contiguous())
        out, lse = m.attend(0, q[0].contiguous())
        r, n = m.centroids()
        res.append((m.assignments(), r, n, out.float().cpu().numpy(), lse.cpu().numpy()))
        assert m.stats().lloyd_runs == 1 + 3
        m.close()
    for other in res[1:]:
        for a, b in zip(res[0], other):
            np.testing.assert_array_equal(a, b)


@pytest.mark.parametrize("kw,over", [
    (dict(), dict(aug_global_reps=1, aug_window_frames=5)),          # value summaries formed by the one-launch path
    (dict(kv_dtype="fp32", head_dim=64, n_q_heads=8, n_kv_heads=4), dict()),   # fp32 pages, D = 64
    (dict(n_clusters=150, top_k=6, n_frames=400), dict()),           # table too large for the one-launch path
])
def test_single_frame_calls_equal_batched_ingest_variants(kw, over):
    """A single-frame call of the online phase takes one launch (pages, summary, assignment, Eq. 3)
    where the register-table kernel applies; its state and outputs equal the batched path's bit for bit."""
    wl = _small(n_frames=kw.pop("n_frames", 140), **kw)
    st = inputs.SceneStream(wl)
    K, V = [x.to(DEV) for x in st.frames(0, wl.n_frames)]
    q = st.question(0, 1, 0).to(DEV)
    res = []
    for pattern in ((1,), (16,)):
        m = _ingest_all(wl, K, V, pattern, **over)
        m.retrieve(0, q[0].contiguous())
        out, lse = m.attend(0, q[0].contiguous())
        r, n = m.centroids()
        res.append((m.assignments(), r, n, m.summaries(), out.float().cpu().numpy(), lse.cpu().numpy()))
        m.close()
    for a, b in zip(res[0], res[1]):
        np.testing.assert_array_equal(a, b)


@pytest.mark.parametrize("over", [
    dict(),
    dict(maint_mode=binding.MAINT_EAGER, init_clusters=4, tau_min=1.0, tau_max=2.0, tau_n0=8.0, recluster_every=0),
])
def test_overlapped_ingest_equals_plain_ingest_bitwise(over):
    """ingest_overlap = 1 (Sec. VII-A pipelining: the order-dependent part of a batched call on the context's
    own stream, the next call's page stores beside it) leaves the same state and outputs bit for bit as the
    plain call order, with queries, observers, single-frame calls and a reset in between."""
    wl = _small(n_frames=300, recluster_every=over.pop("recluster_every", 64), warmup_frames=24, lloyd_iters=3)
    st = inputs.SceneStream(wl)
    K, V = [x.to(DEV) for x in st.frames(0, wl.n_frames)]
    q = st.question(0, 2, 0).to(DEV)[0].contiguous()
    pattern = (16, 37, 1, 64, 5, 1, 16)
    res = []
    for overlap in (0, 1):
        m = binding.Mosaic(binding.config_for(wl, ingest_overlap=overlap, **over), device=DEV)
        seen = []
        for rounds in range(2):                    # the second round after a reset
            f = i = 0
            while f < wl.n_frames:
                nb = min(pattern[i % len(pattern)], wl.n_frames - f)
                m.ingest_frame(K[f:f + nb].contiguous(), V[f:f + nb].contiguous())
                f += nb
                i += 1
                if f >= wl.warmup_frames and i % 3 == 0:     # a query between ingest calls
                    m.retrieve(0, q)
                    out, lse = m.attend(0, q)
                    seen.append((out.float().cpu().numpy(), lse.cpu().numpy()))
                if i % 5 == 0:
                    seen.append((m.assignments(),))          # an observer between ingest calls
            if overlap:
                m.ingest_join()
            torch.cuda.synchronize()
            r, n = m.centroids()
            seen.append((m.assignments(), r, n, m.summaries()))
            if rounds == 0:
                m.reset()
        res.append(seen)
        m.close()
    assert len(res[0]) == len(res[1])
    for a, b in zip(res[0], res[1]):
        for x, y in zip(a, b):
            np.testing.assert_array_equal(x, y)


def test_reset_and_rerun_is_deterministic():
    wl = _small(n_frames=80, n_clusters=6, top_k=2)
    st = inputs.SceneStream(wl)
    K, V = [x.to(DEV) for x in st.frames(0, wl.n_frames)]
    q = st.question(1, 1, 0).to(DEV)[0].contiguous()
    m = _ingest_all(wl, K, V, (16,))
    m.retrieve(0, q)
    o1, l1 = m.attend(0, q)
    a1 = m.assignments()
    m.reset()
    assert m.stats().frames_ingested == 0
    with pytest.raises(binding.MosaicError) as e:
        m.retrieve(0, q)
    assert e.value.code == binding.ENOTREADY
    for f in range(0, wl.n_frames, 16):
        m.ingest_frame(K[f:f + 16].contiguous(), V[f:f + 16].contiguous())
    m.retrieve(0, q)
    o2, l2 = m.attend(0, q)
    np.testing.assert_array_equal(a1, m.assignments())
    assert torch.equal(o1, o2) and torch.equal(l1, l2)
    m.close()


def test_error_paths():
    wl = _small(n_frames=40, n_clusters=8, top_k=2)
    st = inputs.SceneStream(wl)
    K, V = [x.to(DEV) for x in st.frames(0, wl.n_frames)]
    q = st.question(0, 1, 0).to(DEV)[0].contiguous()
    m = binding.Mosaic(binding.config_for(wl), device=DEV)
    m.ingest_frame(K[:10].contiguous(), V[:10].contiguous())
    assert (m.assignments() == -1).all()                       # still buffered
    with pytest.raises(binding.MosaicError) as e:               # before the initial clustering
        m.retrieve(0, q)
    assert e.value.code == binding.ENOTREADY
    m.ingest_frame(K[10:30].contiguous(), V[10:30].contiguous())
    with pytest.raises(binding.MosaicError) as e:               # attend without a selection
        m.attend(0, q)
    assert e.value.code == binding.ENOTREADY
    m.retrieve(0, q)
    m.attend(0, q)
    m.ingest_frame(K[30:31].contiguous(), V[30:31].contiguous())
    with pytest.raises(binding.MosaicError) as e:               # selection is stale after an ingest
        m.attend(0, q)
    assert e.value.code == binding.ENOTREADY
    with pytest.raises(binding.MosaicError) as e:               # capacity
        m.ingest_frame(K[:10].contiguous(), V[:10].contiguous())
    assert e.value.code == binding.ECAPACITY
    assert m.stats().frames_ingested == 31                      # nothing was ingested by the failed call
    L = binding.load_library()
    assert L.mosaic_retrieve(m._h, 3, q.data_ptr(), 1) == binding.EINVAL      # layer out of range
    assert L.mosaic_retrieve(m._h, 0, q.data_ptr(), 0) == binding.EINVAL      # no query tokens
    assert L.mosaic_retrieve(m._h, 0, q.data_ptr(), 10 ** 6) == binding.EINVAL
    assert L.mosaic_ingest_frame(m._h, None, None, 1) == binding.EINVAL
    assert b"NULL" in L.mosaic_last_error(m._h)
    assert L.mosaic_ingest_frame(m._h, K.data_ptr(), V.data_ptr(), 0) == binding.EINVAL       # empty batch
    assert m.stats().frames_ingested == 31
    m.close()
    # arena too small
    cfg = binding.config_for(wl)
    need = binding.workspace_size(cfg)
    buf = torch.empty(need // 2, dtype=torch.uint8, device=DEV)
    cfg.dev_arena = (buf.data_ptr() + 255) // 256 * 256
    cfg.dev_arena_bytes = need // 2 - 256
    import ctypes as C
    h = C.c_void_p()
    assert L.mosaic_create(C.byref(cfg), C.byref(h)) == binding.ENOMEM


def test_cfg1_full_size():
    """Single-layer realistic workload at full size in the launch configuration
    the benchmark times: 32-token question, then decode steps."""
    rep = harness.run_workload(inputs.CONFIGS[1], decode_steps=4)
    _report(rep)
    assert rep.max_out_err <= 2e-2


def test_cfg2_full_size_sampled_units():
    """The full stack at full size (28 layers, 4096 frames of 64 tokens, 15 GB of KV, a
    full re-clustering every 256 frames): two sampled units against the oracle in the three
    launch configurations the benchmark times (all layers in one call, one decode-step call
    per layer, retrieve + attend per layer)."""
    rep = harness.run_full_size(inputs.CONFIGS[2], [(3, 1), (27, 2)],
                                layer_modes=("all", "fused", "per_layer"))
    _report(rep)
    assert rep.max_out_err <= 2e-2


@pytest.mark.parametrize("kw", [dict(n_frames=8192, n_scenes=320), dict(n_frames=13000, n_scenes=500, head_dim=64)])
def test_decode_step_fused_on_a_store_beyond_the_caches(kw):
    """A long stream with a narrow selection: 0.85-1.07 GB of stored KV (the decode kernels then load K/V
    with the non-temporal hint) but only ~30 MB per step, so mosaic_decode_step still takes the one-kernel
    path -- the streaming instantiation of the fused kernel, which no benchmark configuration reaches."""
    wl = inputs.CONFIGS[1].scaled(name="long_stream_narrow_selection", top_k=2, **kw)
    rep = harness.run_full_size(wl, [(0, 0), (0, 3)], layer_modes=("fused", "per_layer"), ingest_batch=64,
                                decode_steps=2, question=False)
    _report(rep)
    fused = [v for (k, v) in rep.notes if k == "decode_step_fused"]
    assert fused and all(v == 1 for v in fused), fused
    assert rep.max_out_err <= 2e-2


@pytest.mark.parametrize("stream_id", [0, 5])
def test_cfg4_full_size_question_prefill(stream_id):
    """One stream of the 8-stream prefill workload at full size (2048 frames, 256 clusters,
    top-32): a 256-token question through the multi-token MFMA kernel, one sampled unit.
    Stream 5 changes scene every few frames (many small clusters, ragged selection)."""
    wl = inputs.cfg4_stream(stream_id)
    rep = harness.run_full_size(wl, [(0, 1 + stream_id % 3)], ingest_batch=64, decode_steps=0)
    _report(rep)
    assert rep.online_decisions == wl.n_frames - wl.warmup


def test_cfg3_full_shape_one_layer_host_tier():
    """The host-offload workload with its per-layer shape kept (16384 frames of 196 tokens, a table of
    512 clusters, top-32, slabs of 8 frames) and one of its 28 layers: 8.8 GB of KV in pinned host
    memory, a GPU cluster cache capped at 10 % of the stream's pages and 10 % of the cluster table, the
    self-adaptive maintainer keeping the clusters small enough for it (the benchmark's parameters).
    One sampled unit: every assignment and the maintainer's counters against the oracle, then decode
    steps (ids, token lists, attention)."""
    wl = inputs.CONFIGS[3].scaled(n_layers=1)
    mt = _mt(1, 64, 1.0, 4.0, n0=32.0)
    dev = DEV
    st = inputs.SceneStream(wl, device=dev)
    F = wl.n_frames
    m = binding.Mosaic(binding.config_for(wl, warmup_frames=0, tier=binding.TIER_HOST, slab_frames=8,
                                          cache_fraction=0.10, cache_pages_per_unit=F // 10,
                                          **harness.maintainer_overrides(mt)), device=dev)
    unit = (0, 2)
    keepK, keepV = [], []
    for f0 in range(0, F, 256):
        K, V = st.frames(f0, min(F, f0 + 256))
        keepK.append(K[:, unit[0], unit[1]].cpu()); keepV.append(V[:, unit[0], unit[1]].cpu())
        for b in range(0, K.shape[0], 64):
            m.ingest_frame(K[b:b + 64], V[b:b + 64])
    torch.cuda.synchronize()
    Ku = torch.cat(keepK).float().numpy().astype(np.float64)
    Vu = torch.cat(keepV).float().numpy().astype(np.float64)
    from oracle import mosaic_oracle as orc
    o = orc.OracleUnit(wl.n_clusters, wl.head_dim, wl.tokens_per_frame, F, 0, wl.lloyd_iters, 0, maintainer=mt)
    for f in range(F):
        o.ingest(Ku[f])
    u = unit[0] * wl.n_kv_heads + unit[1]
    np.testing.assert_array_equal(m.assignments()[u], o.assignments())
    _, N = m.centroids()
    np.testing.assert_array_equal(N[u], o.sizes())
    assert m.maintainer()["n_slots"][u] == o.n_slots and o.counters()["split_now"] > 100
    assert N[u].max() < 200                        # no degenerate cluster: top-32 fits a tenth of the pages
    G, D = wl.group, wl.head_dim
    for i in range(3):
        q = st.question(st.draw_scene(), 1, i)
        m.retrieve(0, q[0].contiguous())
        out, lse = m.attend(0, q[0].contiguous())
        torch.cuda.synchronize()
        ids, n_ids, sc, toks = m.selection(0)
        qh = q[0].float().cpu().numpy().astype(np.float64)
        ids_o, sc_o, tok_o, gap = o.retrieve(qh, unit[1], G, wl.top_k)
        np.testing.assert_array_equal(ids[unit[1], : n_ids[unit[1]]], ids_o)
        np.testing.assert_array_equal(toks[unit[1]], tok_o)
        assert len(tok_o) <= (F // 10) * wl.tokens_per_frame
        want, want_lse = orc.attend(qh, Ku.reshape(-1, D), Vu.reshape(-1, D), tok_o, unit[1], G)
        got = out[:, unit[1] * G:(unit[1] + 1) * G].float().cpu().numpy()
        assert np.abs(got - want).max() <= harness.OUT_TOL["bf16"]
        assert np.abs(lse[:, unit[1] * G:(unit[1] + 1) * G].cpu().numpy() - want_lse).max() <= harness.LSE_TOL["bf16"]
    s = m.stats()
    assert s.cache_misses > 0 and s.h2d_bytes > 0
    m.close()


# --------------------------------------------------------------------------
# host tier: pinned-host cluster slabs + GPU cluster cache
# --------------------------------------------------------------------------
HOST = dict(tier=binding.TIER_HOST, slab_frames=4)


def test_host_tier_parity():
    rep = harness.run_workload(_small(n_frames=200), decode_steps=3, **HOST)
    _report(rep)


def test_host_tier_parity_ragged_pages_two_layers():
    wl = _small(n_layers=2, tokens_per_frame=50, n_frames=120, n_clusters=9, top_k=3, question_tokens=3)
    rep = harness.run_workload(wl, decode_steps=2, slab_frames=3, tier=binding.TIER_HOST)
    _report(rep)


def test_host_tier_matches_hbm_tier_bitwise_and_overlaps_layers():
    wl = _small(n_layers=3, n_frames=144, n_clusters=10, top_k=3)
    st = inputs.SceneStream(wl)
    K, V = [x.to(DEV) for x in st.frames(0, wl.n_frames)]
    qs = [st.question(st.draw_scene(), 1, i).to(DEV) for i in range(4)]
    outs = {}
    for name, over in (("hbm", {}), ("host", HOST)):
        m = _ingest_all(wl, K, V, (16,), **over)
        res = []
        for q in qs:
            o = torch.empty_like(q)
            l = torch.empty(q.shape[:-1], dtype=torch.float32, device=DEV)
            # software pipeline: the selection/fetch of layer l+1 is issued before attend(l)
            m.retrieve(0, q[0].contiguous())
            for layer in range(wl.n_layers):
                if layer + 1 < wl.n_layers:
                    m.retrieve(layer + 1, q[layer + 1].contiguous())
                m.attend(layer, q[layer].contiguous(), o[layer], l[layer])
            torch.cuda.synchronize()
            res.append((o.clone(), l.clone()))
        outs[name] = res
        if name == "host":
            s = m.stats()
            assert s.cache_misses > 0 and s.h2d_bytes > 0 and s.h2d_copies > 0
        m.close()
    for (o1, l1), (o2, l2) in zip(outs["hbm"], outs["host"]):
        assert torch.equal(o1, o2) and torch.equal(l1, l2)


def _model_directory(model, C, membership):
    d = np.full(C, -1, dtype=np.int32)
    for c, p in model.directory(membership).items():
        d[c] = p
    return d


def test_host_tier_cache_follows_the_lru_model_and_grows_with_the_stream():
    """The GPU cluster cache against the oracle's working-set model (least recently used at cluster
    granularity, capacity in pages and in clusters), fed the oracle's own selections and memberships:
    directory after every retrieval, hit / miss / byte counters at the end, while the stream keeps
    growing between questions."""
    from oracle import mosaic_oracle as orc
    wl = _small(n_kv_heads=1, n_q_heads=7, n_frames=240, n_clusters=12, top_k=3, n_scenes=10, warmup_frames=120)
    st = inputs.SceneStream(wl)
    K, V = st.frames(0, wl.n_frames)
    Kd, Vd = K.to(DEV), V.to(DEV)
    Ku = inputs.unit_pages(K, 0, 0)
    pages = 170           # the three largest clusters hold 154 of the 240 frames
    m = binding.Mosaic(binding.config_for(wl, tier=binding.TIER_HOST, slab_frames=4,
                                          cache_pages_per_unit=pages, cache_fraction=5 / 12), device=DEV)
    model = cache_model.ClusterCacheModel(capacity_pages=pages, max_clusters=5)
    o = orc.OracleUnit(wl.n_clusters, wl.head_dim, wl.tokens_per_frame, wl.n_frames, wl.warmup_frames, wl.lloyd_iters)
    m.ingest_frame(Kd[:160].contiguous(), Vd[:160].contiguous())
    for f in range(160):
        o.ingest(Ku[f])
    f = 160
    for i in range(24):
        if i % 6 == 5 and f < wl.n_frames:          # the stream keeps growing between questions
            m.ingest_frame(Kd[f:f + 20].contiguous(), Vd[f:f + 20].contiguous())
            for ff in range(f, f + 20):
                o.ingest(Ku[ff])
            f += 20
        q = st.question(st.draw_scene(), 1, i)
        qd = q.to(DEV)[0].contiguous()
        m.retrieve(0, qd)
        out, _ = m.attend(0, qd)
        ids, n_ids, _, toks = m.selection(0)
        ids_o, _, tok_o, _ = o.retrieve(q[0].float().numpy().astype(np.float64), 0, wl.group, wl.top_k)
        np.testing.assert_array_equal(ids[0, : n_ids[0]], ids_o)
        np.testing.assert_array_equal(toks[0], tok_o)
        mem = cache_model.membership_from_assignments(o.assignments())
        model.access(ids_o, mem)
        np.testing.assert_array_equal(m.cache_directory()[0], _model_directory(model, wl.n_clusters, mem),
                                      err_msg=f"cache directory after question {i}")
        assert torch.isfinite(out.float()).all()
    s = m.stats()
    assert (s.cache_hits, s.cache_misses) == (model.hits, model.misses)
    page_bytes = 2 * wl.tokens_per_frame * wl.head_dim * 2
    assert s.h2d_bytes == model.pages_moved * page_bytes
    assert s.cache_hits > 0 and s.cache_misses > 0 and model.evictions > 0
    m.close()


def test_host_tier_cache_too_small_is_an_error_that_leaves_the_cache_usable():
    """A selection that cannot be resident together is refused without touching the cache: the
    directory still describes what was really fetched, the layer has no selection, and a smaller
    selection afterwards is served and attends correctly (compared with the oracle)."""
    wl = _small(n_frames=120, n_clusters=6, top_k=4)
    st = inputs.SceneStream(wl)
    K, V = st.frames(0, wl.n_frames)
    Kd, Vd = K.to(DEV), V.to(DEV)
    m = binding.Mosaic(binding.config_for(wl, tier=binding.TIER_HOST, slab_frames=4,
                                          cache_pages_per_unit=8), device=DEV)
    m.ingest_frame(Kd, Vd)
    q = st.question(0, 1, 0).to(DEV)[0].contiguous()
    before = m.cache_directory().copy()
    for call in (m.retrieve, m.prefetch):
        with pytest.raises(binding.MosaicError) as e:
            call(0, q)
        assert e.value.code == binding.ECAPACITY
        np.testing.assert_array_equal(m.cache_directory(), before)
        with pytest.raises(binding.MosaicError) as e:     # no selection is current after the refusal
            m.attend(0, q)
        assert e.value.code == binding.ENOTREADY
    s = m.stats()
    assert s.cache_hits == s.cache_misses == s.h2d_bytes == 0
    with pytest.raises(binding.MosaicError) as e:     # all-layers calls are not part of the host tier
        m.retrieve(-1, q[None].contiguous())
    assert e.value.code == binding.EINVAL
    m.close()
    # the same stream with a cache that holds a top-1 selection but not a top-4 one
    _, n = _ingest_all(wl, Kd, Vd, (16,)).centroids()
    biggest = int(n.max())
    wl1 = _small(n_frames=120, n_clusters=6, top_k=1)
    m = binding.Mosaic(binding.config_for(wl1, tier=binding.TIER_HOST, slab_frames=4,
                                          cache_pages_per_unit=biggest, cache_fraction=1 / 6), device=DEV)
    rep = harness.Report()
    oracles = harness.ingest_with_parity(m, wl1, Kd, Vd, [(0, h) for h in range(wl1.n_kv_heads)], rep)
    model = {h: cache_model.ClusterCacheModel(biggest, 1) for h in range(wl1.n_kv_heads)}
    for i in range(4):
        qq = st.question(st.draw_scene(), 1, 10 + i).to(DEV)
        harness.query_with_parity(m, wl1, qq, oracles, K, V, rep)
        q_h = qq.float().cpu().numpy().astype(np.float64)
        for h in range(wl1.n_kv_heads):
            o = oracles[(0, h)]
            mem = cache_model.membership_from_assignments(o.assignments())
            model[h].access(o.retrieve(q_h[0], h, wl1.group, wl1.top_k)[0], mem)
            np.testing.assert_array_equal(m.cache_directory()[h], _model_directory(model[h], wl1.n_clusters, mem))
    s = m.stats()
    assert s.cache_hits == sum(x.hits for x in model.values())
    assert s.cache_misses == sum(x.misses for x in model.values())
    m.close()


# ---------------------------------------------------------------------------
# Self-adaptive maintainer (paper Sec. VI)
# ---------------------------------------------------------------------------
def _mt(mode, c_init, tau_min, tau_max, n0=8.0, split_iters=4, buf_max=0):
    return dict(mode=mode, c_init=c_init, tau_min=tau_min, tau_max=tau_max, n0=n0,
                split_iters=split_iters, buf_max=buf_max)


@pytest.mark.gpu
def test_maintainer_eager_fp32():
    """Config-0 stream (8 scenes), 3 initial clusters in a table of 24: variance tracking,
    threshold and immediate splits must follow the oracle insertion by insertion."""
    wl = inputs.CONFIGS[0].scaled(name="maint_eager_fp32", n_clusters=24, top_k=4)
    rep = harness.run_maintained(wl, _mt(1, 3, 1.5, 6.0))
    tot = rep.notes[-1]
    assert tot["split_now"] > 0, tot
    assert rep.max_out_err <= 1e-4


@pytest.mark.gpu
def test_maintainer_eager_bf16_table_fills_up():
    """D = 128, bf16, a table that is too small: splits until no id is free, then forced absorbs."""
    wl = inputs.CONFIGS[1].scaled(name="maint_eager_bf16", n_frames=192, n_scenes=12, n_clusters=8,
                                  top_k=3, question_tokens=4)
    rep = harness.run_maintained(wl, _mt(1, 2, 0.5, 2.0, n0=6.0, split_iters=3), units=[(0, 0), (0, 3)])
    tot = rep.notes[-1]
    assert tot["split_now"] > 0 and tot["forced_absorb"] > 0, tot


@pytest.mark.gpu
def test_maintainer_deferred_fp32():
    """Alg. 1 in full: nothing is resident before the first query, so invalid insertions are
    buffered as singletons; queries every 12 frames make their selection resident, select
    singletons, and carry out the deferred splits."""
    wl = inputs.CONFIGS[0].scaled(name="maint_deferred_fp32", n_clusters=24, top_k=4)
    rep = harness.run_maintained(wl, _mt(2, 3, 1.5, 6.0, buf_max=12), query_every=12)
    tot = rep.notes[-1]
    assert tot["deferred"] > 0 and tot["split_deferred"] > 0, tot
    assert rep.max_out_err <= 1e-4


@pytest.mark.gpu
def test_maintainer_deferred_bf16_small_buffer():
    """D = 128, bf16, a 3-entry buffer that overflows (forced absorbs) and a multi-token question."""
    wl = inputs.CONFIGS[1].scaled(name="maint_deferred_bf16", n_frames=224, n_scenes=14, n_clusters=20,
                                  top_k=3, question_tokens=5)
    rep = harness.run_maintained(wl, _mt(2, 2, 0.5, 2.0, n0=6.0, split_iters=3, buf_max=3),
                                 units=[(0, 1), (0, 2)], query_every=20)
    tot = rep.notes[-1]
    assert tot["deferred"] > 0 and tot["forced_absorb"] > 0, tot


@pytest.mark.gpu
@pytest.mark.parametrize("mode", [1, 2])
def test_maintainer_on_the_host_tier_fp32(mode):
    """Sec. VI on the offloading tier: clusters live in pinned host memory, "in GPU memory" (Alg. 1
    line 4) means that the GPU cluster cache holds frames of the cluster.  Whole maintainer state,
    selections (singletons included), token lists and attention against the oracle, whose residency
    flags come from the working-set model; the library's cache directory against the model's after
    every call; splits move no page (hit / miss / byte counters equal the model's)."""
    wl = inputs.CONFIGS[0].scaled(name="maint_host_fp32", n_clusters=24, top_k=4)
    rep = harness.run_maintained(wl, _mt(mode, 3, 1.5, 6.0, buf_max=12 if mode == 2 else 0), query_every=12,
                                 host=dict(slab_frames=4, cache_pages_per_unit=100, cache_fraction=0.25))
    tot = rep.notes[-1]
    print("  ", tot, flush=True)
    assert tot["split_now"] + tot["split_deferred"] > 0, tot
    if mode == 2:
        assert tot["deferred"] > 0 and tot["split_deferred"] > 0, tot
    assert tot["cache"]["evictions"] > 0 and tot["cache"]["hits"] > 0
    assert rep.max_out_err <= 1e-4


@pytest.mark.gpu
def test_maintainer_deferred_on_the_host_tier_bf16_small_buffer():
    """D = 128, bf16 pages (MFMA attention over cache slots), ragged pages, a buffer that overflows."""
    wl = inputs.CONFIGS[1].scaled(name="maint_host_bf16", n_frames=224, n_scenes=14, n_clusters=20,
                                  top_k=3, question_tokens=5, tokens_per_frame=50, n_kv_heads=2, n_q_heads=14)
    rep = harness.run_maintained(wl, _mt(2, 2, 0.5, 2.0, n0=6.0, split_iters=3, buf_max=3), query_every=20,
                                 host=dict(slab_frames=3, cache_pages_per_unit=150, cache_fraction=0.3))
    tot = rep.notes[-1]
    print("  ", tot, flush=True)
    assert tot["deferred"] > 0 and tot["forced_absorb"] > 0, tot
    assert tot["cache"]["hits"] > 0


@pytest.mark.gpu
def test_maintainer_config_errors():
    wl = inputs.CONFIGS[0]
    base = dict(maint_mode=binding.MAINT_EAGER, init_clusters=4, tau_min=1.0, tau_max=2.0, tau_n0=8.0)
    for bad in (dict(tau_n0=0.0), dict(init_clusters=wl.n_clusters + 1), dict(maint_mode=3),
                dict(recluster_every=64),
                dict(maint_mode=binding.MAINT_DEFERRED, buffer_max=1024)):
        kw = dict(base); kw.update(bad)
        with pytest.raises(binding.MosaicError) as ei:
            binding.workspace_sizes(binding.config_for(wl, **kw))
        assert ei.value.code == binding.EINVAL
    m = binding.Mosaic(binding.config_for(wl))          # maintainer off: the observer says so
    with pytest.raises(binding.MosaicError):
        m.maintainer()
    m.close()


# ---------------------------------------------------------------------------
# Retrieval augmentation (paper Sec. V-C)
# ---------------------------------------------------------------------------
@pytest.mark.gpu
@pytest.mark.parametrize("window,reps", [(6, False), (0, True), (9, True)])
def test_augmentation_fp32(window, reps):
    rep = harness.run_augmented(inputs.CONFIGS[0], window, reps)
    assert rep.max_out_err <= 1e-4


@pytest.mark.gpu
def test_augmentation_bf16_mfma_decode_and_question():
    wl = inputs.CONFIGS[1].scaled(name="aug_bf16", n_frames=160, n_scenes=10, n_clusters=12, top_k=3,
                                  question_tokens=37)
    rep = harness.run_augmented(wl, 5, True, units=[(0, 0), (0, 3)], decode_steps=3)
    assert rep.max_out_err <= 2e-2


@pytest.mark.gpu
def test_augmentation_window_larger_than_stream_and_recluster():
    """Window >= frames ingested: nothing comes from the clusters; with re-clustering on, the
    representatives' values follow the changed membership."""
    wl = inputs.CONFIGS[0].scaled(name="aug_recluster", recluster_every=48)
    rep = harness.run_augmented(wl, 1000, True)
    assert rep.max_out_err <= 1e-4


@pytest.mark.gpu
def test_augmentation_is_bitwise_repeatable():
    """The pseudo tokens' values are per-cluster sums over the member frames, added in ascending frame
    order by one workgroup per cluster: two contexts fed the same stream, and a reset + re-run of one
    of them, give bit-identical outputs and log-sum-exps."""
    wl = inputs.CONFIGS[1].scaled(name="aug_repeat", n_frames=224, n_scenes=9, n_clusters=12, top_k=3,
                                  question_tokens=5)
    st = inputs.SceneStream(wl)
    K, V = [x.to(DEV) for x in st.frames(0, wl.n_frames)]
    qs = [st.question(st.draw_scene(), n, i).to(DEV) for i, n in enumerate((5, 1, 1))]

    def run(m):
        m.ingest_frame(K, V)
        res = []
        for q in qs:
            m.retrieve(0, q[0].contiguous())
            o, l = m.attend(0, q[0].contiguous())
            res.append((o.clone(), l.clone()))
        torch.cuda.synchronize()
        return res
    cfg = dict(aug_global_reps=1, aug_window_frames=4)
    m1 = binding.Mosaic(binding.config_for(wl, **cfg), device=DEV)
    m2 = binding.Mosaic(binding.config_for(wl, **cfg), device=DEV)
    a, b = run(m1), run(m2)
    m1.reset()
    c = run(m1)
    for x, y, z in zip(a, b, c):
        assert torch.equal(x[0], y[0]) and torch.equal(x[1], y[1])
        assert torch.equal(x[0], z[0]) and torch.equal(x[1], z[1])
    m1.close(); m2.close()


@pytest.mark.gpu
def test_augmentation_config_errors():
    wl = inputs.CONFIGS[0]
    for bad in (dict(aug_global_reps=2), dict(aug_window_frames=-1), dict(aug_window_frames=2000),
                dict(aug_window_frames=4, tier=binding.TIER_HOST),
                dict(aug_global_reps=1, maint_mode=binding.MAINT_DEFERRED, init_clusters=4, tau_n0=8.0)):
        with pytest.raises(binding.MosaicError) as ei:
            binding.workspace_sizes(binding.config_for(wl, **bad))
        assert ei.value.code == binding.EINVAL


# ---------------------------------------------------------------------------
# Overlap-aware cross-layer prefetch (paper Sec. VII-B), host tier
# ---------------------------------------------------------------------------
@pytest.mark.gpu
def test_prefetch_never_changes_results_and_perfect_proxy_covers_everything():
    """Layer l's query predicts layer l+1's clusters.  Results must be bitwise those of the run
    without prefetch, whatever the proxy; with the actual next-layer query as the 'proxy' every
    cluster the retrieval selects has been prefetched (no completion fetch), with an unrelated
    proxy the completion step fetches the rest."""
    wl = _small(n_layers=3, n_frames=160, n_clusters=10, top_k=3)
    st = inputs.SceneStream(wl)
    K, V = [x.to(DEV) for x in st.frames(0, wl.n_frames)]
    qs = [st.question(st.draw_scene(), 1, i).to(DEV) for i in range(5)]
    unrelated = [st.question(st.draw_scene(), 1, 100 + i).to(DEV) for i in range(5)]

    def run(mode):
        m = _ingest_all(wl, K, V, (16,), **HOST)
        res = []
        for qi, q in enumerate(qs):
            o = torch.empty_like(q)
            l = torch.empty(q.shape[:-1], dtype=torch.float32, device=DEV)
            for layer in range(wl.n_layers):
                m.retrieve(layer, q[layer].contiguous())
                if layer + 1 < wl.n_layers and mode != "none":
                    proxy = q[layer + 1] if mode == "perfect" else unrelated[qi][layer]
                    m.prefetch(layer + 1, proxy.contiguous())
                m.attend(layer, q[layer].contiguous(), o[layer], l[layer])
            torch.cuda.synchronize()
            res.append((o.clone(), l.clone()))
        s = m.stats()
        m.close()
        return res, s

    base, s0 = run("none")
    perfect, s1 = run("perfect")
    wrong, s2 = run("unrelated")
    for a, b, c in zip(base, perfect, wrong):
        assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])
        assert torch.equal(a[0], c[0]) and torch.equal(a[1], c[1])
    assert s0.prefetch_calls == 0 and s1.prefetch_calls == 2 * len(qs) == s2.prefetch_calls
    # retrievals of layers 1.. found everything in the cache; only layer 0 (never predicted) misses
    per_call = wl.n_kv_heads * wl.top_k
    assert s1.prefetch_fetched > 0 and s1.prefetch_useful == s1.prefetch_fetched
    assert s1.cache_misses <= len(qs) * per_call and s1.cache_misses < s0.cache_misses
    assert s2.prefetch_useful <= s2.prefetch_fetched and s2.cache_misses > s1.cache_misses
    assert s1.cache_hits + s1.cache_misses == s0.cache_hits + s0.cache_misses == len(qs) * wl.n_layers * per_call


@pytest.mark.gpu
@pytest.mark.parametrize("prefetch_top_k", [0, 2])
def test_prefetch_follows_the_oracle_predict_verify_complete(prefetch_top_k):
    """Sec. VII-B against the oracle: for every layer transition and unit, the clusters predicted
    with the previous layer's query, the clusters the actual query selects and the completion set
    come from oracle units + the working-set model; the library's cache directory must equal the
    model's after every call, and its prefetch / hit / miss / byte counters at the end."""
    wl = _small(n_layers=3, n_frames=160, n_clusters=10, top_k=3, warmup_frames=80)
    st = inputs.SceneStream(wl)
    K, V = st.frames(0, wl.n_frames)
    Kd, Vd = K.to(DEV), V.to(DEV)
    pages = 120           # a unit's three largest clusters hold at most 116 of the 160 frames
    m = binding.Mosaic(binding.config_for(wl, prefetch_top_k=prefetch_top_k, cache_pages_per_unit=pages,
                                          cache_fraction=0.4, **HOST), device=DEV)
    rep = harness.Report()
    units = [(l, h) for l in range(wl.n_layers) for h in range(wl.n_kv_heads)]
    oracles = harness.ingest_with_parity(m, wl, Kd, Vd, units, rep)
    H, G, C = wl.n_kv_heads, wl.group, wl.n_clusters
    models = {key: cache_model.ClusterCacheModel(pages, 4) for key in units}

    mems = {key: cache_model.membership_from_assignments(o.assignments()) for key, o in oracles.items()}

    def check_directory(where):
        d = m.cache_directory()
        for (l, h), mod in models.items():
            np.testing.assert_array_equal(d[l * H + h], _model_directory(mod, C, mems[(l, h)]), err_msg=f"{where}, unit {(l, h)}")

    for qi in range(6):
        q = st.question(st.draw_scene(), 1, qi).to(DEV)
        q_h = q.float().cpu().numpy().astype(np.float64)
        # a related proxy on even questions (the next layer's own query plus noise-free copy of this
        # layer's), an unrelated one on odd questions
        other = st.question(st.draw_scene(), 1, 50 + qi).to(DEV)
        m.retrieve(0, q[0].contiguous())
        for h in range(H):
            o = oracles[(0, h)]
            models[(0, h)].access(o.retrieve(q_h[0], h, G, wl.top_k)[0], mems[(0, h)])
        check_directory(f"question {qi}, layer 0 retrieve")
        for layer in range(wl.n_layers):
            if layer + 1 < wl.n_layers:
                proxy = q[layer] if qi % 2 == 0 else other[layer]
                proxy_h = proxy.float().cpu().numpy().astype(np.float64)
                m.prefetch(layer + 1, proxy.contiguous())
                rounds = {}
                for h in range(H):
                    # the model's prefetch step now, its verification + completion after the retrieve
                    o = oracles[(layer + 1, h)]
                    ids_p = [int(c) for c in o.retrieve(proxy_h, h, G, wl.top_k)[0]]
                    if prefetch_top_k:
                        ids_p = ids_p[:prefetch_top_k]
                    rounds[h] = models[(layer + 1, h)].access(ids_p, mems[(layer + 1, h)], prefetch=True)
                check_directory(f"question {qi}, prefetch for layer {layer + 1}")
            m.attend(layer, q[layer].contiguous())
            if layer + 1 < wl.n_layers:
                m.retrieve(layer + 1, q[layer + 1].contiguous())
                ids, n_ids, _, _ = m.selection(layer + 1)
                for h in range(H):
                    o = oracles[(layer + 1, h)]
                    want = o.retrieve(q_h[layer + 1], h, G, wl.top_k)[0]
                    np.testing.assert_array_equal(ids[h, : n_ids[h]], want)
                    models[(layer + 1, h)].access(want, mems[(layer + 1, h)])
                check_directory(f"question {qi}, layer {layer + 1} retrieve (verification + completion)")
        torch.cuda.synchronize()
    s = m.stats()
    tot = lambda name: sum(getattr(x, name) for x in models.values())
    assert (s.prefetch_fetched, s.prefetch_useful) == (tot("prefetch_fetched"), tot("prefetch_useful"))
    assert (s.cache_hits, s.cache_misses) == (tot("hits"), tot("misses"))
    page_bytes = 2 * wl.tokens_per_frame * wl.head_dim * 2
    assert s.h2d_bytes == tot("pages_moved") * page_bytes
    assert s.prefetch_calls == 6 * (wl.n_layers - 1)
    assert tot("prefetch_fetched") > 0 and tot("evictions") > 0 and tot("prefetch_useful") > 0
    m.close()


@pytest.mark.gpu
def test_prefetch_round_of_the_oracle_matches_the_library_on_one_transition():
    """cache_model.prefetch_round (predict, verify, complete in one call) on a cold cache against
    the library's prefetch + retrieve for one layer transition."""
    wl = _small(n_layers=2, n_frames=128, n_clusters=8, top_k=3)
    st = inputs.SceneStream(wl)
    K, V = st.frames(0, wl.n_frames)
    Kd, Vd = K.to(DEV), V.to(DEV)
    m = binding.Mosaic(binding.config_for(wl, cache_pages_per_unit=wl.n_frames, cache_fraction=1.0, **HOST), device=DEV)
    rep = harness.Report()
    units = [(1, h) for h in range(wl.n_kv_heads)]
    oracles = harness.ingest_with_parity(m, wl, Kd, Vd, units, rep)
    q = st.question(st.draw_scene(), 1, 0).to(DEV)
    q_h = q.float().cpu().numpy().astype(np.float64)
    m.prefetch(1, q[0].contiguous())
    m.retrieve(1, q[1].contiguous())
    d = m.cache_directory()
    s = m.stats()
    fetched = useful = misses = 0
    for (l, h), o in oracles.items():
        mod = cache_model.ClusterCacheModel(wl.n_frames, wl.n_clusters)
        out = cache_model.prefetch_round(o, mod, q_h[0], q_h[1], h, wl.group, wl.top_k)
        np.testing.assert_array_equal(d[l * wl.n_kv_heads + h],
                                      _model_directory(mod, wl.n_clusters, cache_model.membership_from_assignments(o.assignments())))
        assert set(out["actual"]) - set(out["predicted"]) == {c for c, _ in out["completion"]}
        fetched += mod.prefetch_fetched; useful += mod.prefetch_useful; misses += mod.misses
    assert (s.prefetch_fetched, s.prefetch_useful, s.cache_misses) == (fetched, useful, misses)
    m.close()


@pytest.mark.gpu
def test_prefetch_errors():
    wl = _small(n_frames=96)
    st = inputs.SceneStream(wl)
    K, V = [x.to(DEV) for x in st.frames(0, wl.n_frames)]
    q = st.question(st.draw_scene(), 1, 0).to(DEV)
    m = _ingest_all(wl, K, V, (16,))                     # HBM tier: nothing to prefetch
    with pytest.raises(binding.MosaicError) as ei:
        m.prefetch(0, q[0].contiguous())
    assert ei.value.code == binding.EINVAL
    m.close()
    m = _ingest_all(wl, K, V, (16,), **HOST)
    m.prefetch(0, q[0].contiguous())
    with pytest.raises(binding.MosaicError) as ei:       # a prediction is not a selection
        m.attend(0, q[0].contiguous())
    assert ei.value.code == binding.ENOTREADY
    with pytest.raises(binding.MosaicError) as ei:
        m._check(m._L.mosaic_prefetch(m._h, -1, q.data_ptr(), 1))
    assert ei.value.code == binding.EINVAL
    m.retrieve(0, q[0].contiguous()); m.attend(0, q[0].contiguous())
    torch.cuda.synchronize()
    m.close()


# ---------------------------------------------------------------------------
# Nested visual-semantic hierarchy and two-stage retrieval (paper Sec. V-B, V-C)
# ---------------------------------------------------------------------------
@pytest.mark.gpu
@pytest.mark.parametrize("score_mode", [0, 1])
def test_nested_fp32(score_mode):
    wl = inputs.CONFIGS[0].scaled(name="nested_fp32", visual_dim=24, n_visual=4, n_clusters=16, top_k=4)
    rep = harness.run_nested(wl, 4, 2, score_mode=score_mode)
    _report(rep)
    assert rep.max_out_err <= 1e-4 and rep.online_decisions > 0


@pytest.mark.gpu
def test_nested_bf16_ragged_visual_dim_and_short_partitions():
    """Dv not a multiple of 64, more ids per partition than some partitions have warm-up members
    (ids that are never started), a question spanning several row tiles, and decode steps."""
    wl = inputs.CONFIGS[1].scaled(name="nested_bf16", n_frames=200, n_scenes=14, n_clusters=48, top_k=5,
                                  question_tokens=21, visual_dim=100, n_visual=5, warmup_frames=60)
    rep = harness.run_nested(wl, 6, 2, units=[(0, 0), (0, 2), (0, 3)], decode_steps=3)
    _report(rep)
    assert rep.max_out_err <= 2e-2


@pytest.mark.gpu
def test_nested_two_layers_all_partitions_kept_equals_flat_selection_over_nested_clusters():
    """top_partitions = P: the first stage prunes nothing, so every non-empty cluster is scored."""
    wl = inputs.CONFIGS[0].scaled(name="nested_2l", n_layers=2, visual_dim=64, n_visual=3, n_clusters=12,
                                  top_k=3)
    rep = harness.run_nested(wl, 3, 3)
    _report(rep)
    assert rep.max_out_err <= 1e-4


@pytest.mark.gpu
def test_nested_single_partition_is_bitwise_the_flat_index():
    wl = inputs.CONFIGS[0].scaled(name="nested_p1", visual_dim=8)
    st = inputs.SceneStream(wl)
    K, V = st.frames(0, wl.n_frames)
    E = st.embeddings(0, wl.n_frames).to(DEV)
    Kd, Vd = K.to(DEV), V.to(DEV)
    flat = binding.Mosaic(binding.config_for(wl), device=DEV)
    nest = binding.Mosaic(binding.config_for(wl, n_partitions=1, visual_dim=8, top_partitions=1), device=DEV)
    flat.ingest_frame(Kd, Vd)
    nest.ingest_frame_visual(Kd, Vd, E)
    np.testing.assert_array_equal(flat.assignments(), nest.assignments())
    Rf, Nf = flat.centroids()
    Rn, Nn = nest.centroids()
    np.testing.assert_array_equal(Rf, Rn)
    np.testing.assert_array_equal(Nf, Nn)
    q = st.question(0, 4, 0).to(DEV)[0].contiguous()
    for m in (flat, nest):
        m.retrieve(0, q)
    of, lf = flat.attend(0, q)
    on, ln = nest.attend(0, q)
    torch.cuda.synchronize()
    a, b = flat.selection(0), nest.selection(0)
    np.testing.assert_array_equal(a[0], b[0])
    np.testing.assert_array_equal(a[2], b[2])
    assert torch.equal(of, on) and torch.equal(lf, ln)
    flat.close(); nest.close()


@pytest.mark.gpu
def test_nested_config_and_call_errors():
    wl = inputs.CONFIGS[0].scaled(visual_dim=8)
    ok = dict(n_partitions=4, visual_dim=8, top_partitions=2)
    for bad in (dict(n_partitions=3), dict(n_partitions=65), dict(visual_dim=0), dict(visual_dim=5000),
                dict(top_partitions=5), dict(tier=binding.TIER_HOST), dict(recluster_every=64),
                dict(aug_window_frames=4),
                dict(maint_mode=binding.MAINT_EAGER, init_clusters=4, tau_n0=8.0)):
        kw = dict(ok); kw.update(bad)
        with pytest.raises(binding.MosaicError) as ei:
            binding.workspace_sizes(binding.config_for(wl, **kw))
        assert ei.value.code == binding.EINVAL
    st = inputs.SceneStream(wl)
    K, V = st.frames(0, 2)
    E = st.embeddings(0, 2).to(DEV)
    m = binding.Mosaic(binding.config_for(wl, **ok), device=DEV)
    with pytest.raises(binding.MosaicError) as ei:
        m.ingest_frame(K.to(DEV), V.to(DEV))                 # needs the embeddings
    assert ei.value.code == binding.EINVAL
    m.ingest_frame_visual(K.to(DEV), V.to(DEV), E)
    assert np.all(m.partitions()["frame_to_partition"] == -1)   # still warming up
    m.close()
    m = binding.Mosaic(binding.config_for(wl), device=DEV)
    with pytest.raises(binding.MosaicError) as ei:
        m.ingest_frame_visual(K.to(DEV), V.to(DEV), E)       # flat index: no visual level
    assert ei.value.code == binding.EINVAL
    with pytest.raises(binding.MosaicError):
        m.partitions()
    m.close()


# ---------------------------------------------------------------------------
# Large cluster tables: the binned exact top-k (more than 128 representatives)
# ---------------------------------------------------------------------------
@pytest.mark.gpu
@pytest.mark.parametrize("C,k", [(160, 24), (384, 1), (384, 383), (1024, 48), (1024, 1024)])
def test_large_cluster_table_topk(C, k):
    """k = 1, a mid-sized k and k close to the number of clusters (all bins become candidates);
    1024 is the largest table the library accepts."""
    wl = _small(name=f"large_table_{C}_{k}", n_frames=2 * C + 40, n_scenes=40, n_clusters=C, top_k=k,
                tokens_per_frame=8, question_tokens=3)
    rep = harness.run_workload(wl, units=[(0, 0), (0, 3)], n_questions=2, decode_steps=3)
    _report(rep)
    assert rep.max_out_err <= 2e-2


@pytest.mark.gpu
def test_nested_reset_and_reingest_reproduces_the_state():
    wl = inputs.CONFIGS[0].scaled(name="nested_reset", visual_dim=16, n_visual=3, n_clusters=16)
    st = inputs.SceneStream(wl)
    K, V = st.frames(0, wl.n_frames)
    E = st.embeddings(0, wl.n_frames).to(DEV)
    Kd, Vd = K.to(DEV), V.to(DEV)
    m = binding.Mosaic(binding.config_for(wl, n_partitions=4, visual_dim=16, top_partitions=2), device=DEV)
    snaps = []
    for batch in (7, 128):                       # different call sizes, same result
        m.reset()
        assert m.stats().frames_ingested == 0
        for f in range(0, wl.n_frames, batch):
            m.ingest_frame_visual(Kd[f:f + batch].contiguous(), Vd[f:f + batch].contiguous(),
                                  E[f:f + batch].contiguous())
        p = m.partitions()
        R, N = m.centroids()
        snaps.append((m.assignments().copy(), R.copy(), N.copy(), p["frame_to_partition"].copy(),
                      p["visual_r"].copy(), p["part_r"].copy(), p["part_n"].copy()))
    for a, b in zip(*snaps):
        np.testing.assert_array_equal(a, b)
    m.close()


# ---------------------------------------------------------------------------
# mosaic_decode_step: retrieve + attend in one call / one kernel
# ---------------------------------------------------------------------------
@pytest.mark.gpu
@pytest.mark.parametrize("kw", [
    dict(),                                                   # the realistic head shape, C = 12
    dict(n_clusters=200, top_k=9, n_frames=460),              # C > 128: one thread per entry in the ranking
    dict(tokens_per_frame=50, n_frames=140),                  # ragged pages (two chunks, the second partly empty)
    dict(head_dim=64, n_q_heads=8, n_kv_heads=2),             # D = 64, G = 4
    dict(n_layers=2, n_frames=120),                           # two layers, one call each
])
def test_decode_step_fused_parity(kw):
    wl = _small(name="fused", **kw)
    rep = harness.run_workload(wl, n_questions=0, decode_steps=4, layer_mode="fused")
    _report(rep)
    assert rep.max_out_err <= 2e-2


@pytest.mark.gpu
@pytest.mark.parametrize("kw", [
    dict(),                                                          # D = 128, 4 KV heads, G = 7
    dict(head_dim=64, n_q_heads=8, n_kv_heads=2, tokens_per_frame=50, n_clusters=9, top_k=3),   # ragged pages, G = 4
    dict(n_q_heads=16, n_kv_heads=1, n_clusters=200, top_k=150, n_frames=420, n_scenes=30),     # G = 16, one unit, C > 128
    dict(n_layers=3, n_frames=2600, n_scenes=60, n_clusters=40, top_k=6),                       # frame lists beyond one batch
])
def test_decode_step_one_launch_with_proportional_splits_parity(kw):
    """mosaic_decode_step in its one-launch form for bandwidth-bound steps (the launch's first workgroups
    select and publish, all workgroups then share out the pages in proportion to the units' sizes),
    forced on small workloads: scores, ids, token lists and attention against the oracle, bitwise equal
    to mosaic_retrieve + mosaic_attend (the same splits), and no in-kernel wait ever ran out."""
    wl = _small(name="layer_fused", **kw)
    rep = harness.run_workload(wl, n_questions=0, decode_steps=3, layer_mode="fused", decode_fused_max_mib=-1)
    _report(rep)
    assert [v for (k_, v) in rep.notes if k_ == "decode_step_fused"] == [2] * (3 * wl.n_layers)
    st = inputs.SceneStream(wl)
    K, V = [x.to(DEV) for x in st.frames(0, wl.n_frames)]
    a = _ingest_all(wl, K, V, (16,), decode_fused_max_mib=-1)
    b = _ingest_all(wl, K, V, (16,), decode_fused_max_mib=-2)
    for i in range(4):
        q = st.question(st.draw_scene(), 1, i).to(DEV)
        for l in range(wl.n_layers):
            oa, la = a.decode_step(l, q[l].contiguous())
            ob, lb = b.decode_step(l, q[l].contiguous())
            torch.cuda.synchronize()
            assert a.stats().last_decode_fused == 2 and b.stats().last_decode_fused == 0
            assert torch.equal(oa, ob) and torch.equal(la, lb)
            sa, sb = a.selection(l), b.selection(l)
            np.testing.assert_array_equal(sa[0], sb[0]); np.testing.assert_array_equal(sa[2], sb[2])
            for ta, tb in zip(sa[3], sb[3]):
                np.testing.assert_array_equal(ta, tb)
    assert a.stats().sync_timeouts == 0
    a.close(); b.close()


@pytest.mark.gpu
def test_decode_step_equals_retrieve_then_attend():
    """Same ids, scores and token lists bit for bit; outputs equal up to the merge order of the
    fp32 partials (equal splits per unit instead of proportional ones)."""
    wl = _small(name="fused_vs_calls", n_frames=300, n_clusters=24, top_k=6)
    st = inputs.SceneStream(wl)
    K, V = st.frames(0, wl.n_frames)
    a = binding.Mosaic(binding.config_for(wl), device=DEV)
    b = binding.Mosaic(binding.config_for(wl), device=DEV)
    for m in (a, b):
        m.ingest_frame(K.to(DEV), V.to(DEV))
    for i in range(3):
        q = st.question(st.draw_scene(), 1, i).to(DEV)[0].contiguous()
        a.retrieve(0, q)
        oa, la = a.attend(0, q)
        ob, lb = b.decode_step(0, q)
        torch.cuda.synchronize()
        assert b.stats().last_decode_fused == 1           # the single-kernel path is what is compared
        sa, sb = a.selection(0), b.selection(0)
        np.testing.assert_array_equal(sa[0], sb[0])
        np.testing.assert_array_equal(sa[1], sb[1])
        np.testing.assert_array_equal(sa[2], sb[2])
        for x, y in zip(sa[3], sb[3]):
            np.testing.assert_array_equal(x, y)
        assert (oa.float() - ob.float()).abs().max().item() <= 2e-2
        assert (la - lb).abs().max().item() <= 1e-3
        # a plain attend after the fused step uses the selection it left behind
        oc, lc = b.attend(0, q)
        torch.cuda.synchronize()
        assert torch.equal(oc, oa) and torch.equal(lc, la)
    a.close(); b.close()


@pytest.mark.gpu
def test_decode_step_falls_back_where_the_fused_kernel_does_not_apply():
    # fp32 KV (vector-ALU attention), a multi-token question, all layers at once, the host tier
    rep = harness.run_workload(inputs.CONFIGS[0], n_questions=1, decode_steps=2, layer_mode="fused")
    assert rep.max_out_err <= 1e-4
    wl = _small(name="fused_fallback", question_tokens=5)
    rep = harness.run_workload(wl, n_questions=2, decode_steps=0, layer_mode="fused")
    assert rep.max_out_err <= 2e-2
    m = binding.Mosaic(binding.config_for(wl), device=DEV)
    q = torch.zeros((1, 28, 128), dtype=torch.bfloat16, device=DEV)
    with pytest.raises(binding.MosaicError) as ei:
        m.decode_step(0, q)                                   # nothing ingested yet
    assert ei.value.code == binding.ENOTREADY
    st = inputs.SceneStream(wl)
    K, V = st.frames(0, wl.n_frames)
    m.ingest_frame(K.to(DEV), V.to(DEV))
    q5 = st.question(0, 5, 0).to(DEV)[0].contiguous()         # 35 query rows per KV head: two calls
    m.decode_step(0, q5)
    assert m.stats().last_decode_fused == 0
    m.decode_step(0, q5[:1].contiguous())                     # one token: the fused kernel
    assert m.stats().last_decode_fused == 1
    m.close()


# --------------------------------------------------------------------------
# the extensions at the sizes the benchmark runs them at (one layer of the stack)
# --------------------------------------------------------------------------
@pytest.mark.parametrize("mode,query_every", [(1, 0), (2, 64)])
def test_maintainer_benchmark_recipe(mode, query_every):
    """Maintainer on the config-2 stream recipe (4096 frames of 64 tokens, geometric scenes, 5 %
    outlier tokens), 32 initial clusters in a table of 256, the benchmark's thresholds; eager, and
    deferred with a decode query every 64 frames.  One layer, two units followed by the oracle."""
    wl = inputs.CONFIGS[2].scaled(name="cfg2_recipe_maintained", n_layers=1, n_clusters=256, top_k=16,
                                  recluster_every=0)
    mt = dict(mode=mode, c_init=32, tau_min=4.0, tau_max=16.0, n0=32.0, split_iters=4, buf_max=256)
    rep = harness.run_maintained(wl, mt, units=[(0, 1), (0, 3)], batch_pattern=(16, 1, 16, 5),
                                 query_every=query_every, question_tokens=1)
    _report(rep)
    tot = rep.notes[-1]
    print("  ", tot, flush=True)
    assert tot["split_now"] + tot["split_deferred"] > 0
    assert rep.max_out_err <= 2e-2


def test_nested_benchmark_recipe():
    """Nested index on the config-2 stream recipe: 512 clusters in 16 visual partitions, the 4 best
    partitions kept, 1024-wide visual embeddings; one layer, one unit followed by the oracle."""
    wl = inputs.CONFIGS[2].scaled(name="cfg2_recipe_nested", n_layers=1, n_clusters=512, top_k=16,
                                  recluster_every=0, visual_dim=1024, n_visual=16, visual_key_corr=0.5)
    rep = harness.run_nested(wl, 16, 4, units=[(0, 2)], batch_pattern=(16, 1, 16, 7), n_questions=1,
                             decode_steps=3)
    _report(rep)
    assert rep.max_out_err <= 2e-2 and rep.online_decisions > 0


def test_augmentation_on_a_store_beyond_the_caches():
    """840 MB of stored KV: the decode kernel's instantiation with the representatives' extra workgroups
    and non-temporal K/V loads (no benchmark leg combines the two)."""
    wl = inputs.CONFIGS[1].scaled(name="aug_long_stream", n_frames=6400, n_scenes=250, question_tokens=2)
    rep = harness.run_augmented(wl, 16, True, units=[(0, 2)], decode_steps=2, ingest_between=False)
    _report(rep)
    assert rep.max_out_err <= 2e-2


def test_augmentation_cfg1_full_size():
    """Config 1 at full size with the benchmark's augmentation (window of 16 frames and the
    representatives as pseudo-KV)."""
    rep = harness.run_augmented(inputs.CONFIGS[1], 16, True, decode_steps=3)
    _report(rep)
    assert rep.max_out_err <= 2e-2


# --------------------------------------------------------------------------
# ranking: scores that differ only beyond fp32 resolution
# --------------------------------------------------------------------------
@pytest.mark.parametrize("higher_id_wins", [False, True])
@pytest.mark.parametrize("n_clusters", [4, 160])
def test_topk_scores_that_collide_in_fp32_are_ordered_exactly(higher_id_wins, n_clusters):
    """The pair count of the ranking compares fp32 roundings of the scores and settles collisions in
    fp64.  Two scenes whose constant key vectors differ by 2^-20 in one channel the query does not
    use give two clusters whose scores differ by ~1e-12 relative: equal in fp32, ordered in fp64.
    With k = 1 the selection must be the cluster the oracle picks, whichever of the two ids it has
    (table of 4: the direct count; table of 160: the binned path), through mosaic_retrieve and
    through mosaic_decode_step."""
    from oracle import mosaic_oracle as orc
    C, D, T, Hkv, G = n_clusters, 128, 8, 1, 2
    W = 2 * C
    F = W + 8
    wl = inputs.CONFIGS[1].scaled(name="fp32_collision", n_layers=1, n_q_heads=Hkv * G, n_kv_heads=Hkv, head_dim=D,
                                  tokens_per_frame=T, n_frames=F, n_clusters=C, top_k=1, warmup_frames=W)
    rng = np.random.Generator(np.random.PCG64(42))
    base = rng.standard_normal((C, D)).astype(np.float32)
    base = torch.tensor(base).to(torch.bfloat16).float().numpy()       # bf16-representable centres
    base[:, 0] = 0.0
    base[1] = base[0]                                                   # scenes 0 and 1: same vector ...
    base[1 if not higher_id_wins else 0, 0] = 2.0 ** -20                # ... but for channel 0 of one of them
    # warm-up frames 2j, 2j+1 show scene j (the K-means seeds are frames 0, 2, 4, ...); then more of 0 and 1
    scene_of = [j // 2 for j in range(W)] + [0, 1] * 4
    K = torch.tensor(np.stack([np.tile(base[sc], (1, Hkv, T, 1)) for sc in scene_of])).to(torch.bfloat16)
    V = torch.tensor(rng.standard_normal(K.shape).astype(np.float32)).to(torch.bfloat16)
    q = torch.tensor(np.tile(base[0] + 0.25 * base[2], (1, 1, Hkv * G, 1))).to(torch.bfloat16)   # [L][Tq][Hq][D]
    q[..., 0] = 0.0
    Kd, Vd, qd = K.to(DEV), V.to(DEV), q.to(DEV)
    o = orc.OracleUnit(C, D, T, F, W, wl.lloyd_iters, 0)
    Kc = inputs.unit_pages(K, 0, 0)
    for f in range(F):
        o.ingest(Kc[f])
    ids_o, sc_o, tok_o, gap = o.retrieve(q[0].float().numpy().astype(np.float64), 0, G, 1)
    top2 = np.sort(sc_o[o.sizes() > 0])[::-1][:2]
    rel = (top2[0] - top2[1]) / abs(top2[0])
    assert 0 < rel < 1e-9 and np.float32(top2[0]) == np.float32(top2[1]), (top2, rel)   # the case is what it claims
    assert int(ids_o[0]) == (1 if higher_id_wins else 0)
    m = binding.Mosaic(binding.config_for(wl), device=DEV)
    for f in range(0, F, 5):
        m.ingest_frame(Kd[f:f + 5].contiguous(), Vd[f:f + 5].contiguous())
    np.testing.assert_array_equal(m.assignments()[0], o.assignments())
    m.retrieve(0, qd[0].contiguous())
    ids, n_ids, scores, toks = m.selection(0)
    assert n_ids[0] == 1 and int(ids[0, 0]) == int(ids_o[0])
    np.testing.assert_array_equal(toks[0], tok_o)
    m.decode_step(0, qd[0].contiguous())
    if C <= 256:
        assert m.stats().last_decode_fused == 1
    ids, n_ids, scores, toks = m.selection(0)
    assert n_ids[0] == 1 and int(ids[0, 0]) == int(ids_o[0])
    m.close()
