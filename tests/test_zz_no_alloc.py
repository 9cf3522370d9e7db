"""mosaic_attend_static (attention with its split partials in the library's static device buffer,
for callers that cannot allocate) against mosaic_attend, through the C ABI.  The same kernels run
with the same split counts wherever the static buffer is at least as large as the arena's, so the
two must agree bit for bit there, and to the attention bar of the parity harness where the static
buffer forces fewer splits."""
import numpy as np
import pytest
import torch

from paper_2604_10060_amd import binding, inputs
from tests import harness

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _context(wl):
    st = inputs.SceneStream(wl)
    K, V = [x.to(DEV) for x in st.frames(0, wl.n_frames)]
    m = binding.Mosaic(binding.config_for(wl), device=DEV)
    m.ingest_frame(K, V)
    return st, m


def _both(m, layer, q):
    """-> (out, lse) of mosaic_attend and of mosaic_attend_static for the current selection"""
    ref = m.attend(layer, q)
    out = torch.full_like(ref[0], float("nan"))
    lse = torch.full_like(ref[1], float("nan"))
    m.attend_static(layer, q, out, lse)
    torch.cuda.synchronize()
    return ref, (out, lse)


def test_attend_static_matches_attend_two_calls_second_smaller():
    wl = inputs.CONFIGS[1].scaled(name="static_bf16", n_frames=160, n_scenes=10, n_clusters=12, top_k=4,
                                  question_tokens=12)
    st, m = _context(wl)
    tol = harness.OUT_TOL[wl.kv_dtype]
    # first call: a 12-token question (six row tiles per KV head, the multi-token kernel);
    # second call, right after it, on a smaller input: one decode token
    for i, tq in enumerate((12, 1)):
        q = st.question(st.draw_scene(), tq, i).to(DEV)[0].contiguous()
        m.retrieve(0, q)
        (o_ref, l_ref), (o, l) = _both(m, 0, q)
        assert torch.isfinite(o.float()).all() and torch.isfinite(l).all()
        assert (o.float() - o_ref.float()).abs().max().item() <= tol
        assert (l - l_ref).abs().max().item() <= harness.LSE_TOL[wl.kv_dtype]
        assert torch.equal(o, o_ref) and torch.equal(l, l_ref)     # same kernels, same splits
    m.close()


def test_attend_static_fp32_all_layers_and_against_the_oracle():
    wl = inputs.CONFIGS[0].scaled(name="static_fp32", n_layers=2)
    st, m = _context(wl)
    for i, tq in enumerate((wl.question_tokens, 1)):
        q = st.question(st.draw_scene(), tq, i).to(DEV)
        m.retrieve(-1, q)
        (o_ref, l_ref), (o, l) = _both(m, -1, q)
        assert torch.equal(o, o_ref) and torch.equal(l, l_ref)
    # and against the oracle's attention over the library's token list, one unit
    from oracle import mosaic_oracle as orc
    K, V = st.frames(0, wl.n_frames)
    ids, n_ids, scores, toks = m.selection(1)
    h, G = 1, wl.group
    Ku = inputs.unit_pages(K, 1, h).reshape(-1, wl.head_dim)
    Vu = inputs.unit_pages(V, 1, h).reshape(-1, wl.head_dim)
    want, want_lse = orc.attend(q[1].float().cpu().numpy().astype(np.float64), Ku, Vu, toks[h], h, G)
    got = o[1].float().cpu().numpy()[:, h * G:(h + 1) * G, :]
    assert np.abs(got - want).max() <= harness.OUT_TOL["fp32"]
    assert np.abs(l[1].cpu().numpy()[:, h * G:(h + 1) * G] - want_lse).max() <= harness.LSE_TOL["fp32"]
    m.close()


def test_attend_static_rejects_what_does_not_fit_and_takes_fewer_splits_when_short():
    # 24 layers x 4 KV heads x 112 row tiles = 10752 entries: beyond the 2001 the buffer holds at D = 128
    wl = inputs.CONFIGS[1].scaled(name="static_big", n_layers=24, n_frames=64, n_scenes=4, n_clusters=4,
                                  top_k=2, question_tokens=256)
    st, m = _context(wl)
    q = st.question(st.draw_scene(), 256, 0).to(DEV)
    m.retrieve(-1, q)
    out = torch.empty_like(q)
    lse = torch.empty(q.shape[:-1], dtype=torch.float32, device=DEV)
    with pytest.raises(binding.MosaicError) as ei:
        m.attend_static(-1, q, out, lse)
    assert ei.value.code == binding.ECAPACITY and "entries" in str(ei.value)
    # one layer of the same question fits (4 x 112 entries) with fewer splits than the arena allows:
    # results then differ only in the order the partials are merged
    m.retrieve(3, q[3].contiguous())
    (o_ref, l_ref), (o, l) = _both(m, 3, q[3].contiguous())
    assert (o.float() - o_ref.float()).abs().max().item() <= harness.OUT_TOL["bf16"]
    assert (l - l_ref).abs().max().item() <= 1e-4
    m.close()
