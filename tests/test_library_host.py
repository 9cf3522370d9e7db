"""Host-side checks that need no GPU: the built library loads, exports every
symbol the public header declares, validates configurations and sizes arenas."""
import ctypes as C
import os
import re

import pytest

from paper_2604_10060_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "mosaic.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mosaic_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    lib = binding.load_library()
    names = _declared_functions()
    assert "mosaic_ingest_frame" in names and "mosaic_retrieve" in names
    assert "mosaic_attend" in names and "mosaic_reset" in names
    for name in names:
        assert hasattr(lib, name), f"{name} declared in mosaic.h but not exported"
    assert sorted(binding.EXPORTS) == names


def test_struct_layout_matches_header():
    # 16 int32 fields; pointer, size_t, pointer; 2 int32, float, int32; pointer, size_t; 4 int32; 3 doubles;
    # 2 int32; 4 int32; 1 int32 and 4 bytes of tail padding
    assert C.sizeof(binding.Config) == 16 * 4 + 3 * 8 + 4 * 4 + 2 * 8 + 4 * 4 + 3 * 8 + 2 * 4 + 4 * 4 + 4 + 4
    assert C.sizeof(binding.Stats) == 5 * 8 + 4 * 4 + 5 * 8 + 3 * 8 + 5 * 8


def _cfg(**kw):
    base = dict(n_layers=1, n_q_heads=4, n_kv_heads=2, head_dim=64, tokens_per_frame=16,
                max_frames=128, n_clusters=16, top_k=4, kv_dtype="fp32")
    base.update(kw)
    return binding.make_config(**base)


def test_workspace_size_grows_with_the_stream():
    a = binding.workspace_size(_cfg())
    b = binding.workspace_size(_cfg(max_frames=256))
    assert b > a > 2 * 2 * 128 * 16 * 64 * 4          # at least the K and V pages
    # bf16 pages are half the bytes of fp32 pages
    kv32 = 2 * 2 * 4096 * 64 * 128 * 4
    d = binding.workspace_size(_cfg(head_dim=128, tokens_per_frame=64, max_frames=4096)) - \
        binding.workspace_size(_cfg(head_dim=128, tokens_per_frame=64, max_frames=4096, kv_dtype="bf16"))
    assert d == kv32 // 2


@pytest.mark.parametrize("bad", [
    dict(head_dim=96), dict(n_q_heads=5), dict(top_k=0), dict(top_k=17), dict(n_clusters=0),
    dict(n_clusters=2000, top_k=4), dict(kv_dtype=7), dict(tokens_per_frame=0),
    dict(warmup_frames=8), dict(score_mode=2), dict(attend_impl=binding.ATTEND_MFMA),
    dict(max_frames=1 << 30, tokens_per_frame=64), dict(attend_impl=9), dict(tier=2),
    dict(tier=1, recluster_every=16), dict(tier=1, cache_fraction=1.5),
    dict(ingest_overlap=2), dict(decode_fused_max_mib=-3),
])
def test_bad_configurations_are_rejected(bad):
    with pytest.raises(binding.MosaicError) as e:
        binding.workspace_size(_cfg(**bad))
    assert e.value.code == binding.EINVAL
    assert len(str(e.value)) > 10


def test_host_tier_sizes():
    hbm = binding.workspace_sizes(_cfg(kv_dtype="bf16", head_dim=128, tokens_per_frame=64, max_frames=4096))
    assert hbm[1] == 0
    cfg = _cfg(kv_dtype="bf16", head_dim=128, tokens_per_frame=64, max_frames=4096, tier=binding.TIER_HOST,
               slab_frames=8, cache_fraction=0.1)
    dev, host = binding.workspace_sizes(cfg)
    # host pool: (4096/8 + 16) slabs of 8 pages per unit, K and V pages of 16 KiB each, 2 units
    assert host >= 2 * (4096 // 8 + 16) * 8 * 2 * 64 * 128 * 2
    # the device side only holds the cache and the staging ring, not the whole stream
    assert dev < hbm[0]


def test_null_arguments_do_not_crash():
    lib = binding.load_library()
    assert lib.mosaic_workspace_size(None, None, None) == binding.EINVAL
    assert lib.mosaic_reset(None) == binding.EINVAL
    assert lib.mosaic_ingest_frame(None, None, None, 1) == binding.EINVAL
    assert lib.mosaic_retrieve(None, 0, None, 1) == binding.EINVAL
    assert lib.mosaic_attend(None, 0, None, 1, None, None) == binding.EINVAL
    assert lib.mosaic_destroy(None) == binding.EINVAL
    assert lib.mosaic_ingest_join(None) == binding.EINVAL
    assert lib.mosaic_decode_step(None, 0, None, 1, None, None) == binding.EINVAL
    assert isinstance(lib.mosaic_last_error(None), bytes)


def test_running_mean_division_scheme_is_correctly_rounded():
    """Eq. 3's division by n + 1 in the register-table assignment kernel: y = RN(1 / b) once, then per channel
    q = RN(x y) and two residual corrections q <- RN(q + RN(x - b q) y), each residual exact in a fused
    multiply-add.  Emulated here with exact rational arithmetic (one rounding per operation, as the hardware's
    FMA): the result must be the correctly rounded x / b, i.e. what the oracle's plain division returns, also
    for quotients that lie next to a rounding boundary."""
    import math
    import random
    from fractions import Fraction as Fr

    def fma(a, b, c):
        return float(Fr(a) * Fr(b) + Fr(c))

    rng = random.Random(7)
    for t in range(20000):
        b = float(rng.randint(1, 1 << rng.randint(1, 24)))
        x = math.ldexp(1.0 + rng.getrandbits(52) / 2.0 ** 52, rng.randint(-60, 60)) * rng.choice((-1, 1))
        if t % 2 == 0:      # x ~ b * (q +- half an ulp of q)
            q = math.ldexp(1.0 + rng.getrandbits(52) / 2.0 ** 52, rng.randint(-20, 20))
            x = float(Fr(q) * Fr(b) + Fr(math.ulp(q)) * Fr(b) * Fr(rng.choice((1, -1)), 2)
                      * Fr(rng.randint(999999, 1000001), 1000000))
        want = float(Fr(x) / Fr(b))
        y = float(Fr(1) / Fr(b))
        q = x * y
        q = fma(fma(-b, q, x), y, q)
        q = fma(fma(-b, q, x), y, q)
        assert q == want, (x, b, q, want)
