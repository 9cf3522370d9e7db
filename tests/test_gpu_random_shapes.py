"""Seeded random shapes through the C ABI against the oracle (GPU): a sweep over head sizes, group sizes,
page lengths (ragged and whole chunks), table sizes, question lengths (decode, short and multi-row-block
questions), call modes and dtypes, beyond the hand-picked cases of test_gpu_parity.py; and the same for the
host tier with the self-adaptive maintainer (the oracle's residency comes from the working-set model)."""
import random

import pytest

from oracle import cache_model
from paper_2604_10060_amd import binding, inputs
from tests import harness

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("seed", [101, 202, 303])
def test_random_shapes_against_the_oracle(seed):
    rng = random.Random(seed)
    for it in range(8):
        D = rng.choice([64, 128])
        Hkv = rng.choice([1, 2, 4])
        G = rng.choice([1, 2, 4, 7, 8])
        T = rng.choice([1, 5, 16, 32, 33, 50, 64, 100])
        C = rng.choice([1, 2, 5, 12, 16, 33, 64, 100, 130, 200, 256, 300])
        k = rng.randint(1, min(C, 40))
        F = max(2 * C + rng.randint(1, 60), 20)
        dtype = rng.choice(["bf16", "bf16", "fp32"])
        L = rng.choice([1, 1, 2])
        tq = rng.choice([1, 2, 3, 9, 17, 40, 70])
        mode = rng.choice(["per_layer", "all", "fused"])
        rec = rng.choice([0, 0, 64]) if C <= 64 else 0
        wl = inputs.CONFIGS[1].scaled(name=f"rnd{seed}_{it}", n_layers=L, n_q_heads=Hkv * G, n_kv_heads=Hkv, head_dim=D,
                                      tokens_per_frame=T, n_frames=F, n_clusters=C, top_k=k, kv_dtype=dtype,
                                      n_scenes=max(2, min(F // 4, 25)), question_tokens=tq, recluster_every=rec,
                                      seed=5000 + seed + it)
        print(f"  {it}: D{D} Hkv{Hkv} G{G} T{T} C{C} k{k} F{F} {dtype} L{L} tq{tq} {mode} rec{rec}", flush=True)
        units = [(l, h) for l in range(L) for h in range(Hkv)][:3]
        harness.run_workload(wl, units=units, n_questions=1, decode_steps=2, layer_mode=mode)


@pytest.mark.parametrize("seed", [11, 22])
def test_random_host_tier_with_the_maintainer_against_the_oracle(seed):
    rng = random.Random(seed)
    ran = 0
    for it in range(6):
        D = rng.choice([64, 128]); Hkv = rng.choice([1, 2]); G = rng.choice([1, 4, 7])
        T = rng.choice([3, 16, 33, 50, 64]); dtype = rng.choice(["bf16", "fp32"])
        Ct = rng.choice([8, 24, 40]); ci = rng.randint(1, max(1, Ct // 3)); F = rng.randint(80, 260)
        mode = rng.choice([1, 2])
        mt = dict(mode=mode, c_init=ci, tau_min=rng.choice([1.0, 2.0, 4.0]), tau_max=rng.choice([6.0, 16.0]),
                  n0=rng.choice([4.0, 16.0]), split_iters=rng.choice([1, 4]),
                  buf_max=rng.choice([3, 12]) if mode == 2 else 0)
        wl = inputs.CONFIGS[1].scaled(name=f"rndh{seed}_{it}", n_layers=rng.choice([1, 2]), n_q_heads=Hkv * G, n_kv_heads=Hkv,
                                      head_dim=D, tokens_per_frame=T, kv_dtype=dtype, question_tokens=rng.choice([1, 3, 9]),
                                      seed=9000 + seed + it, n_frames=F, n_clusters=Ct, top_k=rng.randint(1, min(Ct, 5)),
                                      n_scenes=rng.randint(3, 12))
        host = dict(slab_frames=rng.choice([2, 4, 8]), cache_pages_per_unit=F, cache_fraction=rng.choice([0.5, 1.0]))
        pattern = rng.choice([(1, 3, 8, 2, 16), (64,), (70, 1, 5), (16,)])
        print(f"  {it}: mode{mode} {mt} D{D} Hkv{Hkv} G{G} T{T} C{Ct} F{F} {dtype} L{wl.n_layers} {host} {pattern}", flush=True)
        try:
            harness.run_maintained(wl, mt, query_every=rng.choice([12, 20, 40]), host=host, batch_pattern=pattern)
            ran += 1
        except binding.MosaicError as ex:          # a selection larger than the cluster count the cache may hold
            if ex.code != binding.ECAPACITY:
                raise
        except cache_model.CapacityError:
            pass
    assert ran >= 3
