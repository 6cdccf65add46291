"""GPU parity for the banded K-cache layout (bands of 32 rows, head-major inside a band): the same
seeded problems as the row-major parity tests, the cache re-laid by slim_band_kcache.  The layout
changes addresses only, never arithmetic or its order, so besides the oracle's tolerance the result
must equal the row-major one bit for bit."""
import numpy as np
import pytest

from paper_2503_05840_amd import binding, synth
from gpu_harness import BlockCase, KCase, TOL, row_rel_err, say

pytestmark = pytest.mark.gpu
C = synth.CONFIGS

CASES = {
    "cfg1-like": synth.scaled(C[1], H=8, d=1024, T=1000),
    "cfg2-like-ragged": synth.scaled(C[2], B=3, H=8, d=768, T=700, len_lo=100),
    "cfg3-like": synth.scaled(C[3], B=5, T=333),
    "one-head": synth.scaled(C[1], H=1, d=128, T=65),
    "whisper-width-all-waves": synth.scaled(C[3], B=1, T=6144),
    "two-heads-per-unit-multi-tile": synth.scaled(C[3], B=3, H=32, d=2048, T=5000, len_lo=3000),
    "dk96-multi-tile": synth.scaled(C[2], B=2, T=9000, len_lo=4000),
    "dk32-four-heads-per-unit": synth.scaled(C[1], B=2, H=32, d=1024, d_k=32, T=900, len_lo=500),
    "batch-by-sequence": synth.scaled(C[1], B=40, H=16, d=2048, T=203),
    "batch-by-sequence-ragged": synth.scaled(C[1], B=130, H=32, d=4096, T=150, len_lo=1),
}
FUSED = {"auto": binding.VARIANT_AUTO, "fused": binding.VARIANT_FUSED, "fused_split": binding.VARIANT_FUSED_SPLIT}


def rows32(T):
    return (T + 31) // 32 * 32


@pytest.fixture(scope="module")
def cases():
    cache = {}

    def get(name, **kw):
        key = (name, tuple(sorted(kw.items())))
        if key not in cache:
            cache[key] = KCase(CASES[name], t_stride=rows32(CASES[name].T), need_v=False, **kw)
        return cache[key]
    return get


@pytest.mark.parametrize("name", list(CASES))
def test_banded_cache_matches_oracle_and_the_row_major_result(cases, name):
    k = cases(name)
    for vname, variant in FUSED.items():
        say(f"[case] slim_decode banded {name} variant={vname}")
        got = k.run_slim(banded=True, variant=variant)
        e = k.err(got)
        say(f"  rel err {e:.3e} (tol {TOL['bf16']})")
        assert e <= TOL["bf16"]
        assert np.array_equal(got, k.run_slim(variant=variant)), "banded and row-major results differ"


@pytest.mark.parametrize("factor", [50.0, 2000.0])
def test_banded_cache_peaky_softmax(cases, factor):
    for name in ("cfg1-like", "cfg2-like-ragged"):
        say(f"[case] banded peaky {name} x{factor}")
        k = cases(name).set_query_scale(factor)
        try:
            got = k.run_slim(banded=True)
            assert k.err(got) <= TOL["bf16"]
            assert np.array_equal(got, k.run_slim())
        finally:
            k.set_query_scale(1.0)


@pytest.mark.parametrize("name", ["cfg1-like", "dk96-multi-tile", "batch-by-sequence"])
def test_banded_cache_with_rotary_keys(cases, name):
    say(f"[case] banded + rope {name}")
    k = cases(name, rope_base=10000.0, q_scale=30.0)
    got = k.run_slim(banded=True)
    assert k.err(got) <= TOL["bf16"]
    assert np.array_equal(got, k.run_slim())


def test_banded_cache_one_row_and_partial_last_band():
    say("[case] banded T=1")
    k = KCase(synth.scaled(C[1], H=4, d=512, T=1), t_stride=32, need_v=False)
    assert k.err(k.run_slim(banded=True)) <= TOL["bf16"]
    say("[case] banded ragged with len 1, 32, 33 and T")
    cfg = synth.scaled(C[2], B=5, H=8, d=768, T=130, len_lo=0)
    k = KCase(cfg, lens=[1, 130, 32, 33, 64], t_stride=160, need_v=False)
    got = k.run_slim(banded=True)
    assert k.err(got) <= TOL["bf16"]
    assert np.array_equal(got, k.run_slim())


def test_banded_cache_refusals():
    say("[case] banded refusals")
    # rows per sequence not a multiple of 32
    k = KCase(synth.scaled(C[1], H=8, d=1024, T=100), need_v=False)
    with pytest.raises(binding.SlimError) as ei:
        binding.slim_decode(k.q, k.K, k.Wkv, k.q.clone(), 1, 8, 100, 1024, k_layout=binding.K_BANDED)
    assert ei.value.code == binding.SLIM_ERR_LAYOUT
    # the plain kernels read row-major caches only
    k = KCase(synth.scaled(C[1], H=8, d=1024, T=96), need_v=False)
    with pytest.raises(binding.SlimError) as ei:
        k.run_slim(banded=True, variant=binding.VARIANT_GENERIC)
    assert ei.value.code == binding.SLIM_ERR_LAYOUT
    # fp32 caches take the plain kernels
    k = KCase(synth.scaled(C[0], B=2, H=4, d=256, T=64), need_v=False)
    with pytest.raises(binding.SlimError) as ei:
        k.run_slim(banded=True)
    assert ei.value.code == binding.SLIM_ERR_LAYOUT


@pytest.mark.parametrize("rope_base", [None, 10000.0])
def test_attention_block_appends_into_a_banded_cache(rope_base):
    say(f"[case] slim_attention_block banded rope={rope_base}")
    cfg = synth.scaled(C[2], B=3, H=8, d=768, T=700, len_lo=100)
    k = BlockCase(cfg, rope_base=rope_base, t_stride=704)
    y_b, krow_b = k.run_slim(banded=True)
    y_r, krow_r = k.run_slim()
    assert row_rel_err(y_b, k.ref) <= TOL["bf16"]
    assert np.array_equal(y_b, y_r)
    assert np.array_equal(krow_b, krow_r)
