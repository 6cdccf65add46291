"""GPU parity: the HIP path, called through the C ABI, against the fp64 CPU oracle on the
same seeded inputs.  Bars: max norm-wise relative error per head vector <= 1e-4 for fp32
caches and <= 2e-2 for bf16 caches (fp32 accumulation)."""
import numpy as np
import pytest

from paper_2503_05840_amd import binding, synth
from gpu_harness import KCase, NonSquareCase, XCase, TOL, say

pytestmark = pytest.mark.gpu
C = synth.CONFIGS

SMALL = {
    # several tiles, a ragged tail, every d_k the configs use
    "cfg0-exact": C[0],
    "cfg1-like": synth.scaled(C[1], H=8, d=1024, T=1000),
    "cfg2-like-ragged": synth.scaled(C[2], B=3, H=8, d=768, T=700, len_lo=100),
    "cfg3-like": synth.scaled(C[3], B=5, T=333),
    "f32-ragged": synth.scaled(C[0], B=2, H=4, d=256, T=300, len_lo=40),
    "f32-dk128": synth.scaled(C[0], B=1, H=2, d=256, d_k=128, T=77),
    "one-head": synth.scaled(C[1], H=1, d=128, T=65),
    # every wave of the stream kernel's workgroups busy, two heads per column unit, several tiles
    # per wave and several sequences per group
    "whisper-width-all-waves": synth.scaled(C[3], B=1, T=6144),
    "two-heads-per-unit-multi-tile": synth.scaled(C[3], B=3, H=32, d=2048, T=5000, len_lo=3000),
    "dk96-multi-tile": synth.scaled(C[2], B=2, T=9000, len_lo=4000),
    # batches that fill the wave-pair slots: whole sequences per pair (uniform lengths with a partial
    # last tile; ragged with many sequences per slot, 1-row sequences included)
    "batch-by-sequence": synth.scaled(C[1], B=40, H=16, d=2048, T=203),
    "batch-by-sequence-ragged": synth.scaled(C[1], B=130, H=32, d=4096, T=150, len_lo=1),
}
VARIANTS = {"auto": binding.VARIANT_AUTO, "generic": binding.VARIANT_GENERIC, "fused": binding.VARIANT_FUSED,
            "fused_split": binding.VARIANT_FUSED_SPLIT}


@pytest.fixture(scope="module")
def cases():
    cache = {}

    def get(name, **kw):
        key = (name, tuple(sorted(kw.items())))
        if key not in cache:
            cache[key] = KCase(SMALL[name], **kw)
        return cache[key]
    return get


@pytest.mark.parametrize("variant", list(VARIANTS))
@pytest.mark.parametrize("name", list(SMALL))
def test_slim_decode_matches_oracle(cases, name, variant):
    say(f"[case] slim_decode {name} variant={variant}")
    k = cases(name)
    e = k.err(k.run_slim(variant=VARIANTS[variant]))
    say(f"  rel err {e:.3e} (tol {TOL[k.cfg.dtype]})")
    assert e <= TOL[k.cfg.dtype]


@pytest.mark.parametrize("name", list(SMALL))
def test_vanilla_kv_decode_matches_oracle(cases, name):
    say(f"[case] vanilla_kv_decode {name}")
    k = cases(name)
    e = k.err(k.run_vanilla())
    say(f"  rel err {e:.3e}")
    assert e <= TOL[k.cfg.dtype]


@pytest.mark.parametrize("factor", [50.0, 2000.0])
@pytest.mark.parametrize("name", ["cfg1-like", "cfg2-like-ragged", "f32-ragged"])
def test_peaky_softmax(cases, name, factor):
    """Scaled queries: running max, rescale and near one-hot weights."""
    say(f"[case] peaky {name} x{factor}")
    k = cases(name).set_query_scale(factor)
    for variant in VARIANTS.values():
        e = k.err(k.run_slim(variant=variant))
        say(f"  slim variant {variant}: {e:.3e}")
        assert e <= TOL[k.cfg.dtype]
    e = k.err(k.run_vanilla())
    k.set_query_scale(1.0)
    assert e <= TOL[k.cfg.dtype]


ROPE_CASES = ["cfg0-exact", "cfg1-like", "cfg2-like-ragged", "cfg3-like", "f32-dk128", "dk96-multi-tile",
              "two-heads-per-unit-multi-tile", "batch-by-sequence-ragged"]


@pytest.mark.parametrize("name", ROPE_CASES)
def test_slim_decode_with_rotary_keys_matches_oracle(cases, name):
    """RoPE appendix, option 1: raw keys in the cache, rotated by position after the read for the
    scores only.  Queries are scaled up so that the weights depend visibly on the rotation."""
    say(f"[case] slim_decode + rope {name}")
    k = cases(name, rope_base=10000.0, q_scale=30.0)
    tol = TOL[k.cfg.dtype]
    for vname, variant in VARIANTS.items():
        e = k.err(k.run_slim(variant=variant))
        say(f"  variant {vname}: rel err {e:.3e} (tol {tol})")
        assert e <= tol
    e = k.err(k.run_vanilla())                      # rotated keys stored, no table
    say(f"  vanilla on rotated keys: {e:.3e}")
    assert e <= tol
    # the check has teeth: the same call without the table is far from this reference
    e0 = k.err(k.run_slim(rope_table=None))
    say(f"  without the table: {e0:.3e}")
    assert e0 > 5 * tol


def test_rotary_keys_other_base_near_uniform_weights_and_one_row():
    say("[case] rope base 500, q x1")
    k = KCase(synth.scaled(C[1], H=8, d=1024, T=1000), rope_base=500.0)
    for variant in VARIANTS.values():
        assert k.err(k.run_slim(variant=variant)) <= TOL["bf16"]
    say("[case] rope T=1")
    k = KCase(synth.scaled(C[1], H=4, d=512, T=1), rope_base=10000.0)
    for variant in VARIANTS.values():
        assert k.err(k.run_slim(variant=variant)) <= TOL["bf16"]


def test_single_row_context_and_length_one_sequences():
    say("[case] T=1")
    k = KCase(synth.scaled(C[1], H=4, d=512, T=1))
    assert k.err(k.run_slim()) <= TOL["bf16"]
    assert k.err(k.run_vanilla()) <= TOL["bf16"]
    say("[case] ragged with len 1 and len T")
    cfg = synth.scaled(C[2], B=4, H=8, d=768, T=130, len_lo=0)
    k = KCase(cfg, lens=[1, 130, 9, 64])
    assert k.err(k.run_slim()) <= TOL["bf16"]
    assert k.err(k.run_vanilla()) <= TOL["bf16"]


def test_padded_cache_stride_and_caller_workspace():
    import torch
    cfg = synth.scaled(C[2], B=3, H=8, d=768, T=200, len_lo=50)
    say("[case] t_stride > T, caller workspace")
    k = KCase(cfg, t_stride=256)
    need = binding.slim_workspace_bytes(cfg.B, cfg.H, cfg.T, cfg.d, cfg.dtype)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    a = k.run_slim(workspace=ws)
    assert k.err(a) <= TOL["bf16"]
    b = k.run_slim()
    assert np.array_equal(a, b)
    small = torch.empty(need // 2, dtype=torch.uint8, device="cuda")
    with pytest.raises(binding.SlimError) as ei:
        k.run_slim(workspace=small)
    assert ei.value.code == -5


def test_repeat_calls_are_bitwise_identical(cases):
    k = cases("cfg2-like-ragged")
    say("[case] determinism")
    a, b = k.run_slim(), k.run_slim()
    assert np.array_equal(a, b)
    a, b = k.run_vanilla(), k.run_vanilla()
    assert np.array_equal(a, b)


def test_slim_and_vanilla_agree_with_each_other(cases):
    """Not a parity claim (both are ours): a cross-check that the two kernels see the same data."""
    k = cases("cfg3-like")
    a, b = k.run_slim(), k.run_vanilla()
    from gpu_harness import head_rel_err
    assert head_rel_err(a, b.astype(np.float64), k.cfg.H) <= 2 * TOL["bf16"]


@pytest.mark.parametrize("name,cfg", [
    ("xcache-bf16", synth.scaled(C[4], B=2, H=16, d=128, d_k=32, T=300)),
    ("xcache-f32", synth.scaled(C[4], B=1, H=6, d=64, d_k=32, T=70, dtype="f32", x_pre_rounded=False)),
    ("xcache-wide-heads", synth.scaled(C[4], B=1, H=40, d=256, d_k=128, T=129)),
])
def test_xcache_decode_matches_oracle(name, cfg):
    say(f"[case] slim_decode_xcache {name}")
    x = XCase(cfg)
    for vname in ("auto", "generic"):
        e = x.err(x.run(variant=VARIANTS[vname]))
        say(f"  {vname}: rel err {e:.3e}")
        assert e <= TOL[cfg.dtype]


@pytest.mark.parametrize("name,cfg,q_scale,lens", [
    # d_model = 1024 as in the T5-11B shape: all eight column waves, several context splits, a ragged tail
    ("xcache-t5-width", synth.scaled(C[4], B=2, H=32, d=1024, d_k=64, T=1100), 1.0, None),
    ("xcache-peaky", synth.scaled(C[4], B=2, H=32, d=1024, d_k=64, T=1100), 8.0, None),
    ("xcache-ragged-padded-heads", synth.scaled(C[4], B=3, H=24, d=512, d_k=32, T=900), 4.0, [900, 1, 333]),
    ("xcache-two-column-blocks", synth.scaled(C[4], B=1, H=8, d=1280, d_k=32, T=200), 1.0, None),
    # the one-pass kernel's corners: one row, one row more than a tile, fewer column owners than waves, five heads
    ("xcache-onepass-one-row", synth.scaled(C[4], B=2, H=5, d=512, d_k=32, T=1), 2.0, None),
    ("xcache-onepass-tile-plus-one", synth.scaled(C[4], B=3, H=5, d=640, d_k=32, T=33), 2.0, [33, 1, 32]),
    ("xcache-onepass-many-splits", synth.scaled(C[4], B=1, H=40, d=768, d_k=32, T=2500), 1.0, None),
    # rows wider than 1024 columns: the one-pass kernel's ten-wave shape (16 heads per group) -- nine column
    # owners (one wave without columns), one row, one row more than a tile, 40 heads over many splits, peaky scores
    ("xcache-onepass-wide-nine-owners", synth.scaled(C[4], B=2, H=9, d=1152, d_k=32, T=300), 2.0, [300, 31]),
    ("xcache-onepass-wide-one-row", synth.scaled(C[4], B=2, H=20, d=1280, d_k=64, T=1), 2.0, None),
    ("xcache-onepass-wide-tile-plus-one", synth.scaled(C[4], B=3, H=17, d=1280, d_k=32, T=33), 2.0, [33, 1, 32]),
    ("xcache-onepass-wide-many-splits", synth.scaled(C[4], B=1, H=40, d=1280, d_k=32, T=2500), 1.0, None),
    ("xcache-onepass-wide-peaky", synth.scaled(C[4], B=2, H=20, d=1280, d_k=64, T=900), 8.0, None),
    # 33 (sequence, split) units: dealt to the 8 XCDs with seven empty places at the end of the launch
    ("xcache-units-not-a-multiple-of-8", synth.scaled(C[4], B=33, H=8, d=512, d_k=32, T=70), 2.0, None),
    ("xcache-wide-units-not-a-multiple-of-8", synth.scaled(C[4], B=35, H=20, d=1280, d_k=32, T=40), 2.0, None),
    # the encoder-decoder section's option 2: the cross-attention K and V of a Whisper-large-shaped layer
    # (square projections, 20 heads: 16 heads per score workgroup, a padded head tile) from the encoder output
    ("ecache-whisper-shape", synth.scaled(C[3], kind="xcache", B=3, T=333), 4.0, None),
    ("ecache-whisper-shape-ragged", synth.scaled(C[3], kind="xcache", B=4, T=700), 2.0, [700, 2, 257, 512]),
])
def test_xcache_mfma_path_matches_oracle(name, cfg, q_scale, lens):
    say(f"[case] slim_decode_xcache {name} (q x{q_scale}, lens {lens})")
    x = XCase(cfg, q_scale=q_scale, lens=lens)
    a = x.run()
    e = x.err(a)
    say(f"  auto: rel err {e:.3e}")
    e2 = x.err(x.run(variant=VARIANTS["generic"]))
    say(f"  generic: rel err {e2:.3e}")
    assert e <= TOL[cfg.dtype]
    assert e2 <= TOL[cfg.dtype]
    assert np.array_equal(a, x.run()), "two runs of the same launch configuration differ"
    # the two-pass kernels (scores written out, then the weighted sum): what shapes outside the one-pass kernel's
    # range take by themselves, asked for explicitly here
    e3 = x.err(x.run(variant=VARIANTS["fused_split"]))
    say(f"  two passes over X: rel err {e3:.3e}")
    assert e3 <= TOL[cfg.dtype]


def test_xcache_mfma_path_on_very_peaky_scores():
    """Queries x40 make the softmax nearly one-hot.  At that scale the bf16 rounding of W_K alone moves
    the result by more than the tolerance (3.7e-2 in both implementations), so the oracle is given the
    weights as stored (rounded to bf16): what is then compared is the streaming maximum / rescaling of
    the MFMA path.  The plain fp32 vector-ALU kernels, which share its inputs bit for bit, ride along as
    a cross-check."""
    from gpu_harness import head_rel_err
    cfg = synth.scaled(C[4], B=2, H=32, d=1024, d_k=64, T=1100)
    say("[case] slim_decode_xcache very peaky (oracle on the stored weights), MFMA path and plain kernels")
    x = XCase(cfg, q_scale=40.0, oracle_sees_rounded_weights=True)
    a, g = x.run(), x.run(variant=VARIANTS["generic"])
    ea, eg = x.err(a), x.err(g)
    e2p = x.err(x.run(variant=VARIANTS["fused_split"]))
    say(f"  MFMA path vs oracle {ea:.3e} (one pass), {e2p:.3e} (two passes), plain kernels vs oracle {eg:.3e}")
    assert ea <= TOL[cfg.dtype] and eg <= TOL[cfg.dtype] and e2p <= TOL[cfg.dtype]
    e = head_rel_err(a, g.astype(np.float64), cfg.H)
    say(f"  MFMA path vs plain kernels {e:.3e}")
    assert e <= 1e-2          # bf16 weights and bf16 q~ operands vs fp32 arithmetic on the same inputs


@pytest.mark.parametrize("name,cfg,q_scale", [
    ("t5-like-r4", synth.scaled(C[4], B=2, H=8, d=256, d_k=128, T=700), 2.0),
    ("r2-many-heads", synth.scaled(C[4], B=3, H=32, d=1024, d_k=64, T=300), 1.0),
    ("r4-f32", synth.scaled(C[4], B=1, H=8, d=64, d_k=32, T=130, dtype="f32", x_pre_rounded=False), 4.0),
])
def test_nonsquare_option1_right_inverse_decode_matches_oracle(name, cfg, q_scale):
    """Non-square section, option 1: e-wide K-cache, W_KV (e x e) from the right inverse of the d x e W_K."""
    say(f"[case] non-square option 1 {name} (d={cfg.d}, e={cfg.e}, q x{q_scale})")
    k = NonSquareCase(cfg, q_scale=q_scale)
    for vname, variant in VARIANTS.items():
        e = k.err(k.run_slim(variant=variant))
        say(f"  slim {vname}: rel err {e:.3e} (rcond of W_K W_K^T {k.rcond:.2e})")
        assert e <= TOL[cfg.dtype]
    ev = k.err(k.run_vanilla())
    say(f"  vanilla e-wide K+V: {ev:.3e}")
    assert ev <= TOL[cfg.dtype]


@pytest.mark.parametrize("fill", [0, 1, 2, 0x7FC00000, -1])
def test_workspace_needs_no_initialisation(cases, fill):
    """The caller's scratch may hold anything -- small integers (which could pass for counters, flags or
    launch ids), NaN patterns, all ones: results are bitwise those of a zeroed scratch."""
    import torch
    from gpu_harness import BlockCase, XCase
    say(f"[case] workspace pre-filled with int32 {fill}")

    def scratch(nbytes, value):
        return torch.full(((nbytes + 3) // 4,), value, dtype=torch.int32, device="cuda").view(torch.uint8)

    for name in ("cfg1-like", "cfg2-like-ragged", "batch-by-sequence"):
        k = cases(name)
        c = k.cfg
        need = binding.slim_workspace_bytes(c.B, c.H, c.T, c.d, c.dtype)
        for variant in VARIANTS.values():
            ref = k.run_slim(variant=variant, workspace=scratch(need, 0))
            got = k.run_slim(variant=variant, workspace=scratch(need, fill))
            assert np.array_equal(ref, got), (name, variant)
        assert np.array_equal(k.run_vanilla(workspace=scratch(need, 0)), k.run_vanilla(workspace=scratch(need, fill)))
    cfg = synth.scaled(C[4], B=2, H=32, d=256, d_k=64, T=300)
    x = XCase(cfg, oracle_seqs=set())
    need = binding.slim_workspace_bytes_xcache(cfg.B, cfg.H, cfg.T, cfg.d, cfg.d_k, cfg.dtype)
    assert np.array_equal(x.run(workspace=scratch(need, 0)), x.run(workspace=scratch(need, fill)))
    cfg = synth.scaled(C[1], B=3, H=8, d=1024, T=200, len_lo=20)
    b = BlockCase(cfg)
    need = binding.slim_workspace_bytes_block(cfg.B, cfg.H, cfg.T, cfg.d, cfg.dtype)
    assert np.array_equal(b.run_slim(workspace=scratch(need, 0))[0], b.run_slim(workspace=scratch(need, fill))[0])
    assert np.array_equal(b.run_vanilla(workspace=scratch(need, 0))[0], b.run_vanilla(workspace=scratch(need, fill))[0])


def test_calls_on_two_streams_with_their_own_scratch(cases):
    """Launches of the fast path need the whole chip; issued from two streams they are ordered by the
    library and both give the single-stream result."""
    import torch
    say("[case] two streams, interleaved calls")
    k1, k2 = cases("cfg1-like"), cases("cfg2-like-ragged")
    ref1, ref2 = k1.run_slim(), k2.run_slim()
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    ws = [torch.empty(binding.slim_workspace_bytes(k.cfg.B, k.cfg.H, k.cfg.T, k.cfg.d, k.cfg.dtype), dtype=torch.uint8,
                      device="cuda") for k in (k1, k2)]
    outs1 = [torch.full((k1.cfg.B, k1.cfg.d), float("nan"), device="cuda") for _ in range(6)]
    outs2 = [torch.full((k2.cfg.B, k2.cfg.d), float("nan"), device="cuda") for _ in range(6)]
    torch.cuda.synchronize()
    for i in range(6):
        with torch.cuda.stream(s1):
            binding.slim_decode(k1.q, k1.K, k1.Wkv, outs1[i], k1.cfg.B, k1.cfg.H, k1.cfg.T, k1.cfg.d,
                                **k1._kw(workspace=ws[0]))
        with torch.cuda.stream(s2):
            binding.slim_decode(k2.q, k2.K, k2.Wkv, outs2[i], k2.cfg.B, k2.cfg.H, k2.cfg.T, k2.cfg.d,
                                **k2._kw(workspace=ws[1]))
    torch.cuda.synchronize()
    for o in outs1:
        assert np.array_equal(o.cpu().numpy(), ref1)
    for o in outs2:
        assert np.array_equal(o.cpu().numpy(), ref2)
