"""The seeded input recipe: determinism, the stated distributions, dtype rounding.  CPU only."""
import numpy as np
import torch

from paper_2503_05840_amd import synth


def test_same_seed_same_inputs():
    a = synth.make_problem(synth.CONFIGS[0])
    b = synth.make_problem(synth.CONFIGS[0])
    assert np.array_equal(a.w.W_K, b.w.W_K) and np.array_equal(a.seqs[0].X, b.seqs[0].X)
    assert np.array_equal(a.q, b.q)


def test_wk_singular_values_in_recipe_range():
    p = synth.make_problem(synth.CONFIGS[0])
    d = p.cfg.d
    sv = np.linalg.svd(p.w.W_K * np.sqrt(d), compute_uv=False)
    assert sv.min() >= 0.5 - 1e-9 and sv.max() <= 2.0 + 1e-9
    np.testing.assert_allclose(np.sort(sv), np.sort(p.w.s), rtol=1e-9)
    assert abs(p.w.W_V.std() * np.sqrt(d) - 1.0) < 0.02


def test_ragged_lengths_and_skipped_sequences_keep_later_draws():
    cfg = synth.scaled(synth.CONFIGS[2], B=4, H=4, d=64, d_k=16, T=96, len_lo=24)
    full = synth.make_problem(cfg)
    part = synth.make_problem(cfg, keep={3})
    assert all(24 <= s.length <= 96 for s in full.seqs)
    assert part.seqs[0].X is None and np.array_equal(part.seqs[3].X, full.seqs[3].X)
    assert np.array_equal(part.q, full.q)


def test_bf16_rounding_is_rne_and_matches_torch():
    rng = np.random.default_rng(0)
    a = np.concatenate([rng.standard_normal(4096) * 10.0 ** rng.integers(-6, 6, 4096),
                        [0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895313892515355e38]])
    bits = synth.f64_to_bf16_bits(a)
    ref = torch.from_numpy(a).to(torch.float32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bits, ref)
    back = synth.bf16_bits_to_f64(bits)
    assert np.all(np.abs(back[:4096] - a[:4096]) <= np.abs(a[:4096]) * 2.0 ** -8)
    # ties to even: 1 + 2^-8 is halfway between 1 and 1 + 2^-7 -> 1 ; 1 + 3*2^-8 -> 1 + 2^-6
    assert synth.round_through(np.array([1.00390625]), "bf16")[0] == 1.0
    assert synth.round_through(np.array([1.01171875]), "bf16")[0] == 1.015625
