"""GPU parity at the full sizes of the five configs, in the launch configuration bench.py
times (library-chosen variant, ragged lengths where the config has them).  Configs 2 and 4 have a
quick test on a sample of sequences (shortest, longest and two seeded picks; two sequences) and a
slower one that compares every sequence of the batch with the fp64 oracle."""
import numpy as np
import pytest

from paper_2503_05840_amd import binding, synth
from gpu_harness import KCase, XCase, TOL, head_rel_err, say

pytestmark = pytest.mark.gpu
C = synth.CONFIGS


def test_config1_codellama_16k_full():
    say("[case] config 1 full size (B=1 H=32 d=4096 T=16384 bf16)")
    k = KCase(C[1])
    assert binding.auto_variant_name(1, 32, 16384, 4096, "bf16") == "fused"
    a = k.run_slim()
    e = k.err(a)
    say(f"  slim rel err {e:.3e}")
    assert e <= TOL["bf16"]
    assert np.array_equal(a, k.run_slim())                       # bitwise repeatable
    assert np.array_equal(a, k.run_slim(banded=True))            # the banded cache: other addresses, same arithmetic
    ev = k.err(k.run_vanilla())
    say(f"  vanilla rel err {ev:.3e}")
    assert ev <= TOL["bf16"]
    eg = k.err(k.run_slim(variant=binding.VARIANT_GENERIC))
    say(f"  slim (generic kernels) rel err {eg:.3e}")
    assert eg <= TOL["bf16"]
    k.set_query_scale(50.0)                                      # peaky softmax at full length
    e50 = k.err(k.run_slim())
    say(f"  slim rel err with q x50: {e50:.3e}")
    assert e50 <= TOL["bf16"]


def test_config1_with_rotary_keys_full():
    """Positions up to 16383 (angles far past 2 pi at the first frequencies), one-launch mode."""
    say("[case] config 1 full size + rotary keys (raw keys cached, q x30)")
    k = KCase(C[1], rope_base=10000.0, q_scale=30.0, need_v=False)
    a = k.run_slim()
    e = k.err(a)
    say(f"  slim rel err {e:.3e}")
    assert e <= TOL["bf16"]
    assert np.array_equal(a, k.run_slim())
    eg = k.err(k.run_slim(variant=binding.VARIANT_GENERIC))
    say(f"  slim (generic kernels) rel err {eg:.3e}")
    assert eg <= TOL["bf16"]
    assert k.err(k.run_slim(rope_table=None)) > 5 * TOL["bf16"]


def test_config3_whisper_cross_attention_full():
    say("[case] config 3 full size (B=64 H=20 d=1280 T=1500 bf16)")
    k = KCase(C[3], t_stride=1504)                               # whole 32-row bands per sequence
    a = k.run_slim()
    e = k.err(a)
    say(f"  slim rel err {e:.3e} over all 64 sequences")
    assert e <= TOL["bf16"]
    assert np.array_equal(a, k.run_slim(banded=True))
    ev = k.err(k.run_vanilla())
    say(f"  vanilla rel err {ev:.3e}")
    assert ev <= TOL["bf16"]


def test_config2_phi3_ragged_batch_sampled():
    cfg = C[2]
    lens = synth.make_problem(synth.scaled(cfg, T=cfg.T), keep=set()).lengths
    rng = np.random.default_rng(7)
    picks = {int(np.argmin(lens)), int(np.argmax(lens))}
    while len(picks) < 4:
        picks.add(int(rng.integers(0, cfg.B)))
    say(f"[case] config 2 full size (B=16 H=32 d=3072 ragged {lens.min()}..{lens.max()}); oracle on sequences {sorted(picks)}")
    k = KCase(cfg, oracle_seqs=picks)
    a = k.run_slim()
    e = k.err(a)
    say(f"  slim rel err {e:.3e} on the sampled sequences")
    assert e <= TOL["bf16"]
    v = k.run_vanilla()
    assert np.isfinite(a).all() and np.isfinite(v).all()
    cross = head_rel_err(a, v.astype(np.float64), cfg.H)          # all 16 sequences, kernel vs kernel
    say(f"  slim vs vanilla over the whole batch: {cross:.3e}")
    assert cross <= 2 * TOL["bf16"]


def test_config2_phi3_ragged_batch_every_sequence():
    """All 16 sequences of config 2 against the fp64 oracle (the oracle's K and V for the whole batch:
    about 17 GB of host memory, a few minutes of fp64 products)."""
    cfg = C[2]
    say("[case] config 2 full size, oracle on all 16 sequences")
    k = KCase(cfg)
    assert len(k.oracle_rows) == cfg.B
    a = k.run_slim()
    e = k.err(a)
    say(f"  slim rel err {e:.3e} over all {cfg.B} sequences")
    assert e <= TOL["bf16"]
    ab = k.run_slim(banded=True)
    eb = k.err(ab)
    say(f"  slim on the banded cache: rel err {eb:.3e}")
    assert eb <= TOL["bf16"] and np.array_equal(a, ab)
    ev = k.err(k.run_vanilla())
    say(f"  vanilla rel err {ev:.3e} over all {cfg.B} sequences")
    assert ev <= TOL["bf16"]


def test_config4_t5_xcache_every_sequence():
    cfg = C[4]
    say("[case] config 4 full size, oracle on all 8 sequences")
    x = XCase(cfg)
    assert len(x.oracle_rows) == cfg.B
    out = x.run()
    e = x.err(out)
    say(f"  xcache rel err {e:.3e} over all {cfg.B} sequences")
    assert e <= TOL["bf16"]
    g = x.run(variant=binding.VARIANT_GENERIC)
    eg = x.err(g)
    say(f"  plain kernels rel err {eg:.3e}")
    assert eg <= TOL["bf16"]
    e2 = x.err(x.run(variant=binding.VARIANT_FUSED_SPLIT))
    say(f"  two passes over X rel err {e2:.3e}")
    assert e2 <= TOL["bf16"]
    assert np.array_equal(out, x.run())                          # repeatable


def test_config4_t5_xcache_sampled():
    cfg = C[4]
    say("[case] config 4 full size (B=8 H=128 d_model=1024 d_k=128 T=4096); oracle on sequences 0 and 5")
    x = XCase(cfg, oracle_seqs={0, 5})
    out = x.run()
    e = x.err(out)
    say(f"  xcache rel err {e:.3e}")
    assert e <= TOL["bf16"]


def test_config1_whole_attention_block_full():
    """The steps either side of the decode step at config 1's size: q and k projections, append as row
    16383, decode over 16384 rows, W_O; slim and vanilla, with rotary keys."""
    from gpu_harness import BlockCase, row_rel_err
    say("[case] config 1 full size, whole attention block + rotary keys (W_Q x10)")
    k = BlockCase(C[1], rope_base=10000.0, q_gain=10.0)
    y, krow = k.run_slim()
    e, ek = row_rel_err(y, k.ref), row_rel_err(krow, k.k_new)
    say(f"  slim block rel err {e:.3e}, appended key row {ek:.3e}")
    assert e <= TOL["bf16"] and ek <= TOL["bf16"]
    y, krow, vrow = k.run_vanilla()
    e = row_rel_err(y, k.ref)
    say(f"  vanilla block rel err {e:.3e}")
    assert e <= TOL["bf16"]
    assert row_rel_err(krow, k.k_new_rot) <= TOL["bf16"] and row_rel_err(vrow, k.v_new) <= TOL["bf16"]


def test_config3_as_encoder_cache_sampled():
    """Option 2 of the encoder-decoder section at config 3's size: the cross-attention layer reads the
    encoder output E (B x 1500 x 1280) through slim_decode_xcache; no cross K or V cache exists."""
    cfg = synth.scaled(C[3], kind="xcache")
    say("[case] config 3 as E-cache (B=64 H=20 d=1280 T=1500); oracle on sequences 0, 21 and 63")
    x = XCase(cfg, oracle_seqs={0, 21, 63})
    out = x.run()
    e = x.err(out)
    say(f"  E-cache rel err {e:.3e}")
    assert e <= TOL["bf16"]
    g = x.run(variant=binding.VARIANT_GENERIC)
    cross = head_rel_err(out, g.astype(np.float64), cfg.H)          # all 64 sequences, kernel vs kernel
    say(f"  MFMA path vs plain kernels over the whole batch: {cross:.3e}")
    assert cross <= TOL["bf16"]
