"""GPU parity of the whole attention block of one generated token (projections, append to the
cache, decode step, W_O), called through the C ABI, against the fp64 oracle's attention_block.
Bars as for the decode step, norm-wise per output row: 1e-4 (fp32), 2e-2 (bf16); the rows the call
writes into the caches are compared with the oracle's new key / value rows to the same bars."""
import numpy as np
import pytest

from paper_2503_05840_amd import binding, synth
from gpu_harness import BlockCase, TOL, row_rel_err, say

pytestmark = pytest.mark.gpu
C = synth.CONFIGS

CASES = {
    "cfg0-exact": (C[0], {}),
    "cfg1-like": (synth.scaled(C[1], H=8, d=1024, T=1000), {}),
    "cfg1-like-peaky": (synth.scaled(C[1], H=8, d=1024, T=1000), dict(q_gain=30.0)),
    "cfg2-like-ragged": (synth.scaled(C[2], B=3, H=8, d=768, T=700, len_lo=100), dict(q_gain=10.0)),
    "cfg3-like-batch": (synth.scaled(C[3], B=40, T=333), {}),
    "f32-ragged-first-token": (synth.scaled(C[0], B=3, H=4, d=256, T=300, len_lo=1), dict(q_gain=10.0)),
    "padded-stride": (synth.scaled(C[2], B=2, H=8, d=768, T=200, len_lo=50), dict(t_stride=256)),
}
VARIANTS = {"auto": binding.VARIANT_AUTO, "generic": binding.VARIANT_GENERIC}


@pytest.mark.parametrize("rope", [None, 10000.0])
@pytest.mark.parametrize("name", list(CASES))
def test_attention_block_matches_oracle(name, rope):
    cfg, kw = CASES[name]
    say(f"[case] attention block {name} rope={rope}")
    k = BlockCase(cfg, rope_base=rope, **kw)
    tol = TOL[cfg.dtype]
    for vname, variant in VARIANTS.items():
        y, krow = k.run_slim(variant=variant)
        e, ek = row_rel_err(y, k.ref), row_rel_err(krow, k.k_new)
        say(f"  slim {vname}: y {e:.3e}, appended key row {ek:.3e} (tol {tol})")
        assert e <= tol and ek <= tol
    y2, _ = k.run_slim()
    assert np.array_equal(y2, k.run_slim()[0])
    y, krow, vrow = k.run_vanilla()
    e = row_rel_err(y, k.ref)
    ek = row_rel_err(krow, k.k_new_rot if rope else k.k_new)
    ev = row_rel_err(vrow, k.v_new)
    say(f"  vanilla: y {e:.3e}, appended key row {ek:.3e}, value row {ev:.3e}")
    assert e <= tol and ek <= tol and ev <= tol


def test_first_token_of_a_sequence_is_two_products():
    """Length 1 after the append: the block returns x W_V W_O through W_KV (slim) whatever the scores."""
    say("[case] attention block, empty caches")
    cfg = synth.scaled(C[1], B=2, H=4, d=512, T=1)
    k = BlockCase(cfg, rope_base=10000.0)
    y, _ = k.run_slim()
    assert row_rel_err(y, k.ref) <= TOL["bf16"]
    y, _, _ = k.run_vanilla()
    assert row_rel_err(y, k.ref) <= TOL["bf16"]


def test_block_workspace_is_checked():
    import torch
    cfg = synth.scaled(C[1], H=8, d=1024, T=100)
    k = BlockCase(cfg)
    need = binding.slim_workspace_bytes_block(cfg.B, cfg.H, cfg.T, cfg.d, cfg.dtype)
    assert need > binding.slim_workspace_bytes(cfg.B, cfg.H, cfg.T, cfg.d, cfg.dtype)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    y, _ = k.run_slim(workspace=ws)
    assert row_rel_err(y, k.ref) <= TOL["bf16"]
    with pytest.raises(binding.SlimError) as ei:
        k.run_slim(workspace=torch.empty(need - 4096, dtype=torch.uint8, device="cuda"))
    assert ei.value.code == -5
