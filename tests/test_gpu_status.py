"""The failure path of the bounded waits between workgroups, driven from the host: with a wait budget of
zero every wait that is not satisfied at its first check gives up, every kernel still runs to its end,
the call's outputs are NaN and slim_status reports the time-out; the next ordinary call on the same
workspace is clean again."""
import numpy as np
import pytest

from paper_2503_05840_amd import binding, synth
from gpu_harness import KCase, TOL, say

pytestmark = pytest.mark.gpu


def test_wait_budget_zero_gives_nan_outputs_and_timeout_status():
    import torch
    # config-1-shaped, long enough that every wave walks several tiles: some word of some tile is not there
    # at a first look, so with no budget at least one wait gives up
    cfg = synth.scaled(synth.CONFIGS[1], T=8192)
    k = KCase(cfg, need_v=False)
    assert binding.auto_variant_name(cfg.B, cfg.H, cfg.T, cfg.d, "bf16") == "fused"
    ws = torch.empty(binding.slim_workspace_bytes(cfg.B, cfg.H, cfg.T, cfg.d, "bf16"), dtype=torch.uint8, device="cuda")
    binding.slim_init()
    say("[case] wait budget: ordinary call")
    good = k.run_slim(workspace=ws)
    assert binding.slim_status(ws) == binding.SLIM_OK
    assert k.err(good) <= TOL["bf16"]
    say("[case] wait budget: no waiting at all (every kernel must still end)")
    bad = k.run_slim(workspace=ws, wait_budget_us=-1)
    assert binding.slim_status(ws) == binding.SLIM_ERR_TIMEOUT
    assert np.isnan(bad).all()
    say("[case] wait budget: ordinary call on the same workspace again")
    again = k.run_slim(workspace=ws)
    assert binding.slim_status(ws) == binding.SLIM_OK
    assert np.array_equal(again, good)


def test_status_of_library_owned_scratch_is_ok_after_ordinary_calls():
    cfg = synth.scaled(synth.CONFIGS[1], H=8, d=1024, T=700)
    k = KCase(cfg, need_v=False)
    assert k.err(k.run_slim()) <= TOL["bf16"]
    assert binding.slim_status(None) == binding.SLIM_OK
