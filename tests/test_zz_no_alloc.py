"""slim_decode_static (the entry point for callers that cannot allocate) against slim_decode, through the
C ABI: two calls in a row on the shared static scratch, the second with a smaller input, each compared
with the existing entry point's output (same kernels: bit for bit) and with the fp64 oracle; a shape
whose scratch plan exceeds the array is refused before anything is launched."""
import ctypes

import numpy as np
import pytest

from paper_2503_05840_amd import binding, synth
from gpu_harness import KCase, TOL, say

pytestmark = pytest.mark.gpu


def _static(k, **kw):
    import torch
    c = k.cfg
    out = torch.full((c.B, c.d), float("nan"), device="cuda", dtype=torch.float32)
    binding.slim_decode_static(k.q, k.K, k.Wkv, out, c.B, c.H, c.T, c.d, **k._kw(**kw))
    torch.cuda.synchronize()
    return out.cpu().numpy()


def test_static_scratch_entry_point_matches_slim_decode_on_two_calls_in_a_row():
    binding.slim_init()
    big = KCase(synth.scaled(synth.CONFIGS[2], B=3, T=3000, len_lo=1200), need_v=False)      # ragged, d_k = 96, fast path
    small = KCase(synth.scaled(synth.CONFIGS[1], H=8, d=1024, T=333), need_v=False)           # smaller, other geometry
    tiny32 = KCase(synth.scaled(synth.CONFIGS[0], T=100), need_v=False)                       # fp32: the plain kernels
    for name, k in (("first (larger)", big), ("second (smaller)", small), ("third (fp32)", tiny32)):
        c = k.cfg
        assert binding.slim_workspace_bytes(c.B, c.H, c.T, c.d, c.dtype) <= binding.slim_static_scratch_bytes()
        say(f"[case] static scratch, {name}: B={c.B} H={c.H} d={c.d} T={c.T} {c.dtype}")
        got = _static(k)
        assert binding.slim_status(binding.STATIC_SCRATCH) == binding.SLIM_OK
        want = k.run_slim()
        assert np.array_equal(got, want)
        assert k.err(got) <= TOL[c.dtype]
    # and the larger one once more, after the smaller ones have left their contents in the array
    again = _static(big)
    assert np.array_equal(again, big.run_slim())


def test_static_scratch_entry_point_refuses_what_does_not_fit_and_foreign_scratch():
    import torch
    lib = binding.load()
    B, H, T, d = 16, 32, 32768, 3072                    # config 2: its scratch plan is larger than the array
    assert binding.slim_workspace_bytes(B, H, T, d, "bf16") > binding.slim_static_scratch_bytes()
    x = torch.zeros(256, device="cuda")
    o = binding.SlimOpts()
    o.dtype = binding.SLIM_BF16
    p = x.data_ptr()
    assert lib.slim_decode_static(p, p, p, p, B, H, T, d, ctypes.byref(o)) == -5          # SLIM_ERR_WORKSPACE, nothing launched
    o.workspace = p
    o.workspace_bytes = 1024
    assert lib.slim_decode_static(p, p, p, p, 1, 8, 64, 512, ctypes.byref(o)) == -1       # SLIM_ERR_ARG: brings its own scratch
    torch.cuda.synchronize()
