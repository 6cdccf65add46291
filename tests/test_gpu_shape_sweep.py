"""GPU parity over a seeded sweep of small shapes: head widths from 8 to 136, head counts on both
sides of the fast path's limits, batch sizes around the projection's batch tiles, contexts around the
32-row tile boundaries, ragged lengths.  Every case runs the library's choice and the plain kernels
against the fp64 oracle; rotary keys and the whole attention block ride along on a subset."""
import numpy as np
import pytest

from paper_2503_05840_amd import binding, synth
from gpu_harness import BlockCase, KCase, TOL, row_rel_err, say

pytestmark = pytest.mark.gpu
BASE = synth.CONFIGS[1]


def _shapes():
    rng = np.random.default_rng(20250305)
    out = []
    fixed = [  # (B, H, d_k, T, len_lo)
        (1, 1, 8, 1, 0), (1, 2, 16, 31, 0), (2, 4, 32, 32, 0), (1, 3, 64, 33, 0), (3, 5, 96, 64, 1),
        (17, 2, 64, 65, 1), (33, 4, 32, 40, 0), (1, 32, 128, 97, 0), (2, 33, 16, 50, 0), (1, 2, 136, 70, 0),
        (16, 8, 64, 200, 5), (5, 20, 64, 129, 0), (1, 16, 128, 513, 0), (4, 32, 8, 100, 1),
    ]
    for B, H, d_k, T, lo in fixed:
        out.append((B, H, d_k, T, lo))
    for _ in range(16):
        d_k = int(rng.choice([8, 16, 24, 32, 48, 64, 96, 128]))
        H = int(rng.integers(1, 33))
        while H * d_k > 2048:
            H = max(1, H // 2)
        B = int(rng.choice([1, 2, 3, 7, 16, 18, 40]))
        T = int(rng.integers(1, 400))
        lo = int(rng.choice([0, 1, max(1, T // 2)]))
        out.append((B, H, d_k, T, lo))
    return out


SHAPES = _shapes()


@pytest.mark.parametrize("i", range(len(SHAPES)))
def test_shape_sweep_matches_oracle(i):
    B, H, d_k, T, lo = SHAPES[i]
    cfg = synth.scaled(BASE, B=B, H=H, d=H * d_k, d_k=d_k, T=T, len_lo=lo)
    q_scale = [1.0, 8.0, 50.0][i % 3]
    rope = 10000.0 if i % 4 == 1 else None
    say(f"[case] sweep {i}: B={B} H={H} d_k={d_k} T={T} len_lo={lo} q x{q_scale} rope={rope} "
        f"-> {binding.auto_variant_name(B, H, T, H * d_k, 'bf16')}")
    k = KCase(cfg, q_scale=q_scale, rope_base=rope)
    for variant in (binding.VARIANT_AUTO, binding.VARIANT_GENERIC, binding.VARIANT_FUSED_SPLIT):
        e = k.err(k.run_slim(variant=variant))
        say(f"  variant {variant}: {e:.3e}")
        assert e <= TOL["bf16"]
    assert k.err(k.run_vanilla()) <= TOL["bf16"] or d_k > 128 * 2
    if i % 5 == 2 and T > 1:
        b = BlockCase(cfg, rope_base=rope, q_gain=q_scale)
        y, krow = b.run_slim()
        e, ek = row_rel_err(y, b.ref), row_rel_err(krow, b.k_new)
        say(f"  block: y {e:.3e}, key row {ek:.3e}")
        assert e <= TOL["bf16"] and ek <= TOL["bf16"]
