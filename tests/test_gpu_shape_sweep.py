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
    k = KCase(cfg, q_scale=q_scale, rope_base=rope, t_stride=(T + 31) // 32 * 32)    # whole 32-row bands per sequence
    fast = binding.auto_variant_name(B, H, T, H * d_k, "bf16") == "fused"
    for variant in (binding.VARIANT_AUTO, binding.VARIANT_GENERIC, binding.VARIANT_FUSED_SPLIT):
        o = k.run_slim(variant=variant)
        e = k.err(o)
        say(f"  variant {variant}: {e:.3e}")
        assert e <= TOL["bf16"]
        if fast and variant != binding.VARIANT_GENERIC:           # the banded cache: same arithmetic, other addresses
            assert np.array_equal(o, k.run_slim(variant=variant, banded=True))
    assert k.err(k.run_vanilla()) <= TOL["bf16"]
    if i % 5 == 2 and T > 1:
        b = BlockCase(cfg, rope_base=rope, q_gain=q_scale)
        y, krow = b.run_slim()
        e, ek = row_rel_err(y, b.ref), row_rel_err(krow, b.k_new)
        say(f"  block: y {e:.3e}, key row {ek:.3e}")
        assert e <= TOL["bf16"] and ek <= TOL["bf16"]


def _xshapes():
    rng = np.random.default_rng(20250306)
    out = [  # (B, H, d_model, d_k, T, ragged)
        (1, 1, 128, 32, 1, False), (2, 3, 128, 64, 31, False), (1, 16, 256, 32, 129, True), (3, 17, 128, 32, 200, True),
        (1, 20, 1280, 64, 150, False), (17, 4, 256, 96, 77, True), (1, 33, 384, 32, 260, False), (2, 130, 128, 32, 140, True),
        (1, 8, 2560, 32, 40, False),
    ]
    for _ in range(9):
        H = int(rng.choice([2, 5, 12, 24, 40, 64]))
        d_k = int(rng.choice([32, 64, 128]))
        dm = int(rng.choice([128, 256, 512, 640]))
        out.append((int(rng.choice([1, 2, 5])), H, dm, d_k, int(rng.integers(1, 500)), bool(rng.integers(0, 2))))
    return out


XSHAPES = _xshapes()


@pytest.mark.parametrize("i", range(len(XSHAPES)))
def test_xcache_shape_sweep_matches_oracle(i):
    from gpu_harness import XCase
    B, H, dm, d_k, T, ragged = XSHAPES[i]
    cfg = synth.scaled(synth.CONFIGS[4], B=B, H=H, d=dm, d_k=d_k, T=T)
    lens = None
    if ragged:
        lens = np.random.default_rng(i).integers(1, T + 1, size=B).astype(np.int32)
        lens[0] = T
    q_scale = [1.0, 2.0, 4.0][i % 3]
    say(f"[case] xcache sweep {i}: B={B} H={H} d_model={dm} d_k={d_k} T={T} lens={None if lens is None else lens.tolist()} q x{q_scale}")
    x = XCase(cfg, q_scale=q_scale, lens=lens)
    for variant in (binding.VARIANT_AUTO, binding.VARIANT_GENERIC, binding.VARIANT_FUSED_SPLIT):   # (FUSED_SPLIT: two passes over X)
        e = x.err(x.run(variant=variant))
        say(f"  variant {variant}: {e:.3e}")
        assert e <= TOL["bf16"]


PARTITIONS = [  # (B, H, d_k, T, len_lo): batches and lengths that move the host's choice of partition and launch count
    (20, 16, 128, 203, 0), (64, 20, 64, 300, 0), (100, 8, 64, 50, 0), (200, 4, 32, 33, 1), (1024, 2, 32, 5, 1),
    (1025, 2, 32, 3, 0), (16, 32, 96, 1000, 1), (2, 32, 128, 5000, 100), (9, 12, 64, 777, 300), (1, 24, 128, 2049, 0),
    (17, 32, 128, 64, 0), (48, 32, 64, 96, 10), (130, 20, 64, 31, 0),
    # more than 32 heads / more than 1024 sequences: plain score and sum kernels, MFMA merge + projection
    (2, 40, 64, 300, 50), (1, 64, 128, 257, 0), (3, 96, 32, 90, 1), (1100, 2, 32, 4, 1), (20, 48, 96, 70, 0),
]


@pytest.mark.parametrize("i", range(len(PARTITIONS)))
def test_partition_sweep_matches_oracle(i):
    B, H, d_k, T, lo = PARTITIONS[i]
    cfg = synth.scaled(BASE, B=B, H=H, d=H * d_k, d_k=d_k, T=T, len_lo=lo)
    rope = 10000.0 if i % 3 == 0 else None
    say(f"[case] partition sweep {i}: B={B} H={H} d_k={d_k} T={T} len_lo={lo} rope={rope} "
        f"-> {binding.auto_variant_name(B, H, T, H * d_k, 'bf16')}")
    k = KCase(cfg, q_scale=8.0, rope_base=rope, need_v=False, t_stride=(T + 31) // 32 * 32)
    outs = []
    for variant in (binding.VARIANT_AUTO, binding.VARIANT_FUSED_SPLIT, binding.VARIANT_GENERIC):
        o = k.run_slim(variant=variant)
        e = k.err(o)
        say(f"  variant {variant}: {e:.3e}")
        assert e <= TOL["bf16"]
        outs.append(o)
    assert np.array_equal(outs[0], k.run_slim())                  # repeatable
    if binding.auto_variant_name(B, H, T, H * d_k, "bf16") == "fused":
        assert np.array_equal(outs[0], k.run_slim(banded=True))   # and the same from the banded cache
        assert np.array_equal(outs[1], k.run_slim(variant=binding.VARIANT_FUSED_SPLIT, banded=True))
