"""slim_prepare_wkv (host fp64 LU solve, eq. 6) and slim_pack_weights.  CPU only: these
entry points never touch the GPU."""
import math

import numpy as np
import pytest

from oracle import mha_oracle as orc
from paper_2503_05840_amd import binding, synth


def test_closed_form_from_the_svd_construction():
    p = synth.make_problem(synth.CONFIGS[0])
    w, d = p.w, p.cfg.d
    closed = math.sqrt(d) * (w.Vt.T / w.s) @ w.U.T @ w.W_V
    got, rcond = binding.slim_prepare_wkv(w.W_K, w.W_V)
    assert np.abs(got - closed).max() <= 1e-11 * np.abs(closed).max()
    assert np.allclose(w.W_K @ got, w.W_V)                       # App. A acceptance check
    assert 1e-4 < rcond <= 1.0


@pytest.mark.parametrize("d", [1, 2, 7, 63, 64, 65, 130, 257])
def test_matches_numpy_solve_across_block_boundaries(d):
    rng = np.random.default_rng(d)
    A = rng.standard_normal((d, d)) + 0.1 * np.eye(d)
    Bm = rng.standard_normal((d, d))
    got, rcond = binding.slim_prepare_wkv(A, Bm, allow_illcond=True)
    ref = np.linalg.solve(A, Bm)
    assert np.abs(got - ref).max() <= 1e-9 * max(1.0, np.abs(ref).max())
    true_rcond = 1.0 / np.linalg.cond(A, 1)
    assert true_rcond / 3.0 <= rcond * (1 + 1e-9) and rcond <= true_rcond * 10.0 + 1e-300


def test_special_cases():
    rng = np.random.default_rng(1)
    d = 96
    W_V = rng.standard_normal((d, d))
    got, _ = binding.slim_prepare_wkv(np.eye(d), W_V)
    assert np.array_equal(got, W_V)
    W_K = rng.standard_normal((d, d))
    got, _ = binding.slim_prepare_wkv(W_K, W_K)
    assert np.abs(got - np.eye(d)).max() < 1e-10
    perm = rng.permutation(d)
    Pm = np.eye(d)[perm]
    got, _ = binding.slim_prepare_wkv(Pm, W_V)
    assert np.array_equal(got, Pm.T @ W_V)


def test_pivoting_is_needed_and_done():
    A = np.array([[0.0, 1.0], [1.0, 0.0]])
    Bm = np.array([[1.0, 2.0], [3.0, 4.0]])
    got, _ = binding.slim_prepare_wkv(A, Bm)
    assert np.array_equal(got, np.array([[3.0, 4.0], [1.0, 2.0]]))


def test_singular_and_nonfinite_inputs_are_rejected():
    rng = np.random.default_rng(2)
    d = 40
    A = rng.standard_normal((d, d))
    A[:, 7] = A[:, 3]
    with pytest.raises(binding.SlimError) as ei:
        binding.slim_prepare_wkv(A, np.eye(d))
    assert ei.value.code == -6
    A = rng.standard_normal((d, d))
    A[2, 2] = np.nan
    with pytest.raises(binding.SlimError) as ei:
        binding.slim_prepare_wkv(A, np.eye(d))
    assert ei.value.code == -6


def test_ill_conditioned_is_flagged_but_written():
    d = 24
    rng = np.random.default_rng(3)
    U, _ = np.linalg.qr(rng.standard_normal((d, d)))
    V, _ = np.linalg.qr(rng.standard_normal((d, d)))
    s = np.logspace(0, -14, d)
    A = (U * s) @ V.T
    with pytest.raises(binding.SlimError) as ei:
        binding.slim_prepare_wkv(A, np.eye(d))
    assert ei.value.code == -7
    got, rcond = binding.slim_prepare_wkv(A, np.eye(d), allow_illcond=True)
    assert rcond < 1e-12 and np.isfinite(got).all()


def test_pack_weights_rounding():
    rng = np.random.default_rng(4)
    W = rng.standard_normal((33, 40)) * 3.0
    f = binding.slim_pack_weights(W, "f32")
    assert f.dtype == np.float32 and np.array_equal(f, W.astype(np.float32))
    b = binding.slim_pack_weights(W, "bf16")
    assert b.dtype == np.uint16 and np.array_equal(b, synth.f64_to_bf16_bits(W))


# ---- non-square projections, option 1 ----------------------------------------------------------
@pytest.mark.parametrize("d,e", [(5, 12), (64, 256), (130, 200), (96, 96)])
def test_nonsquare_right_inverse_matches_the_printed_formula(d, e):
    rng = np.random.default_rng(100 + d)
    W_K = rng.standard_normal((d, e)) / np.sqrt(d)
    W_V = rng.standard_normal((d, e)) / np.sqrt(d)
    got, rcond = binding.slim_prepare_wkv_nonsquare(W_K, W_V)
    want = orc.wkv_right_inverse(W_K, W_V)
    assert got.shape == (e, e)
    assert np.abs(got - want).max() <= 1e-9 * np.abs(want).max()
    assert np.abs(W_K @ got - W_V).max() <= 1e-10 * np.abs(W_V).max()      # W_K W_KV = W_V
    assert 0 < rcond <= 1


def test_nonsquare_from_the_config4_weights_recovers_v_from_k():
    cfg = synth.scaled(synth.CONFIGS[4], B=1, H=8, d=64, d_k=32, T=50)
    p = synth.make_problem(cfg)
    W_KV, _ = binding.slim_prepare_wkv_nonsquare(p.w.W_K, p.w.W_V)
    X = p.seqs[0].X
    assert np.abs((X @ p.w.W_K) @ W_KV - X @ p.w.W_V).max() <= 1e-10


def test_nonsquare_argument_checks():
    lib = binding.load()
    a = np.zeros((4, 8)); out = np.zeros((8, 8))
    assert lib.slim_prepare_wkv_nonsquare(None, a.ctypes.data, out.ctypes.data, 4, 8, None) == -1
    assert lib.slim_prepare_wkv_nonsquare(a.ctypes.data, a.ctypes.data, out.ctypes.data, 8, 4, None) == -2      # e < d
    assert lib.slim_prepare_wkv_nonsquare(a.ctypes.data, a.ctypes.data, out.ctypes.data, 4, 8, None) == -6      # rank 0
