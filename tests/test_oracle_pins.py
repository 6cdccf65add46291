"""Pins for the CPU oracle: each check ties `oracle/mha_oracle.py` to something other than
itself -- brute force with naive exponentials, closed forms, limits, the invariants of the
paper's bias appendix, and numbers the paper prints.  CPU only."""
import math
import os

import numpy as np
import pytest

from oracle import mha_oracle as orc
from paper_2503_05840_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ------------------------------------------------------------------------------------------
# brute force: eq. 4, 5, 2 written with python floats and loops, exp without a max shift
# ------------------------------------------------------------------------------------------
def brute_force_decode(x_q, X, W_K, W_V, h):
    n, d = len(X), len(X[0])
    e = len(W_K[0])
    d_k = e // h
    K = [[sum(X[t][a] * W_K[a][c] for a in range(d)) for c in range(e)] for t in range(n)]
    V = [[sum(X[t][a] * W_V[a][c] for a in range(d)) for c in range(e)] for t in range(n)]
    out = [0.0] * e
    for i in range(h):
        lo = i * d_k
        w = []
        for t in range(n):
            dot = sum(x_q[lo + j] * K[t][lo + j] for j in range(d_k))
            w.append(math.exp(dot / math.sqrt(d_k)))
        z = sum(w)
        for j in range(d_k):
            out[lo + j] = sum(w[t] / z * V[t][lo + j] for t in range(n))
    return out


@pytest.mark.parametrize("n,d,h,seed", [(1, 4, 2, 0), (3, 4, 1, 1), (5, 8, 2, 2), (8, 6, 3, 3), (7, 8, 4, 4)])
def test_vanilla_matches_brute_force(n, d, h, seed):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((n, d))
    W_K = rng.standard_normal((d, d))
    W_V = rng.standard_normal((d, d))
    q = rng.standard_normal(d)
    ref = brute_force_decode(q.tolist(), X.tolist(), W_K.tolist(), W_V.tolist(), h)
    got = orc.vanilla_decode_from_x(q, X, W_K, W_V, h)
    np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-13)


def test_brute_force_nonsquare_projection():
    """e = h*d_k > d_model (the non-square section's shapes), still eq. 2 per head."""
    rng = np.random.default_rng(11)
    n, d, h, d_k = 6, 3, 4, 2
    X = rng.standard_normal((n, d))
    W_K = rng.standard_normal((d, h * d_k))
    W_V = rng.standard_normal((d, h * d_k))
    q = rng.standard_normal(h * d_k)
    ref = brute_force_decode(q.tolist(), X.tolist(), W_K.tolist(), W_V.tolist(), h)
    np.testing.assert_allclose(orc.vanilla_decode_from_x(q, X, W_K, W_V, h), ref, rtol=1e-12)
    np.testing.assert_allclose(orc.xcache_decode_absorbed(q, X, W_K, W_V, h), ref, rtol=1e-11)


def test_hand_worked_softmax_weights():
    """d_k = 4, two cached rows, keys chosen so q.k/sqrt(d_k) = ln1, ln3 -> p = (1/4, 3/4).
    Catches a missing or wrong 1/sqrt(d_k)."""
    d_k = 4
    q = np.array([2.0, 0.0, 0.0, 0.0])
    K = np.array([[0.0, 5.0, 1.0, -2.0],
                  [math.log(3.0) * math.sqrt(d_k) / 2.0, 7.0, 0.0, 1.0]])
    V = np.array([[1.0, 0.0, 4.0, 8.0], [5.0, 4.0, 0.0, -8.0]])
    P = orc.attention_probs(q, K, 1)
    np.testing.assert_allclose(P, [[0.25, 0.75]], rtol=1e-14)
    np.testing.assert_allclose(orc.vanilla_decode(q, K, V, 1), [4.0, 3.0, 1.0, -4.0], rtol=1e-14)


def test_heads_are_column_blocks():
    """Two heads with different queries: head 0 uniform (q=0), head 1 one-hot in the limit."""
    K = np.array([[0.0, 0.0, 1.0, 0.0], [0.0, 0.0, 0.0, 0.0], [0.0, 0.0, -1.0, 0.0]])
    V = np.arange(12.0).reshape(3, 4)
    q = np.array([0.0, 0.0, 200.0, 0.0])
    out = orc.vanilla_decode(q, K, V, 2)
    np.testing.assert_allclose(out[:2], V[:, :2].mean(axis=0), rtol=1e-14)
    np.testing.assert_allclose(out[2:], V[0, 2:], rtol=1e-12)


# ------------------------------------------------------------------------------------------
# invariants and limits
# ------------------------------------------------------------------------------------------
def _small_problem(seed=5, n=33, d=24, h=3):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((n, d))
    W_K = rng.standard_normal((d, d)) / math.sqrt(d)
    W_V = rng.standard_normal((d, d)) / math.sqrt(d)
    q = rng.standard_normal(d)
    return X, W_K, W_V, q, h


def test_probs_sum_to_one():
    X, W_K, W_V, q, h = _small_problem()
    P = orc.attention_probs(q * 7.0, orc.project(X, W_K), h)
    assert P.shape == (h, X.shape[0])
    np.testing.assert_allclose(P.sum(axis=1), 1.0, rtol=0, atol=1e-14)
    assert (P >= 0).all()


def test_zero_query_gives_mean_value():
    X, W_K, W_V, q, h = _small_problem()
    out = orc.vanilla_decode_from_x(np.zeros_like(q), X, W_K, W_V, h)
    np.testing.assert_allclose(out, X.mean(axis=0) @ W_V, rtol=1e-12, atol=1e-14)


def test_single_row_context_returns_that_value():
    X, W_K, W_V, q, h = _small_problem(n=1)
    np.testing.assert_allclose(orc.vanilla_decode_from_x(q, X, W_K, W_V, h), X[0] @ W_V, rtol=1e-13)


def test_row_permutation_invariance():
    X, W_K, W_V, q, h = _small_problem()
    perm = np.random.default_rng(0).permutation(X.shape[0])
    a = orc.vanilla_decode_from_x(q, X, W_K, W_V, h)
    b = orc.vanilla_decode_from_x(q, X[perm], W_K, W_V, h)
    np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-15)


def test_large_query_selects_argmax_row_per_head():
    X, W_K, W_V, q, h = _small_problem()
    K, V = orc.project(X, W_K), orc.project(X, W_V)
    d_k = K.shape[1] // h
    out = orc.vanilla_decode(q * 1e4, K, V, h)
    for i in range(h):
        cols = slice(i * d_k, (i + 1) * d_k)
        t = int(np.argmax(K[:, cols] @ q[cols]))
        np.testing.assert_allclose(out[cols], V[t, cols], rtol=1e-9)


def test_key_bias_cancels_and_value_bias_passes_through():
    """Bias appendix: a constant vector added to every key leaves the softmax unchanged;
    a constant added to every value is added to the output (weights sum to 1)."""
    X, W_K, W_V, q, h = _small_problem()
    K, V = orc.project(X, W_K), orc.project(X, W_V)
    rng = np.random.default_rng(9)
    c = rng.standard_normal(K.shape[1])
    b = rng.standard_normal(V.shape[1])
    np.testing.assert_allclose(orc.attention_probs(q, K + c, h), orc.attention_probs(q, K, h),
                               rtol=1e-11, atol=1e-15)
    np.testing.assert_allclose(orc.vanilla_decode(q, K, V + b, h), orc.vanilla_decode(q, K, V, h) + b,
                               rtol=1e-12, atol=1e-14)


# ------------------------------------------------------------------------------------------
# eq. 6 / eq. 7 / App. A on the synthetic well-conditioned W_K
# ------------------------------------------------------------------------------------------
@pytest.fixture(scope="module")
def cfg0_problem():
    return synth.make_problem(synth.CONFIGS[0])


def test_wkv_closed_form_from_construction(cfg0_problem):
    """W_K = U diag(s) V^T / sqrt(d)  =>  W_K^-1 = sqrt(d) V diag(1/s) U^T."""
    w = cfg0_problem.w
    d = w.W_K.shape[0]
    closed = math.sqrt(d) * (w.Vt.T / w.s) @ w.U.T @ w.W_V
    got = orc.wkv_by_inverse(w.W_K, w.W_V)
    assert np.abs(got - closed).max() <= 1e-11 * np.abs(closed).max()


def test_wkv_special_cases():
    rng = np.random.default_rng(3)
    d = 12
    W_V = rng.standard_normal((d, d))
    np.testing.assert_allclose(orc.wkv_by_inverse(np.eye(d), W_V), W_V, rtol=1e-14)
    W_K = rng.standard_normal((d, d))
    np.testing.assert_allclose(orc.wkv_by_inverse(W_K, W_K), np.eye(d), atol=1e-11)
    perm = rng.permutation(d)
    Pm = np.eye(d)[perm]                       # (Pm W)[r] = W[perm[r]];  Pm^-1 = Pm^T
    np.testing.assert_allclose(orc.wkv_by_inverse(Pm, W_V), Pm.T @ W_V, rtol=1e-14)


def test_appendix_a_acceptance_check(cfg0_problem):
    w = cfg0_problem.w
    W_KV = orc.wkv_by_inverse(w.W_K, w.W_V)
    assert np.allclose(w.W_K @ W_KV, w.W_V)              # the paper's own check, numpy defaults


def test_v_from_k_identity(cfg0_problem):
    w, sq = cfg0_problem.w, cfg0_problem.seqs[0]
    W_KV = orc.wkv_by_inverse(w.W_K, w.W_V)
    V = orc.project(sq.X, w.W_V)
    V2 = orc.project(sq.X, w.W_K) @ W_KV
    assert np.abs(V - V2).max() <= 1e-10 * np.abs(V).max()


def test_option1_equals_option2_equals_vanilla(cfg0_problem):
    p = cfg0_problem
    w, sq, q, h = p.w, p.seqs[0], p.q[0], p.cfg.H
    K = orc.project(sq.X, w.W_K)
    W_KV = orc.wkv_by_inverse(w.W_K, w.W_V)
    ref = orc.vanilla_decode_from_x(q, sq.X, w.W_K, w.W_V, h)
    o1 = orc.slim_option1(q, K, W_KV, h)
    o2 = orc.slim_option2(q, K, W_KV, h)
    scale = np.abs(ref).max()
    assert np.abs(o1 - ref).max() <= 1e-11 * scale
    assert np.abs(o2 - ref).max() <= 1e-11 * scale


def test_xcache_score_identity_and_output():
    cfg = synth.scaled(synth.CONFIGS[4], B=1, H=8, d=64, d_k=16, T=50)
    p = synth.make_problem(cfg)
    w, sq, q = p.w, p.seqs[0], p.q[0]
    K = orc.project(sq.X, w.W_K)
    for i in (0, 3, 7):
        cols = slice(i * cfg.d_k, (i + 1) * cfg.d_k)
        lhs = (w.W_K[:, cols] @ q[cols]) @ sq.X.T
        rhs = K[:, cols] @ q[cols]
        np.testing.assert_allclose(lhs, rhs, rtol=1e-11, atol=1e-13)
    ref = orc.vanilla_decode_from_x(q, sq.X, w.W_K, w.W_V, cfg.H)
    got = orc.xcache_decode_absorbed(q, sq.X, w.W_K, w.W_V, cfg.H)
    assert np.abs(got - ref).max() <= 1e-11 * np.abs(ref).max()


def test_split_merge_equals_unsplit():
    X, W_K, W_V, q, h = _small_problem(n=41)
    K, V = orc.project(X, W_K), orc.project(X, W_V)
    ref = orc.vanilla_decode(q * 9.0, K, V, h)
    rng = np.random.default_rng(21)
    for trial in range(5):
        perm = rng.permutation(41)
        cuts = np.sort(rng.choice(np.arange(1, 41), size=rng.integers(1, 8), replace=False))
        pieces = [p for p in np.split(perm, cuts) if len(p)]
        got = orc.split_merge_decode(q * 9.0, K, V, h, pieces)
        np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-14)
    # length-1 pieces only
    got = orc.split_merge_decode(q * 9.0, K, V, h, [np.array([t]) for t in range(41)])
    np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-14)


# ------------------------------------------------------------------------------------------
# numbers the paper prints
# ------------------------------------------------------------------------------------------
def _table2_rows():
    rows = {}
    with open(os.path.join(GOLDEN, "table2_complexity.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            name, proj, ops, reads = [s.strip() for s in line.split("|")]
            rows[name] = (proj, ops, reads)
    return rows


@pytest.mark.parametrize("n,d,h", [(16384, 4096, 32), (1500, 1280, 20), (7, 64, 4)])
def test_table2_op_and_read_counts(n, d, h):
    env = {"n": n, "d": d, "h": h}
    for variant, (proj, ops, reads) in _table2_rows().items():
        got_ops, got_reads = orc.mha_ops_reads(n, d, h, variant)
        assert got_ops == eval(ops, {}, env), variant
        assert got_reads == eval(reads, {}, env), variant
        assert orc.projection_ops(n, d, variant) == eval(proj, {}, env), variant
    o, r = orc.mha_ops_reads(n, d, h, "optimized")
    assert o / r == 2 * h + 2                              # intensity column


def test_whisper_table_reads_and_speedups():
    with open(os.path.join(GOLDEN, "whisper_table.txt")) as f:
        rows = [l.split() for l in f if l.strip() and not l.startswith("#")]
    assert len(rows) == 5
    for r in rows:
        d, layers, d_ffn = int(r[1]), int(r[2]), int(r[3])
        v = [float(x) for x in r[4:]]
        reads_b1, reads_b64, speed = v[6:9], v[9:12], v[12:14]
        for opt in range(3):
            assert abs(orc.whisper_reads_per_token(d, layers, d_ffn, 1, opt) / 1e6 - reads_b1[opt]) <= 0.051
            assert abs(orc.whisper_reads_per_token(d, layers, d_ffn, 64, opt) / 1e6 - reads_b64[opt]) <= 0.051
        base = orc.whisper_reads_per_token(d, layers, d_ffn, 64, 0)
        for k, opt in enumerate((1, 2)):
            assert abs(base / orc.whisper_reads_per_token(d, layers, d_ffn, 64, opt) - speed[k]) <= 0.051


def test_phi3_worked_example():
    """Intro example: 3.8 GB params, 25 GB KV-cache at 128k (1 byte per element):
    B=1: 28.8 -> 16.3 GB, 1.8x;  B=16: (400+3.8)/(200+3.8) = 2x (as printed, rounded)."""
    d, layers, n = 3072, 32, 128 * 1024
    _, reads_v = orc.mha_ops_reads(n, d, 32, "vanilla")
    _, reads_s = orc.mha_ops_reads(n, d, 32, "optimized")
    kv_gb, k_gb = reads_v * layers / 1e9, reads_s * layers / 1e9
    assert round(kv_gb) == 26 and abs(k_gb - kv_gb / 2) < 1e-9      # Table 1 prints 25.8B
    assert round((25 + 3.8) / (12.5 + 3.8), 1) == 1.8
    assert round((400 + 3.8) / (200 + 3.8)) == 2


# ------------------------------------------------------------------------------------------
# RoPE appendix: the rotation, its inverse, and option 1 (raw keys in the cache)
# ------------------------------------------------------------------------------------------
def test_rope_quarter_turn_by_hand():
    """d_k = 2, theta_0 = 1: at m = pi/2 the printed encoding gives y1 = x2, y2 = -x1."""
    y = orc.rope_encode(np.array([[1.0, 0.0], [0.0, 1.0], [3.0, -2.0]]), 1, [math.pi / 2] * 3)
    np.testing.assert_allclose(y, [[0.0, -1.0], [1.0, 0.0], [-2.0, -3.0]], atol=1e-15)
    x = orc.rope_decode(np.array([[0.0, -1.0]]), 1, [math.pi / 2])
    np.testing.assert_allclose(x, [[1.0, 0.0]], atol=1e-15)


def test_rope_is_complex_multiplication_per_adjacent_pair():
    """(x1 + i x2) e^{-i m theta_j} on pair j of every head, with theta_j = base^(-2j/d_k) --
    written with python complex numbers, element by element."""
    rng = np.random.default_rng(11)
    n, h, d_k, base = 5, 3, 8, 500.0
    M = rng.standard_normal((n, h * d_k))
    pos = [0, 1, 2, 7, 1000]
    got = orc.rope_encode(M, h, pos, base)
    for t in range(n):
        for i in range(h):
            for j in range(d_k // 2):
                z = complex(M[t, i * d_k + 2 * j], M[t, i * d_k + 2 * j + 1])
                w = z * complex(math.cos(pos[t] * base ** (-2 * j / d_k)), -math.sin(pos[t] * base ** (-2 * j / d_k)))
                assert abs(got[t, i * d_k + 2 * j] - w.real) < 1e-12
                assert abs(got[t, i * d_k + 2 * j + 1] - w.imag) < 1e-12


def test_rope_touches_only_its_own_pair():
    """A unit vector in column 2 of a d_k = 4 head moves only into columns 2 and 3."""
    M = np.zeros((1, 8)); M[0, 6] = 1.0                      # head 1, pair 1, first element
    y = orc.rope_encode(M, 2, [3.0], base=100.0)
    th = 3.0 * 100.0 ** (-2 / 4)
    np.testing.assert_allclose(y[0], [0, 0, 0, 0, 0, 0, math.cos(th), -math.sin(th)], atol=1e-15)


def test_rope_decode_undoes_encode_with_the_same_table():
    rng = np.random.default_rng(12)
    M = rng.standard_normal((40, 4 * 16))
    pos = rng.integers(0, 40000, size=40)
    back = orc.rope_decode(orc.rope_encode(M, 4, pos), 4, pos)
    np.testing.assert_allclose(back, M, atol=1e-13)
    np.testing.assert_allclose(orc.rope_encode(M, 4, np.zeros(40)), M, atol=0)      # position 0: identity
    # rotations: norms of every pair are kept, and positions add up
    Y = orc.rope_encode(M, 4, pos)
    np.testing.assert_allclose(Y[:, 0::2] ** 2 + Y[:, 1::2] ** 2, M[:, 0::2] ** 2 + M[:, 1::2] ** 2, rtol=1e-12)
    np.testing.assert_allclose(orc.rope_encode(Y, 4, 17 - pos), orc.rope_encode(M, 4, np.full(40, 17)), atol=1e-10)


def test_rope_scores_depend_on_relative_position_only():
    """<R_m q, R_t k> is a function of m - t: shifting every position by the same amount leaves
    the softmax arguments, and so the decode result, unchanged."""
    rng = np.random.default_rng(13)
    n, h, d_k = 9, 2, 8
    K = rng.standard_normal((n, h * d_k)); V = rng.standard_normal((n, h * d_k))
    q_raw = rng.standard_normal((1, h * d_k))
    outs = []
    for shift in (0, 5, 123):
        q = orc.rope_encode(q_raw, h, [n + shift])[0]
        Kr = orc.rope_encode(K, h, np.arange(n) + shift)
        outs.append(orc.vanilla_decode(q, Kr, V, h))
    np.testing.assert_allclose(outs[1], outs[0], rtol=1e-11)
    np.testing.assert_allclose(outs[2], outs[0], rtol=1e-10)
    # and the unshifted case is what vanilla_decode_rope computes (row t sits at position t)
    np.testing.assert_allclose(orc.vanilla_decode_rope(orc.rope_encode(q_raw, h, [n])[0], K, V, h), outs[0], rtol=1e-13)


def test_rope_brute_force_decode():
    """vanilla_decode_rope against loops over python floats: rotate each key pair with the
    printed encoding, naive exp, weighted sum of the raw values."""
    rng = np.random.default_rng(14)
    n, h, d_k, base = 6, 2, 4, 50.0
    e = h * d_k
    K = rng.standard_normal((n, e)); V = rng.standard_normal((n, e)); q = rng.standard_normal(e)
    want = [0.0] * e
    for i in range(h):
        w = []
        for t in range(n):
            dot = 0.0
            for j in range(d_k // 2):
                th = t * base ** (-2 * j / d_k)
                x1, x2 = K[t, i * d_k + 2 * j], K[t, i * d_k + 2 * j + 1]
                y1 = x1 * math.cos(th) + x2 * math.sin(th)
                y2 = -x1 * math.sin(th) + x2 * math.cos(th)
                dot += q[i * d_k + 2 * j] * y1 + q[i * d_k + 2 * j + 1] * y2
            w.append(math.exp(dot / math.sqrt(d_k)))
        for c in range(d_k):
            want[i * d_k + c] = sum(w[t] * V[t, i * d_k + c] for t in range(n)) / sum(w)
    np.testing.assert_allclose(orc.vanilla_decode_rope(q, K, V, h, base), want, rtol=1e-12)


def test_rope_option1_on_raw_keys_equals_vanilla_with_rotated_keys(cfg0_problem):
    """The cache keeps raw keys (so that V = K W_KV still holds); rotating them after the read,
    for the scores only, gives the result of a vanilla decode over rotated keys and raw values."""
    p = cfg0_problem
    w, sq, h = p.w, p.seqs[0], p.cfg.H
    q = p.q[0] * 30.0                                       # peaky enough that positions matter
    K = orc.project(sq.X, w.W_K); V = orc.project(sq.X, w.W_V)
    W_KV = orc.wkv_by_inverse(w.W_K, w.W_V)
    ref = orc.vanilla_decode_rope(q, K, V, h)
    got = orc.slim_option2_rope(q, K, W_KV, h)
    assert np.abs(got - ref).max() <= 1e-10 * np.abs(ref).max()
    plain = orc.vanilla_decode(q, K, V, h)
    assert np.abs(plain - ref).max() > 1e-2 * np.abs(ref).max()   # the rotation is not a no-op here


# ------------------------------------------------------------------------------------------
# the whole attention block of one generated token
# ------------------------------------------------------------------------------------------
def _block_problem(seed, n, d, h):
    rng = np.random.default_rng(seed)
    W = [rng.standard_normal((d, d)) / math.sqrt(d) for _ in range(4)]
    X = rng.standard_normal((n, d))
    x = rng.standard_normal(d)
    return x, X, W


def test_block_brute_force_with_python_floats():
    """q, k, v, the appended rows, eq. 2 with naive exp, concat, W_O -- all in loops."""
    n, d, h = 4, 6, 2
    x, X, (W_Q, W_K, W_V, W_O) = _block_problem(21, n, d, h)
    d_k = d // h
    rows = [list(r) for r in X] + [list(x)]                      # inputs of the cached rows, then the new token
    K = [[sum(r[a] * W_K[a][c] for a in range(d)) for c in range(d)] for r in rows]
    V = [[sum(r[a] * W_V[a][c] for a in range(d)) for c in range(d)] for r in rows]
    q = [sum(x[a] * W_Q[a][c] for a in range(d)) for c in range(d)]
    cat = [0.0] * d
    for i in range(h):
        w = [math.exp(sum(q[i * d_k + j] * K[t][i * d_k + j] for j in range(d_k)) / math.sqrt(d_k)) for t in range(n + 1)]
        for j in range(d_k):
            cat[i * d_k + j] = sum(w[t] * V[t][i * d_k + j] for t in range(n + 1)) / sum(w)
    want = [sum(cat[a] * W_O[a][c] for a in range(d)) for c in range(d)]
    y, k, v = orc.attention_block(x, X @ W_K, X @ W_V, W_Q, W_K, W_V, W_O, h)
    np.testing.assert_allclose(y, want, rtol=1e-12)
    np.testing.assert_allclose(k, K[n], rtol=1e-12)
    np.testing.assert_allclose(v, V[n], rtol=1e-12)


def test_block_with_an_empty_cache_is_two_products():
    """No cached rows: the one weight is 1, so y = x W_V W_O whatever W_Q, W_K and positions are."""
    x, X, (W_Q, W_K, W_V, W_O) = _block_problem(22, 0, 8, 2)
    empty = np.zeros((0, 8))
    for base in (None, 10000.0):
        y, _, _ = orc.attention_block(x, empty, empty, W_Q, W_K, W_V, W_O, 2, rope_base=base)
        np.testing.assert_allclose(y, x @ W_V @ W_O, rtol=1e-12)


def test_block_with_zero_query_weights_averages_old_and_new_values():
    n, d, h = 7, 8, 4
    x, X, (W_Q, W_K, W_V, W_O) = _block_problem(23, n, d, h)
    y, _, v = orc.attention_block(x, X @ W_K, X @ W_V, np.zeros((d, d)), W_K, W_V, W_O, h)
    mean_v = (np.sum(X @ W_V, axis=0) + v) / (n + 1)
    np.testing.assert_allclose(y, mean_v @ W_O, rtol=1e-12)


def test_block_is_the_decode_step_between_its_projections():
    """attention_block = vanilla_decode over the extended caches, then W_O; with rotary keys the new
    token sits at position n and only the query/key side is rotated."""
    n, d, h = 9, 16, 2
    x, X, (W_Q, W_K, W_V, W_O) = _block_problem(24, n, d, h)
    Xe = np.vstack([X, x[None, :]])
    y, _, _ = orc.attention_block(x, X @ W_K, X @ W_V, W_Q, W_K, W_V, W_O, h)
    np.testing.assert_allclose(y, orc.vanilla_decode_from_x(x @ W_Q, Xe, W_K, W_V, h) @ W_O, rtol=1e-12)
    yr, _, _ = orc.attention_block(x, X @ W_K, X @ W_V, W_Q, W_K, W_V, W_O, h, rope_base=100.0)
    qr = orc.rope_encode((x @ W_Q)[None, :], h, [n], 100.0)[0]
    np.testing.assert_allclose(yr, orc.vanilla_decode_rope(qr, Xe @ W_K, Xe @ W_V, h, 100.0) @ W_O, rtol=1e-12)
    assert np.abs(yr - y).max() > 1e-3 * np.abs(y).max()


# ------------------------------------------------------------------------------------------
# non-square section, option 1: right inverse
# ------------------------------------------------------------------------------------------
def test_right_inverse_properties_and_decode_identity():
    rng = np.random.default_rng(31)
    d, e, h, n = 6, 16, 4, 11
    W_K = rng.standard_normal((d, e)); W_V = rng.standard_normal((d, e))
    X = rng.standard_normal((n, d)); q = rng.standard_normal(e)
    W_KV = orc.wkv_right_inverse(W_K, W_V)
    assert W_KV.shape == (e, e)
    # the defining property, and the library's Moore-Penrose routine (full row rank: they coincide)
    np.testing.assert_allclose(W_K @ W_KV, W_V, atol=1e-12)
    np.testing.assert_allclose(W_KV, np.linalg.pinv(W_K) @ W_V, atol=1e-12)
    # V from K, and the decode result over the e-wide K-cache
    K, V = X @ W_K, X @ W_V
    np.testing.assert_allclose(K @ W_KV, V, atol=1e-12)
    ref = orc.vanilla_decode(q, K, V, h)
    np.testing.assert_allclose(orc.slim_option2(q, K, W_KV, h), ref, rtol=1e-10)
    np.testing.assert_allclose(orc.slim_option1(q, K, W_KV, h), ref, rtol=1e-10)
    # a square W_K brings back eq. 6
    W_sq = rng.standard_normal((d, d)); W_v2 = rng.standard_normal((d, d))
    np.testing.assert_allclose(orc.wkv_right_inverse(W_sq, W_v2), orc.wkv_by_inverse(W_sq, W_v2), atol=1e-10)
