"""CPU fp64 oracle for the slim-attention decode step.  TEST INFRASTRUCTURE ONLY.

This file is the plain definition the HIP path is checked against.  It is slow on
purpose, shares no code with the library under `paper_2503_05840_amd/`, never calls the
library's `slim_prepare_wkv`, and must only be imported by `tests/`, by
`__graft_entry__.smoke()` and by the `cpu_baseline` leg of `bench.py`.

What it computes (row-vector convention, W[in][out], head i = column block
[i*d_k, (i+1)*d_k) of the projection width e = h*d_k):

  * `vanilla_decode`      -- eq. 4, 5, 2 of the paper for a single new query row, storing
                             BOTH caches K = X W_K and V = X W_V, no causal mask, output is
                             concat(head_1..head_h) before W_O.  This is the reference
                             result; slim attention reaches exactly this result.
  * `wkv_by_inverse`      -- eq. 6 / App. A:  W_KV = inv(W_K) W_V in fp64.
  * `wkv_right_inverse`   -- non-square section, option 1: W_KV from the right inverse of a
                             d x e W_K.
  * `slim_option1/2`      -- the two evaluation orders of eq. 7, in fp64, used only to pin
                             the identity the GPU path relies on.
  * `xcache_decode_absorbed` -- the X-cache scheme of the non-square section (Fig. 4):
                             scores via (q_i W_K,i^T) X^T, output via (p X) W_V,i.
  * `split_merge_decode`  -- a decode evaluated on an arbitrary partition of the context
                             with a log-sum-exp merge (the algebra behind split-T).
  * `rope_encode/decode`  -- the 2-D rotation of the RoPE appendix applied to adjacent column
                             pairs of every head, with one angle table for both directions.
  * `vanilla_decode_rope` -- the reference result when keys carry rotary positions: scores
                             against the rotated keys, values untouched.
  * `slim_option2_rope`   -- option 1 of the RoPE appendix on top of eq. 7 option 2: the cache
                             holds raw keys, rotated after reading for the scores only.
  * `attention_block`     -- the whole attention block of one generated token (Fig. 1 / Table 2's
                             projection column): q, k, v from the token's input, the new rows
                             appended to the caches, eq. 2 over old and new rows, then W_O.
  * `mha_ops_reads`       -- App. B / Table 2 op and read counts, by enumerating matmuls.
  * `whisper_reads_per_token` -- the closed-form arithmetic of the Whisper table.

Every function is pinned by `tests/test_oracle_pins.py` against something other than
itself (brute force with naive exp on tiny shapes, closed forms, limits, invariants of
App. F, values printed in the paper's tables); nothing here is "parity unpinned".
"""
from __future__ import annotations

import numpy as np


# --------------------------------------------------------------------------------------
# eq. 4/5: projections (prompt phase; builds the caches the decode step reads)
# --------------------------------------------------------------------------------------
def project(X: np.ndarray, W: np.ndarray) -> np.ndarray:
    """K = X W_K or V = X W_V (eq. 4, 5), fp64."""
    return np.asarray(X, np.float64) @ np.asarray(W, np.float64)


# --------------------------------------------------------------------------------------
# eq. 2: one query row against the cached rows
# --------------------------------------------------------------------------------------
def attention_probs(q: np.ndarray, K: np.ndarray, h: int) -> np.ndarray:
    """softmax(q_i K_i^T / sqrt(d_k)) for every head i; returns (h, n).  eq. 2."""
    q = np.asarray(q, np.float64)
    K = np.asarray(K, np.float64)
    n, e = K.shape
    d_k = e // h
    assert d_k * h == e and q.shape == (e,) and n >= 1
    P = np.empty((h, n))
    for i in range(h):
        cols = slice(i * d_k, (i + 1) * d_k)
        s = (K[:, cols] @ q[cols]) / np.sqrt(d_k)
        w = np.exp(s - s.max())
        P[i] = w / w.sum()
    return P


def vanilla_decode(q: np.ndarray, K: np.ndarray, V: np.ndarray, h: int) -> np.ndarray:
    """concat_i softmax(q_i K_i^T / sqrt(d_k)) V_i  (eq. 2, eq. 5 without W_O).

    q (e,), K and V (n, e): the n cached rows are all attended to; returns (e,)."""
    V = np.asarray(V, np.float64)
    n, e = V.shape
    d_k = e // h
    P = attention_probs(q, K, h)
    out = np.empty(e)
    for i in range(h):
        cols = slice(i * d_k, (i + 1) * d_k)
        out[cols] = P[i] @ V[:, cols]
    return out


def vanilla_decode_from_x(x_q: np.ndarray, X: np.ndarray, W_K: np.ndarray, W_V: np.ndarray,
                          h: int) -> np.ndarray:
    """The reference for one sequence: build K and V from the cached activations X
    (eq. 4, 5), then one vanilla decode step with the already projected query x_q."""
    return vanilla_decode(x_q, project(X, W_K), project(X, W_V), h)


# --------------------------------------------------------------------------------------
# eq. 6 and eq. 7 in fp64
# --------------------------------------------------------------------------------------
def wkv_by_inverse(W_K: np.ndarray, W_V: np.ndarray) -> np.ndarray:
    """W_KV = W_K^{-1} W_V (eq. 6), the route App. A takes: explicit inverse, fp64."""
    return np.linalg.inv(np.asarray(W_K, np.float64)) @ np.asarray(W_V, np.float64)


def wkv_right_inverse(W_K: np.ndarray, W_V: np.ndarray) -> np.ndarray:
    """Non-square section, option 1: for W_K (d x e, e > d) the right inverse is
    W_K^T (W_K W_K^T)^{-1}, so W_KV = W_K^T (W_K W_K^T)^{-1} W_V (e x e).  Written as printed:
    an explicit inverse of the d x d term, fp64."""
    W_K = np.asarray(W_K, np.float64)
    return W_K.T @ np.linalg.inv(W_K @ W_K.T) @ np.asarray(W_V, np.float64)


def slim_option1(q, K, W_KV, h):
    """eq. 7 option 1: softmax(.) [K W_KV,i] -- V_i is rebuilt from the whole K-cache."""
    K = np.asarray(K, np.float64)
    n, d = K.shape
    d_k = d // h
    P = attention_probs(q, K, h)
    out = np.empty(d)
    for i in range(h):
        cols = slice(i * d_k, (i + 1) * d_k)
        V_i = K @ W_KV[:, cols]
        out[cols] = P[i] @ V_i
    return out


def slim_option2(q, K, W_KV, h):
    """eq. 7 option 2: [softmax(.) K] W_KV,i -- weighted sum of full-width K rows first."""
    K = np.asarray(K, np.float64)
    n, d = K.shape
    d_k = d // h
    P = attention_probs(q, K, h)
    out = np.empty(d)
    for i in range(h):
        cols = slice(i * d_k, (i + 1) * d_k)
        c_i = P[i] @ K                      # (d,)
        out[cols] = c_i @ W_KV[:, cols]
    return out


# --------------------------------------------------------------------------------------
# RoPE appendix: rotary positions on the keys, option 1 (rotate after reading the cache)
# --------------------------------------------------------------------------------------
def rope_angles(positions, d_k: int, base: float = 10000.0) -> np.ndarray:
    """m * theta_j for every position m and column pair j of a head; returns (n, d_k/2).

    The appendix writes only "m theta" for the 2-D case; the frequencies are those of the
    RoPE paper it cites: theta_j = base^(-2j/d_k), j = 0 .. d_k/2 - 1."""
    assert d_k % 2 == 0
    m = np.asarray(positions, np.float64).reshape(-1, 1)
    theta = np.asarray([base ** (-2.0 * j / d_k) for j in range(d_k // 2)], np.float64)
    return m * theta.reshape(1, -1)


def _rotate_pairs(M, h, ang, direction):
    M = np.asarray(M, np.float64)
    n, e = M.shape
    d_k = e // h
    assert d_k * h == e and ang.shape == (n, d_k // 2)
    c, s = np.cos(ang), np.sin(ang) * direction
    out = np.empty_like(M)
    for i in range(h):
        x1 = M[:, i * d_k + 0:(i + 1) * d_k:2]     # first element of each adjacent pair
        x2 = M[:, i * d_k + 1:(i + 1) * d_k:2]
        out[:, i * d_k + 0:(i + 1) * d_k:2] = x1 * c + x2 * s
        out[:, i * d_k + 1:(i + 1) * d_k:2] = -x1 * s + x2 * c
    return out


def rope_encode(M, h, positions, base=10000.0):
    """RoPE encoding of the appendix, per head and adjacent pair (x1, x2) at position m:
    y1 = x1 cos(m theta) + x2 sin(m theta),  y2 = -x1 sin(m theta) + x2 cos(m theta)."""
    M = np.asarray(M, np.float64)
    return _rotate_pairs(M, h, rope_angles(positions, M.shape[1] // h, base), +1.0)


def rope_decode(Y, h, positions, base=10000.0):
    """RoPE decoding of the appendix: the opposite rotation with the same coefficients,
    x1 = y1 cos - y2 sin,  x2 = y1 sin + y2 cos."""
    Y = np.asarray(Y, np.float64)
    return _rotate_pairs(Y, h, rope_angles(positions, Y.shape[1] // h, base), -1.0)


def vanilla_decode_rope(q, K, V, h, base=10000.0):
    """Vanilla decode when keys carry rotary positions: cached row t is rotated by position t,
    the query is taken as given (already rotated to its own position by the caller), values
    are not rotated."""
    n = np.asarray(K).shape[0]
    return vanilla_decode(q, rope_encode(K, h, np.arange(n), base), V, h)


def slim_option2_rope(q, K, W_KV, h, base=10000.0):
    """Option 1 of the RoPE appendix with eq. 7 option 2: the cache holds the raw keys; they are
    rotated after reading for the softmax arguments, and the raw rows enter the weighted sum
    that W_KV,i turns into the head output."""
    K = np.asarray(K, np.float64)
    n, d = K.shape
    d_k = d // h
    P = attention_probs(q, rope_encode(K, h, np.arange(n), base), h)
    out = np.empty(d)
    for i in range(h):
        cols = slice(i * d_k, (i + 1) * d_k)
        out[cols] = (P[i] @ K) @ W_KV[:, cols]
    return out


# --------------------------------------------------------------------------------------
# the steps either side of the decode step: one generated token through the attention block
# --------------------------------------------------------------------------------------
def attention_block(x, K_cache, V_cache, W_Q, W_K, W_V, W_O, h, rope_base=None):
    """One token with input row x (d,) through multi-head attention, vanilla and in fp64.

    q = x W_Q, k = x W_K, v = x W_V (eq. 3-5 for one row); k and v are stored after the n rows
    already cached and all n + 1 rows are read back (the generate-phase description under Fig. 2);
    heads as in eq. 2; the concatenation goes through W_O (eq. 1).  With rope_base, the new token
    sits at position n: its query and key are rotated there, cached key row t at position t.
    Returns (y, k, v): the block output (d,) and the raw new rows."""
    x = np.asarray(x, np.float64)
    K_cache = np.asarray(K_cache, np.float64)
    V_cache = np.asarray(V_cache, np.float64)
    n = K_cache.shape[0]
    q, k, v = x @ W_Q, x @ W_K, x @ W_V
    K = np.vstack([K_cache, k[None, :]])
    V = np.vstack([V_cache, v[None, :]])
    if rope_base is not None:
        q = rope_encode(q[None, :], h, [n], rope_base)[0]
        K = rope_encode(K, h, np.arange(n + 1), rope_base)
    return vanilla_decode(q, K, V, h) @ np.asarray(W_O, np.float64), k, v


# --------------------------------------------------------------------------------------
# non-square section, option 2 (Fig. 4): X-cache
# --------------------------------------------------------------------------------------
def xcache_decode_absorbed(q, X, W_K, W_V, h):
    """A_i = (q_i W_K,i^T) X^T ; head_i = (softmax(A_i / sqrt(d_k)) X) W_V,i.

    q (e,) projected query, X (n, d_model), W_K and W_V (d_model, e)."""
    q = np.asarray(q, np.float64)
    X = np.asarray(X, np.float64)
    e = W_K.shape[1]
    d_k = e // h
    out = np.empty(e)
    for i in range(h):
        cols = slice(i * d_k, (i + 1) * d_k)
        q_t = W_K[:, cols] @ q[cols]        # (d_model,)  = q_i W_K,i^T
        s = (X @ q_t) / np.sqrt(d_k)
        w = np.exp(s - s.max())
        p = w / w.sum()
        out[cols] = (p @ X) @ W_V[:, cols]
    return out


# --------------------------------------------------------------------------------------
# split-T algebra: partial (m, l, acc) per piece and a log-sum-exp merge
# --------------------------------------------------------------------------------------
def split_merge_decode(q, K, V, h, pieces):
    """vanilla_decode evaluated piecewise.  `pieces` is a list of index arrays that
    partition range(n).  Per piece and head: m = max score, l = sum exp(s - m),
    acc = sum exp(s - m) V_i[t]; merged with weights exp(m_piece - m_all)."""
    q = np.asarray(q, np.float64)
    K = np.asarray(K, np.float64)
    V = np.asarray(V, np.float64)
    n, e = K.shape
    d_k = e // h
    out = np.empty(e)
    for i in range(h):
        cols = slice(i * d_k, (i + 1) * d_k)
        ms, ls, accs = [], [], []
        for idx in pieces:
            s = (K[idx][:, cols] @ q[cols]) / np.sqrt(d_k)
            m = s.max()
            w = np.exp(s - m)
            ms.append(m); ls.append(w.sum()); accs.append(w @ V[idx][:, cols])
        m_all = max(ms)
        num = sum(np.exp(m - m_all) * a for m, a in zip(ms, accs))
        den = sum(np.exp(m - m_all) * l for m, l in zip(ms, ls))
        out[cols] = num / den
    return out


# --------------------------------------------------------------------------------------
# App. B / Table 2: op and read counts per generated token per layer, batch 1
# --------------------------------------------------------------------------------------
def _matmul_ops(m, k, p):
    """A (m x k)(k x p) product: m*k*p MULs and m*p*(k-1) ADDs, counted as ~2mkp OPs
    (footnote of the option-1/option-2 list and first paragraph of App. B)."""
    return 2 * m * k * p


def mha_ops_reads(n: int, d: int, h: int, variant: str):
    """(OPs, cache reads) of the attention part for one token, by listing the matmuls each
    head performs.  variant: 'vanilla' | 'unoptimized' | 'optimized' (rows of Table 2)."""
    d_k = d // h
    ops = 0
    for _ in range(h):
        ops += _matmul_ops(1, d_k, n)            # softmax argument q_i K_i^T
        if variant in ("vanilla", "unoptimized"):
            ops += _matmul_ops(1, n, d_k)        # weighted sum of V_i
        elif variant == "optimized":
            ops += _matmul_ops(1, n, d)          # weighted sum of full-width K
        else:
            raise ValueError(variant)
    reads = 2 * n * d if variant == "vanilla" else n * d
    return ops, reads


def projection_ops(n: int, d: int, variant: str) -> int:
    """Projection OPs per token (Table 2, left half): x W_Q, x W_K, x W_V or the W_KV
    product, and W_O."""
    if variant == "vanilla":
        return 4 * _matmul_ops(1, d, d)
    if variant == "unoptimized":                 # K W_KV over the whole cache + Q, K, O
        return _matmul_ops(n, d, d) + 3 * _matmul_ops(1, d, d)
    if variant == "optimized":                   # per head (1 x d)(d x d_k), h heads = 2d^2; + Q, K, O
        return _matmul_ops(1, d, d) + 3 * _matmul_ops(1, d, d)
    raise ValueError(variant)


# --------------------------------------------------------------------------------------
# Whisper table (encoder-decoder section): reads per token, in elements
# --------------------------------------------------------------------------------------
def whisper_reads_per_token(d, layers, d_ffn, batch, option, p=1500, n_dec=448, vocab=51865):
    """Memory reads per generated token (elements) = cache + params / batch, for the
    baseline (option 0), option 1 (no V-caches, + cross W_KV... counted as d^2 per layer)
    and option 2 (no cross cache, + 2 d^2 per layer), as the table's Notes column defines."""
    cross = 2 * p * d * layers
    self_ = 2 * n_dec * d * layers
    base_params = d * vocab + layers * (6 * d * d + 2 * d * d_ffn)
    if option == 0:
        cache, params = cross + self_, base_params
    elif option == 1:
        cache, params = (cross + self_) / 2, base_params + d * d * layers
    elif option == 2:
        cache, params = self_ / 2, base_params + 2 * d * d * layers
    else:
        raise ValueError(option)
    return cache + params / batch
