"""Seeded synthetic inputs for the slim-attention decode path.

This module only *draws and shapes inputs* (weights, activations, queries,
context lengths, dtype rounding of the cache).  It holds none of the method's
arithmetic: no softmax, no attention, no W_KV.  Both the CPU oracle's tests and
the HIP path's tests/bench take their inputs from here so that the two sides
see identical numbers.

Shapes follow the models the paper lists (Table 1: CodeLlama-7B d=4096/16k,
Phi-3-mini d=3072/128k, Whisper-large d=1280 with 1500 encoder frames; the
non-square table: T5-11B d=1024, d_k=128, h=128, e=16384).  No weights, prompts
or audio of those models are used; everything is random with a fixed seed.

Draw order per config (fixed, so a seed names one input set):
    s, G_U, G_V, W_V, W_Q, then per sequence b: len_b, X_b, x_b
X-cache config: W_K, W_V, W_Q, then per sequence: X_b, x_b.
"""
from __future__ import annotations

import dataclasses
import numpy as np

SEED_BASE = 2025030500


@dataclasses.dataclass(frozen=True)
class Config:
    index: int
    name: str
    kind: str          # "kcache" (square W_K, K-only cache) or "xcache" (e > d_model)
    B: int
    H: int
    d: int             # d_model (= H*d_k for kcache configs)
    d_k: int
    T: int             # allocated rows per sequence (max context)
    dtype: str         # "f32" or "bf16": element type of the cache and the packed weights
    len_lo: int = 0    # ragged lengths drawn Uniform{len_lo..T} when len_lo > 0
    x_pre_rounded: bool = False   # activations are bf16 values already (the oracle sees them rounded)

    @property
    def e(self) -> int:
        return self.H * self.d_k


CONFIGS = {
    0: Config(0, "tiny-fp32", "kcache", B=1, H=8, d=512, d_k=64, T=256, dtype="f32"),
    1: Config(1, "codellama7b-16k", "kcache", B=1, H=32, d=4096, d_k=128, T=16384, dtype="bf16"),
    2: Config(2, "phi3mini-b16-ragged", "kcache", B=16, H=32, d=3072, d_k=96, T=32768,
              dtype="bf16", len_lo=8192),
    3: Config(3, "whisper-large-cross-b64", "kcache", B=64, H=20, d=1280, d_k=64, T=1500,
              dtype="bf16", x_pre_rounded=True),
    4: Config(4, "t5-11b-xcache", "xcache", B=8, H=128, d=1024, d_k=128, T=4096,
              dtype="bf16", x_pre_rounded=True),
}


def scaled(cfg: Config, **kw) -> Config:
    """A smaller (or otherwise altered) copy of a config for tests; same recipe, same seed."""
    return dataclasses.replace(cfg, **kw)


# ----------------------------------------------------------------------------------------------
# dtype helpers (input preparation only)
# ----------------------------------------------------------------------------------------------
def f64_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """fp64 -> fp32 (RNE) -> bf16 (RNE); returns uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float64).astype(np.float32).view(np.uint32)
    rnd = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + rnd) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def round_through(a: np.ndarray, dtype: str) -> np.ndarray:
    """Value of `a` after storage in `dtype`, returned as fp64."""
    if dtype == "bf16":
        return bf16_bits_to_f64(f64_to_bf16_bits(a))
    if dtype == "f32":
        return np.asarray(a, dtype=np.float64).astype(np.float32).astype(np.float64)
    raise ValueError(dtype)


def to_storage(a: np.ndarray, dtype: str) -> np.ndarray:
    """`a` in the cache's storage type: float32 array, or uint16 bf16 bit patterns."""
    if dtype == "bf16":
        return f64_to_bf16_bits(a)
    if dtype == "f32":
        return np.ascontiguousarray(a, dtype=np.float64).astype(np.float32)
    raise ValueError(dtype)


# ----------------------------------------------------------------------------------------------
# weights
# ----------------------------------------------------------------------------------------------
def _orthogonal_from(G: np.ndarray) -> np.ndarray:
    Q, R = np.linalg.qr(G)
    return Q * np.sign(np.diag(R))          # sign-fixed so the factor is unique


@dataclasses.dataclass
class Weights:
    W_Q: np.ndarray
    W_K: np.ndarray
    W_V: np.ndarray
    # factors of the well-conditioned W_K = U diag(s) V^T / sqrt(d)  (kcache configs only)
    U: np.ndarray | None = None
    s: np.ndarray | None = None
    Vt: np.ndarray | None = None


def make_weights(cfg: Config, rng: np.random.Generator) -> Weights:
    d, e = cfg.d, cfg.e
    if cfg.kind == "kcache":
        assert e == d
        s = rng.uniform(0.5, 2.0, size=d)
        U = _orthogonal_from(rng.standard_normal((d, d)))
        V = _orthogonal_from(rng.standard_normal((d, d)))
        W_K = (U * s) @ V.T / np.sqrt(d)
        W_V = rng.standard_normal((d, d)) / np.sqrt(d)
        W_Q = rng.standard_normal((d, d)) / np.sqrt(d)
        return Weights(W_Q, W_K, W_V, U, s, V.T.copy())
    W_K = rng.standard_normal((d, e)) / np.sqrt(d)
    W_V = rng.standard_normal((d, e)) / np.sqrt(d)
    W_Q = rng.standard_normal((d, e)) / np.sqrt(d)
    return Weights(W_Q, W_K, W_V)


# ----------------------------------------------------------------------------------------------
# per-sequence activations
# ----------------------------------------------------------------------------------------------
@dataclasses.dataclass
class Sequence:
    length: int          # rows attended over (<= cfg.T)
    X: np.ndarray        # (length, d) cached-token activations, fp64 (bf16 values if x_pre_rounded)
    x: np.ndarray        # (d,) the fresh token's activation


def draw_sequence(cfg: Config, rng: np.random.Generator, materialize: bool = True) -> Sequence:
    """Draws (len_b, X_b, x_b).  With materialize=False the draws are still consumed (so later
    sequences keep their values) but X is returned as None."""
    if cfg.len_lo > 0:
        length = int(rng.integers(cfg.len_lo, cfg.T, endpoint=True))
    else:
        length = cfg.T
    X = rng.standard_normal((length, cfg.d))
    x = rng.standard_normal(cfg.d)
    if not materialize:
        return Sequence(length, None, x)
    if cfg.x_pre_rounded:
        X = round_through(X, "bf16")
    return Sequence(length, X, x)


def rng_for(cfg: Config) -> np.random.Generator:
    return np.random.default_rng(SEED_BASE + cfg.index)


@dataclasses.dataclass
class Problem:
    cfg: Config
    w: Weights
    seqs: list          # list[Sequence]
    q: np.ndarray       # (B, e) fp64 projected, un-scaled queries  q_b = x_b W_Q

    @property
    def lengths(self) -> np.ndarray:
        return np.array([s.length for s in self.seqs], dtype=np.int32)


def make_problem(cfg: Config, keep: set | None = None) -> Problem:
    """All inputs of one decode step.  `keep`: indices of sequences whose X is retained
    (None = all); the others are drawn and dropped to bound host memory at full sizes."""
    rng = rng_for(cfg)
    w = make_weights(cfg, rng)
    seqs = []
    for b in range(cfg.B):
        sq = draw_sequence(cfg, rng)
        if keep is not None and b not in keep:
            sq = Sequence(sq.length, None, sq.x)
        seqs.append(sq)
    q = np.stack([sq.x @ w.W_Q for sq in seqs])
    return Problem(cfg, w, seqs, q)


def make_w_o(cfg: Config) -> np.ndarray:
    """Output projection W_O ~ N(0, 1/e), (e, d), for the whole-block workloads.  Drawn from a
    stream of its own so that the decode-step inputs above keep their values."""
    rng = np.random.default_rng([SEED_BASE + cfg.index, 1])
    return rng.standard_normal((cfg.e, cfg.d)) / np.sqrt(cfg.e)


def project_cache(X: np.ndarray, W: np.ndarray) -> np.ndarray:
    """Cache construction (the prompt phase, which lies outside the decode path): the rows
    the decode step will read, K = X W_K, as a plain fp64 product."""
    return np.asarray(X, np.float64) @ np.asarray(W, np.float64)


def stress_query(q: np.ndarray, factor: float) -> np.ndarray:
    """Scaled queries: a large factor makes the softmax peaky so that the running-max and
    rescale logic of a streaming softmax is exercised (the plain recipe gives near-uniform p)."""
    return q * factor
