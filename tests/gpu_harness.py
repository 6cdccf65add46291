"""Shared plumbing of the GPU parity tests: seeded problem -> device buffers -> library
call -> comparison with the fp64 oracle.  Not a test module itself."""
from __future__ import annotations

import os
import sys

import numpy as np

from oracle import mha_oracle as orc
from paper_2503_05840_amd import binding, synth

orc_project = orc.project

TOL = {"f32": 1e-4, "bf16": 2e-2}     # max norm-wise relative error per head vector


_LOG = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "gpurun_out")


def say(*a):
    """Progress line, flushed before the GPU step it names; mirrored to parity.log in the scratch
    output folder when that folder exists."""
    print(*a, flush=True)
    if os.path.isdir(_LOG):
        with open(os.path.join(_LOG, "parity.log"), "a") as f:
            f.write(" ".join(str(x) for x in a) + "\n")


to_device = binding.to_device


def head_rel_err(out: np.ndarray, ref: np.ndarray, H: int) -> float:
    """max over (b, h) of ||out - ref||_inf / ||ref||_inf on the head's d_k outputs."""
    B, e = ref.shape
    o = out.reshape(B, H, e // H).astype(np.float64)
    r = ref.reshape(B, H, e // H)
    num = np.abs(o - r).max(axis=2)
    den = np.abs(r).max(axis=2)
    return float((num / den).max())


def unband(Kb: np.ndarray, H: int) -> np.ndarray:
    """Banded cache (B, t_stride, d) back to row-major: the inverse of slim_band_kcache, as index shuffling."""
    B, ts, d = Kb.shape
    return np.ascontiguousarray(Kb.reshape(B, ts // 32, H, 32, d // H).transpose(0, 1, 3, 2, 4)).reshape(B, ts, d)


class KCase:
    """A K-cache problem resident on the device, with its oracle result.

    oracle_seqs: sequences the fp64 oracle is evaluated on (None = all).  For the others the
    cache rows are still built from the same seeded X (in fp32, which is faster), so the kernels
    see the full batch; only the comparison is sampled."""

    def __init__(self, cfg: synth.Config, q_scale: float = 1.0, t_stride: int = 0, lens=None,
                 oracle_seqs=None, need_v=True, rope_base=None):
        import torch
        self.cfg = cfg
        self.rope_base = rope_base        # keys carry rotary positions (row t at position t)
        keep = None
        p = synth.make_problem(cfg)
        self.p = p
        B, T, d = cfg.B, cfg.T, cfg.d
        self.lens = np.array(lens, dtype=np.int32) if lens is not None else p.lengths
        ts = t_stride or T
        el = np.float32 if cfg.dtype == "f32" else np.uint16
        Kh = np.zeros((B, ts, d), dtype=el)
        Vh = np.zeros((B, ts, d), dtype=el) if need_v else None
        Krh = np.zeros((B, ts, d), dtype=el) if (need_v and rope_base) else None   # rotated keys, for the vanilla kernel
        self.kv64 = {}
        W_K32 = W_V32 = None
        for b, sq in enumerate(p.seqs):
            n = int(self.lens[b])
            X = sq.X[:n]
            if oracle_seqs is None or b in oracle_seqs:
                K = orc_project(X, p.w.W_K)
                V = orc_project(X, p.w.W_V)
                self.kv64[b] = (K, V)
                Kh[b, :n] = synth.to_storage(K, cfg.dtype)
                if need_v:
                    Vh[b, :n] = synth.to_storage(V, cfg.dtype)
                if Krh is not None:
                    Krh[b, :n] = synth.to_storage(orc.rope_encode(K, cfg.H, np.arange(n), rope_base), cfg.dtype)
            else:
                if W_K32 is None:
                    W_K32, W_V32 = p.w.W_K.astype(np.float32), p.w.W_V.astype(np.float32)
                X32 = X.astype(np.float32)
                K32 = X32 @ W_K32
                Kh[b, :n] = synth.to_storage(K32, cfg.dtype)
                if need_v:
                    Vh[b, :n] = synth.to_storage(X32 @ W_V32, cfg.dtype)
                if Krh is not None:
                    Krh[b, :n] = synth.to_storage(orc.rope_encode(K32, cfg.H, np.arange(n), rope_base), cfg.dtype)
            sq.X = None
        self.oracle_rows = sorted(self.kv64)
        wkv, self.rcond = binding.slim_prepare_wkv(p.w.W_K, p.w.W_V)
        self.t_stride = ts
        self.K = to_device(Kh)
        self.V = to_device(Vh) if need_v else None
        self.K_rot = to_device(Krh) if Krh is not None else None
        self.rope_table = to_device(binding.slim_rope_table(T, cfg.d_k, rope_base)) if rope_base else None
        self.Wkv = to_device(binding.slim_pack_weights(wkv, cfg.dtype))
        self.lens_dev = torch.from_numpy(self.lens).cuda()
        self.ragged = bool((self.lens != T).any())
        self.set_query_scale(q_scale)

    def set_query_scale(self, q_scale: float):
        """(Re)computes the oracle for queries scaled by q_scale from the stored fp64 K and V."""
        c = self.cfg
        self.q64 = self.p.q * q_scale
        self.q = to_device(self.q64.astype(np.float32))
        self.ref = np.full((c.B, c.d), np.nan)
        for b, (K, V) in self.kv64.items():
            if self.rope_base:
                self.ref[b] = orc.vanilla_decode_rope(self.q64[b], K, V, c.H, self.rope_base)
            else:
                self.ref[b] = orc.vanilla_decode(self.q64[b], K, V, c.H)
        return self

    def _kw(self, **kw):
        d = dict(dtype=self.cfg.dtype, t_stride=self.t_stride)
        if self.ragged:
            d.update(seq_lens=self.lens_dev, seq_lens_host=self.lens)
        d.update(kw)
        return d

    def banded_cache(self):
        """The same cache in the banded layout (bands of 32 rows, head-major inside a band), on the device."""
        if getattr(self, "K_banded", None) is None:
            self.K_banded = to_device(binding.slim_band_kcache(binding.to_host(self.K), self.cfg.H))
        return self.K_banded

    def run_slim(self, banded=False, **kw):
        import torch
        c = self.cfg
        out = torch.full((c.B, c.d), float("nan"), device="cuda", dtype=torch.float32)
        if self.rope_table is not None:
            kw.setdefault("rope_table", self.rope_table)
        K = self.K
        if banded:
            K = self.banded_cache()
            kw["k_layout"] = binding.K_BANDED
        binding.slim_decode(self.q, K, self.Wkv, out, c.B, c.H, c.T, c.d, **self._kw(**kw))
        torch.cuda.synchronize()
        return out.cpu().numpy()

    def run_vanilla(self, **kw):
        import torch
        c = self.cfg
        out = torch.full((c.B, c.d), float("nan"), device="cuda", dtype=torch.float32)
        Kc = self.K_rot if self.rope_base else self.K       # a vanilla cache stores the rotated keys
        binding.vanilla_kv_decode(self.q, Kc, self.V, out, c.B, c.H, c.T, c.d, **self._kw(**kw))
        torch.cuda.synchronize()
        return out.cpu().numpy()

    def err(self, out):
        rows = self.oracle_rows
        assert np.isfinite(out).all(), "non-finite output"
        return head_rel_err(out[rows], self.ref[rows], self.cfg.H)


class XCase:
    """An X-cache problem (projection width e > d_model) on the device, with its oracle."""

    def __init__(self, cfg: synth.Config, oracle_seqs=None, q_scale: float = 1.0, lens=None, oracle_sees_rounded_weights=False):
        """oracle_sees_rounded_weights: stress cases beyond the five configs whose scores are so peaky that the
        storage rounding of W_K alone exceeds the tolerance; the oracle is then given the weights as stored
        (rounded to the cache dtype), so that what is tested is the streaming logic, not the rounding."""
        self.cfg = cfg
        p = synth.make_problem(cfg)
        self.p = p
        B, T, d = cfg.B, cfg.T, cfg.d
        self.lens = None if lens is None else np.asarray(lens, dtype=np.int32)
        if oracle_sees_rounded_weights:
            p.w.W_K = synth.round_through(p.w.W_K, cfg.dtype)
            p.w.W_V = synth.round_through(p.w.W_V, cfg.dtype)
        q64 = p.q * q_scale
        Xh = np.zeros((B, T, d), dtype=np.uint16 if cfg.dtype == "bf16" else np.float32)
        self.ref = np.full((B, cfg.e), np.nan)
        for b, sq in enumerate(p.seqs):
            Xh[b] = synth.to_storage(sq.X, cfg.dtype)
            if oracle_seqs is None or b in oracle_seqs:
                n = T if self.lens is None else int(self.lens[b])
                self.ref[b] = orc.vanilla_decode_from_x(q64[b], sq.X[:n], p.w.W_K, p.w.W_V, cfg.H)
        self.oracle_rows = [b for b in range(B) if not np.isnan(self.ref[b]).any()]
        self.q = to_device(q64.astype(np.float32))
        self.X = to_device(Xh)
        self.Wk = to_device(binding.slim_pack_weights(p.w.W_K, cfg.dtype))
        self.Wv = to_device(binding.slim_pack_weights(p.w.W_V, cfg.dtype))

    def run(self, **kw):
        import torch
        c = self.cfg
        if self.lens is not None:
            kw.setdefault("seq_lens", torch.from_numpy(self.lens).cuda())
            kw.setdefault("seq_lens_host", self.lens)
        out = torch.full((c.B, c.e), float("nan"), device="cuda", dtype=torch.float32)
        binding.slim_decode_xcache(self.q, self.X, self.Wk, self.Wv, out, c.B, c.H, c.T, c.d, c.d_k,
                                   dtype=c.dtype, **kw)
        torch.cuda.synchronize()
        return out.cpu().numpy()

    def err(self, out):
        rows = self.oracle_rows
        assert np.isfinite(out).all(), "non-finite output"
        return head_rel_err(out[rows], self.ref[rows], self.cfg.H)


def row_rel_err(out: np.ndarray, ref: np.ndarray) -> float:
    """max over rows of ||out - ref||_inf / ||ref||_inf."""
    return float((np.abs(out.astype(np.float64) - ref).max(axis=1) / np.abs(ref).max(axis=1)).max())


class BlockCase:
    """One generated token per sequence through the whole attention block: the config's lengths
    count the rows after the append, so the caches hold lengths[b] - 1 old rows and the kernels
    write row lengths[b] - 1.  q_gain scales W_Q (peakier weights)."""

    def __init__(self, cfg: synth.Config, rope_base=None, q_gain: float = 1.0, t_stride: int = 0):
        import torch
        self.cfg, self.rope_base = cfg, rope_base
        p = synth.make_problem(cfg)
        B, T, d = cfg.B, cfg.T, cfg.d
        W_O = synth.make_w_o(cfg)
        W_Q = p.w.W_Q * q_gain
        self.lens = p.lengths
        ts = self.t_stride = t_stride or T
        el = np.float32 if cfg.dtype == "f32" else np.uint16
        hole = np.float32("nan") if cfg.dtype == "f32" else np.uint16(0x7FC0)     # NaN where the new row goes
        Kh = np.full((B, ts, d), hole, dtype=el)
        Krh = np.full((B, ts, d), hole, dtype=el)
        Vh = np.full((B, ts, d), hole, dtype=el)
        self.ref = np.empty((B, d))
        self.k_new = np.empty((B, d))
        self.v_new = np.empty((B, d))
        for b, sq in enumerate(p.seqs):
            n = int(self.lens[b]) - 1
            K = orc_project(sq.X[:n], p.w.W_K)
            V = orc_project(sq.X[:n], p.w.W_V)
            self.ref[b], self.k_new[b], self.v_new[b] = orc.attention_block(
                sq.x, K, V, W_Q, p.w.W_K, p.w.W_V, W_O, cfg.H, rope_base)
            Kh[b, :n] = synth.to_storage(K, cfg.dtype)
            Vh[b, :n] = synth.to_storage(V, cfg.dtype)
            Krh[b, :n] = synth.to_storage(orc.rope_encode(K, cfg.H, np.arange(n), rope_base), cfg.dtype) if rope_base else Kh[b, :n]
            if rope_base:                                  # what a vanilla cache stores for the new token
                self.k_new_rot = getattr(self, "k_new_rot", np.empty((B, d)))
                self.k_new_rot[b] = orc.rope_encode(self.k_new[b][None, :], cfg.H, [n], rope_base)[0]
        wkv, _ = binding.slim_prepare_wkv(p.w.W_K, p.w.W_V)
        pack = lambda W: to_device(binding.slim_pack_weights(W, cfg.dtype))
        self.Wq, self.Wk, self.Wv, self.Wo, self.Wkv = pack(W_Q), pack(p.w.W_K), pack(p.w.W_V), pack(W_O), pack(wkv)
        self.K, self.K_rot, self.V = to_device(Kh), to_device(Krh), to_device(Vh)
        self.x = to_device(np.stack([sq.x for sq in p.seqs]).astype(np.float32))
        self.lens_dev = torch.from_numpy(self.lens).cuda()
        self.rope_table = to_device(binding.slim_rope_table(T, cfg.d_k, rope_base)) if rope_base else None

    def _kw(self, **kw):
        d = dict(dtype=self.cfg.dtype, t_stride=self.t_stride, seq_lens=self.lens_dev, seq_lens_host=self.lens)
        if self.rope_table is not None:
            d["rope_table"] = self.rope_table
        d.update(kw)
        return d

    def _new_rows(self, cache):
        """The rows the call wrote, as fp64 (B, d)."""
        import torch
        idx = torch.from_numpy(self.lens.astype(np.int64) - 1).cuda()
        rows = cache[torch.arange(self.cfg.B, device="cuda"), idx]
        return rows.float().cpu().numpy().astype(np.float64)

    def run_slim(self, banded=False, **kw):
        import torch
        c = self.cfg
        y = torch.full((c.B, c.d), float("nan"), device="cuda", dtype=torch.float32)
        K = self.K
        if banded:       # the cache (with its hole) in the banded layout; the appended row is read back from there
            K = to_device(binding.slim_band_kcache(binding.to_host(self.K), c.H))
            kw["k_layout"] = binding.K_BANDED
        binding.slim_attention_block(self.x, self.Wq, self.Wk, self.Wkv, self.Wo, K, y, c.B, c.H, c.T, c.d,
                                     **self._kw(**kw))
        torch.cuda.synchronize()
        if banded:
            K = to_device(unband(binding.to_host(K), c.H))
        return y.cpu().numpy(), self._new_rows(K)

    def run_vanilla(self, **kw):
        import torch
        c = self.cfg
        y = torch.full((c.B, c.d), float("nan"), device="cuda", dtype=torch.float32)
        binding.vanilla_attention_block(self.x, self.Wq, self.Wk, self.Wv, self.Wo, self.K_rot, self.V, y,
                                        c.B, c.H, c.T, c.d, **self._kw(**kw))
        torch.cuda.synchronize()
        return y.cpu().numpy(), self._new_rows(self.K_rot), self._new_rows(self.V)


class NonSquareCase:
    """Non-square projections, option 1: W_K and W_V are d x e (e > d), the cache holds the e-wide
    keys K = X W_K, and W_KV (e x e) comes from the right inverse of W_K.  The decode step is the
    ordinary slim_decode with its width set to e."""

    def __init__(self, cfg: synth.Config, q_scale: float = 1.0):
        assert cfg.kind == "xcache" and cfg.e > cfg.d
        self.cfg = cfg
        p = synth.make_problem(cfg)
        B, T, e = cfg.B, cfg.T, cfg.e
        q64 = p.q * q_scale
        Kh = np.zeros((B, T, e), dtype=np.uint16 if cfg.dtype == "bf16" else np.float32)
        Vh = np.zeros_like(Kh)
        self.ref = np.empty((B, e))
        for b, sq in enumerate(p.seqs):
            K, V = orc_project(sq.X, p.w.W_K), orc_project(sq.X, p.w.W_V)
            Kh[b], Vh[b] = synth.to_storage(K, cfg.dtype), synth.to_storage(V, cfg.dtype)
            self.ref[b] = orc.vanilla_decode(q64[b], K, V, cfg.H)
        wkv, self.rcond = binding.slim_prepare_wkv_nonsquare(p.w.W_K, p.w.W_V)
        self.q = to_device(q64.astype(np.float32))
        self.K, self.V = to_device(Kh), to_device(Vh)
        self.Wkv = to_device(binding.slim_pack_weights(wkv, cfg.dtype))

    def run_slim(self, **kw):
        import torch
        c = self.cfg
        out = torch.full((c.B, c.e), float("nan"), device="cuda", dtype=torch.float32)
        binding.slim_decode(self.q, self.K, self.Wkv, out, c.B, c.H, c.T, c.e, dtype=c.dtype, **kw)
        torch.cuda.synchronize()
        return out.cpu().numpy()

    def run_vanilla(self):
        import torch
        c = self.cfg
        out = torch.full((c.B, c.e), float("nan"), device="cuda", dtype=torch.float32)
        binding.vanilla_kv_decode(self.q, self.K, self.V, out, c.B, c.H, c.T, c.e, dtype=c.dtype)
        torch.cuda.synchronize()
        return out.cpu().numpy()

    def err(self, out):
        assert np.isfinite(out).all(), "non-finite output"
        return head_rel_err(out, self.ref, self.cfg.H)
