"""Thin ctypes binding over the C ABI declared in include/slim_attention.h.

Argument marshalling only: every step of the decode path runs inside the library's HIP
kernels.  torch is used for device memory and the current stream, nothing else.  There is no
CPU fallback: if the built library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("SLIM_ATTENTION_LIB") or os.path.join(_PKG, "libslim_attention.so")

SLIM_OK = 0
SLIM_F32, SLIM_BF16 = 0, 1
VARIANT_AUTO, VARIANT_GENERIC, VARIANT_FUSED_SPLIT, VARIANT_FUSED = 0, 1, 2, 3
K_ROWMAJOR, K_BANDED = 0, 1       # slim_opts.k_layout
DTYPES = {"f32": SLIM_F32, "bf16": SLIM_BF16}

EXPORTS = ("slim_strerror", "slim_prepare_wkv", "slim_prepare_wkv_nonsquare", "slim_pack_weights", "slim_rope_table", "slim_workspace_bytes",
           "slim_workspace_bytes_xcache", "slim_workspace_bytes_block", "slim_attention_block", "vanilla_attention_block",
           "slim_variant_for", "slim_decode", "vanilla_kv_decode", "slim_decode_xcache", "slim_init", "slim_status",
           "slim_read_probe", "slim_decode_static", "slim_static_scratch_bytes", "slim_band_kcache")
VARIANT_NAMES = {1: "generic", 2: "fused_split", 3: "fused"}


class SlimOpts(ctypes.Structure):
    _fields_ = [
        ("dtype", ctypes.c_int),
        ("seq_lens", ctypes.c_void_p),
        ("seq_lens_host", ctypes.c_void_p),
        ("t_stride", ctypes.c_int64),
        ("workspace", ctypes.c_void_p),
        ("workspace_bytes", ctypes.c_size_t),
        ("stream", ctypes.c_void_p),
        ("variant", ctypes.c_int),
        ("stage_ms", ctypes.POINTER(ctypes.c_float)),
        ("rope_table", ctypes.c_void_p),
        ("wait_budget_us", ctypes.c_int64),
        ("k_layout", ctypes.c_int),
    ]


MAX_STAGES = 8


class SlimError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"{what}: {strerror(code)} ({code})")
        self.code = code


_lib = None


def load():
    """Loads the in-tree library (after torch, so both share one HIP runtime)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is not built; run `python -m paper_2503_05840_amd.build` "
            "(there is no fallback path)")
    import torch  # noqa: F401  (loads libamdhip64 first)
    lib = ctypes.CDLL(LIB_PATH, mode=ctypes.RTLD_GLOBAL)
    vp, ci, cd = ctypes.c_void_p, ctypes.c_int, ctypes.POINTER(ctypes.c_double)
    lib.slim_strerror.restype = ctypes.c_char_p
    lib.slim_strerror.argtypes = [ci]
    lib.slim_prepare_wkv.restype = ci
    lib.slim_prepare_wkv.argtypes = [vp, vp, vp, ci, cd]
    lib.slim_prepare_wkv_nonsquare.restype = ci
    lib.slim_prepare_wkv_nonsquare.argtypes = [vp, vp, vp, ci, ci, cd]
    lib.slim_pack_weights.restype = ci
    lib.slim_pack_weights.argtypes = [vp, vp, ci, ci, ci]
    lib.slim_rope_table.restype = ci
    lib.slim_rope_table.argtypes = [vp, ci, ci, ctypes.c_double]
    lib.slim_workspace_bytes.restype = ctypes.c_size_t
    lib.slim_workspace_bytes.argtypes = [ci, ci, ci, ci, ci]
    lib.slim_workspace_bytes_xcache.restype = ctypes.c_size_t
    lib.slim_workspace_bytes_xcache.argtypes = [ci, ci, ci, ci, ci, ci]
    lib.slim_variant_for.restype = ci
    lib.slim_variant_for.argtypes = [ci, ci, ci, ci, ci]
    op = ctypes.POINTER(SlimOpts)
    lib.slim_decode.restype = ci
    lib.slim_decode.argtypes = [vp, vp, vp, vp, ci, ci, ci, ci, op]
    lib.vanilla_kv_decode.restype = ci
    lib.vanilla_kv_decode.argtypes = [vp, vp, vp, vp, ci, ci, ci, ci, op]
    lib.slim_decode_xcache.restype = ci
    lib.slim_decode_xcache.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, op]
    lib.slim_workspace_bytes_block.restype = ctypes.c_size_t
    lib.slim_workspace_bytes_block.argtypes = [ci, ci, ci, ci, ci]
    lib.slim_attention_block.restype = ci
    lib.slim_attention_block.argtypes = [vp, vp, vp, vp, vp, vp, vp, ci, ci, ci, ci, op]
    lib.vanilla_attention_block.restype = ci
    lib.vanilla_attention_block.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, ci, ci, ci, ci, op]
    lib.slim_init.restype = ci
    lib.slim_init.argtypes = []
    lib.slim_status.restype = ci
    lib.slim_status.argtypes = [vp, vp]
    lib.slim_decode_static.restype = ci
    lib.slim_decode_static.argtypes = [vp, vp, vp, vp, ci, ci, ci, ci, op]
    lib.slim_static_scratch_bytes.restype = ctypes.c_size_t
    lib.slim_static_scratch_bytes.argtypes = []
    lib.slim_band_kcache.restype = ci
    lib.slim_band_kcache.argtypes = [vp, vp, ci, ctypes.c_int64, ci, ci, ci]
    lib.slim_read_probe.restype = ci
    lib.slim_read_probe.argtypes = [vp, ctypes.c_size_t, vp]
    _lib = lib
    return lib


def strerror(code: int) -> str:
    return load().slim_strerror(code).decode()


# ---- host side -------------------------------------------------------------------------------
def slim_prepare_wkv(W_K: np.ndarray, W_V: np.ndarray, allow_illcond: bool = False):
    """W_KV = W_K^{-1} W_V in fp64 on the host.  Returns (W_KV, rcond)."""
    W_K = np.ascontiguousarray(W_K, dtype=np.float64)
    W_V = np.ascontiguousarray(W_V, dtype=np.float64)
    d = W_K.shape[0]
    if W_K.shape != (d, d) or W_V.shape != (d, d):
        raise ValueError("W_K and W_V must be square and of equal size")
    out = np.empty((d, d), dtype=np.float64)
    rcond = ctypes.c_double(0.0)
    rc = load().slim_prepare_wkv(W_K.ctypes.data, W_V.ctypes.data, out.ctypes.data, d, ctypes.byref(rcond))
    if rc != SLIM_OK and not (allow_illcond and rc == -7):
        raise SlimError(rc, "slim_prepare_wkv")
    return out, rcond.value


def slim_prepare_wkv_nonsquare(W_K: np.ndarray, W_V: np.ndarray):
    """W_KV = W_K^T (W_K W_K^T)^{-1} W_V (e x e) for d x e projections, fp64 on the host.
    Returns (W_KV, rcond of W_K W_K^T)."""
    W_K = np.ascontiguousarray(W_K, dtype=np.float64)
    W_V = np.ascontiguousarray(W_V, dtype=np.float64)
    d, e = W_K.shape
    if W_V.shape != (d, e):
        raise ValueError("W_K and W_V must have the same d x e shape")
    out = np.empty((e, e), dtype=np.float64)
    rcond = ctypes.c_double(0.0)
    rc = load().slim_prepare_wkv_nonsquare(W_K.ctypes.data, W_V.ctypes.data, out.ctypes.data, d, e, ctypes.byref(rcond))
    if rc != SLIM_OK:
        raise SlimError(rc, "slim_prepare_wkv_nonsquare")
    return out, rcond.value


def slim_pack_weights(W: np.ndarray, dtype: str) -> np.ndarray:
    """fp64 row-major matrix -> device element type (float32 array or uint16 bf16 bits)."""
    W = np.ascontiguousarray(W, dtype=np.float64)
    rows, cols = W.shape
    out = np.empty((rows, cols), dtype=np.float32 if dtype == "f32" else np.uint16)
    rc = load().slim_pack_weights(W.ctypes.data, out.ctypes.data, rows, cols, DTYPES[dtype])
    if rc != SLIM_OK:
        raise SlimError(rc, "slim_pack_weights")
    return out


def slim_band_kcache(K: np.ndarray, H: int) -> np.ndarray:
    """Host K-cache (B, t_stride, d) row-major -> the banded layout (K_BANDED), same shape and dtype."""
    K = np.ascontiguousarray(K)
    B, t_stride, d = K.shape
    out = np.empty_like(K)
    rc = load().slim_band_kcache(K.ctypes.data, out.ctypes.data, B, t_stride, H, d // H, K.dtype.itemsize)
    if rc != SLIM_OK:
        raise SlimError(rc, "slim_band_kcache")
    return out


def slim_rope_table(T: int, d_k: int, base: float = 10000.0) -> np.ndarray:
    """(T, d_k/2, 2) float32 table of cos / sin(t * theta_j) for opts.rope_table."""
    out = np.empty((T, max(d_k // 2, 0), 2), dtype=np.float32)
    rc = load().slim_rope_table(out.ctypes.data, T, d_k, float(base))
    if rc != SLIM_OK:
        raise SlimError(rc, "slim_rope_table")
    return out


def slim_workspace_bytes(B, H, T, d, dtype: str) -> int:
    return int(load().slim_workspace_bytes(B, H, T, d, DTYPES[dtype]))


def slim_workspace_bytes_xcache(B, H, T, d_model, d_k, dtype: str) -> int:
    return int(load().slim_workspace_bytes_xcache(B, H, T, d_model, d_k, DTYPES[dtype]))


def slim_workspace_bytes_block(B, H, T, d, dtype: str) -> int:
    return int(load().slim_workspace_bytes_block(B, H, T, d, DTYPES[dtype]))


def auto_variant_name(B, H, T, d, dtype: str) -> str:
    """Which implementation SLIM_VARIANT_AUTO resolves to for this shape."""
    return VARIANT_NAMES[int(load().slim_variant_for(B, H, T, d, DTYPES[dtype]))]


# ---- device side -----------------------------------------------------------------------------
def to_device(a: np.ndarray):
    """numpy array -> device tensor; uint16 arrays are bf16 bit patterns."""
    import torch
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def to_host(t) -> np.ndarray:
    """device tensor -> numpy array; bf16 tensors come back as their uint16 bit patterns."""
    import torch
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


SLIM_ERR_TIMEOUT = -10
SLIM_ERR_LAYOUT = -11
STATIC_SCRATCH = 1          # slim_status: the scratch of slim_decode_static


def slim_init():
    rc = load().slim_init()
    if rc != SLIM_OK:
        raise SlimError(rc, "slim_init")


def slim_status(workspace=None) -> int:
    """SLIM_OK or SLIM_ERR_TIMEOUT for the latest fast-path launch on `workspace` (a device tensor, None for
    the library-owned scratch, STATIC_SCRATCH for slim_decode_static's); waits for the current stream."""
    import torch
    ws = workspace if isinstance(workspace, int) or workspace is None else workspace.data_ptr()
    return int(load().slim_status(ws, torch.cuda.current_stream().cuda_stream))


def slim_read_probe(buf) -> None:
    """Plain streaming read of a device tensor (measurement only: the read rate this GPU sustains)."""
    import torch
    rc = load().slim_read_probe(_dev_ptr(buf), buf.numel() * buf.element_size(), torch.cuda.current_stream().cuda_stream)
    if rc != SLIM_OK:
        raise SlimError(rc, "slim_read_probe")


def _opts(dtype, seq_lens, seq_lens_host, t_stride, workspace, variant, stage_ms=None, rope_table=None, wait_budget_us=0,
          k_layout=0):
    import torch
    o = SlimOpts()
    o.dtype = DTYPES[dtype]
    o.seq_lens = seq_lens.data_ptr() if seq_lens is not None else None
    keep = None
    if seq_lens_host is not None:
        keep = np.ascontiguousarray(seq_lens_host, dtype=np.int32)
        o.seq_lens_host = keep.ctypes.data
    o.t_stride = int(t_stride or 0)
    if workspace is not None:
        o.workspace = workspace.data_ptr()
        o.workspace_bytes = workspace.numel() * workspace.element_size()
    o.stream = torch.cuda.current_stream().cuda_stream
    o.variant = int(variant)
    if stage_ms is not None:      # a ctypes float array of MAX_STAGES entries, filled by the call
        o.stage_ms = ctypes.cast(stage_ms, ctypes.POINTER(ctypes.c_float))
    if rope_table is not None:
        o.rope_table = _dev_ptr(rope_table)
    o.wait_budget_us = int(wait_budget_us)
    o.k_layout = int(k_layout)
    return o, keep


def new_stage_buffer():
    """Host buffer for opts.stage_ms (per-kernel milliseconds of one call; measurement only)."""
    return (ctypes.c_float * MAX_STAGES)()


def _dev_ptr(t):
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous device tensor")
    return t.data_ptr()


def slim_decode(q, Kcache, W_KV, out, B, H, T, d, dtype="bf16", seq_lens=None, seq_lens_host=None,
                t_stride=0, workspace=None, variant=VARIANT_AUTO, stage_ms=None, rope_table=None, wait_budget_us=0,
                k_layout=K_ROWMAJOR):
    o, keep = _opts(dtype, seq_lens, seq_lens_host, t_stride, workspace, variant, stage_ms, rope_table, wait_budget_us,
                    k_layout)
    rc = load().slim_decode(_dev_ptr(q), _dev_ptr(Kcache), _dev_ptr(W_KV), _dev_ptr(out), B, H, T, d,
                            ctypes.byref(o))
    if rc != SLIM_OK:
        raise SlimError(rc, "slim_decode")
    return out


def slim_decode_static(q, Kcache, W_KV, out, B, H, T, d, dtype="bf16", seq_lens=None, seq_lens_host=None,
                       t_stride=0, variant=VARIANT_AUTO, rope_table=None, k_layout=K_ROWMAJOR):
    """slim_decode over the library's static device scratch: no allocation inside the call."""
    o, keep = _opts(dtype, seq_lens, seq_lens_host, t_stride, None, variant, None, rope_table, 0, k_layout)
    rc = load().slim_decode_static(_dev_ptr(q), _dev_ptr(Kcache), _dev_ptr(W_KV), _dev_ptr(out), B, H, T, d,
                                   ctypes.byref(o))
    if rc != SLIM_OK:
        raise SlimError(rc, "slim_decode_static")
    return out


def slim_static_scratch_bytes() -> int:
    return int(load().slim_static_scratch_bytes())


def vanilla_kv_decode(q, Kcache, Vcache, out, B, H, T, d, dtype="bf16", seq_lens=None,
                      seq_lens_host=None, t_stride=0, workspace=None, variant=VARIANT_AUTO, stage_ms=None, rope_table=None):
    o, keep = _opts(dtype, seq_lens, seq_lens_host, t_stride, workspace, variant, stage_ms, rope_table)
    rc = load().vanilla_kv_decode(_dev_ptr(q), _dev_ptr(Kcache), _dev_ptr(Vcache), _dev_ptr(out),
                                  B, H, T, d, ctypes.byref(o))
    if rc != SLIM_OK:
        raise SlimError(rc, "vanilla_kv_decode")
    return out


def slim_decode_xcache(q, X, W_K, W_V, out, B, H, T, d_model, d_k, dtype="bf16", seq_lens=None,
                       seq_lens_host=None, t_stride=0, workspace=None, variant=VARIANT_AUTO, stage_ms=None, rope_table=None):
    o, keep = _opts(dtype, seq_lens, seq_lens_host, t_stride, workspace, variant, stage_ms, rope_table)
    rc = load().slim_decode_xcache(_dev_ptr(q), _dev_ptr(X), _dev_ptr(W_K), _dev_ptr(W_V),
                                   _dev_ptr(out), B, H, T, d_model, d_k, ctypes.byref(o))
    if rc != SLIM_OK:
        raise SlimError(rc, "slim_decode_xcache")
    return out


def slim_attention_block(x, W_Q, W_K, W_KV, W_O, Kcache, y, B, H, T, d, dtype="bf16", seq_lens=None,
                         seq_lens_host=None, t_stride=0, workspace=None, variant=VARIANT_AUTO, stage_ms=None,
                         rope_table=None, k_layout=K_ROWMAJOR):
    o, keep = _opts(dtype, seq_lens, seq_lens_host, t_stride, workspace, variant, stage_ms, rope_table, 0, k_layout)
    rc = load().slim_attention_block(_dev_ptr(x), _dev_ptr(W_Q), _dev_ptr(W_K), _dev_ptr(W_KV), _dev_ptr(W_O),
                                     _dev_ptr(Kcache), _dev_ptr(y), B, H, T, d, ctypes.byref(o))
    if rc != SLIM_OK:
        raise SlimError(rc, "slim_attention_block")
    return y


def vanilla_attention_block(x, W_Q, W_K, W_V, W_O, Kcache, Vcache, y, B, H, T, d, dtype="bf16", seq_lens=None,
                            seq_lens_host=None, t_stride=0, workspace=None, variant=VARIANT_AUTO, stage_ms=None,
                            rope_table=None):
    o, keep = _opts(dtype, seq_lens, seq_lens_host, t_stride, workspace, variant, stage_ms, rope_table)
    rc = load().vanilla_attention_block(_dev_ptr(x), _dev_ptr(W_Q), _dev_ptr(W_K), _dev_ptr(W_V), _dev_ptr(W_O),
                                        _dev_ptr(Kcache), _dev_ptr(Vcache), _dev_ptr(y), B, H, T, d, ctypes.byref(o))
    if rc != SLIM_OK:
        raise SlimError(rc, "vanilla_attention_block")
    return y
