"""ctypes binding of the C ABI declared in ``include/spark.h``.

Argument marshalling only: tensors are PyTorch device tensors used as plain device memory
(``data_ptr()``), the stream is the current HIP stream, and all arithmetic happens in the
library's kernels.  There is no fallback: if ``libspark_hip.so`` has not been built the
import of the library fails with an error that says how to build it.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libspark_hip.so")

F32, BF16, FP8_E4M3, INT8 = 0, 1, 2, 3
FILL_ZERO, FILL_NEG_INF = 0, 1
GELU_ERF, GELU_TANH = 0, 1
MAX_BATCH = 64

EXPORTS = (
    "spark_status_string", "spark_version", "spark_normal_quantile", "spark_stat_topk",
    "spark_stat_topk_huber", "spark_stat_topk_huber_backward",
    "spark_stat_topk_shard_stats", "spark_stat_topk_combine_stats", "spark_stat_topk_apply",
    "spark_ffn_workspace_bytes", "spark_ffn_decode", "spark_ffn_decode_layers",
    "spark_ffn_dense_decode", "spark_ffn_dense_decode_layers",
    "spark_ffn_prefill_workspace_bytes", "spark_ffn_prefill",
    "spark_attn_workspace_bytes", "spark_attn_decode", "spark_stat_topk_workspace_bytes",
    "spark_ffn_decode_layers_tuned", "spark_copy_bytes", "spark_ffn_decode_static",
)


class SparkError(RuntimeError):
    def __init__(self, code: int, what: str):
        self.code = code
        super().__init__(f"{what}: spark_status {code} ({status_string(code)})")


class _Layer(ctypes.Structure):
    _fields_ = [
        ("d_model", ctypes.c_int32), ("d_ff", ctypes.c_int32), ("r", ctypes.c_int32),
        ("k", ctypes.c_int32), ("wdtype", ctypes.c_int32), ("gelu", ctypes.c_int32),
        ("k1n", ctypes.c_void_p), ("k2n", ctypes.c_void_p), ("vn", ctypes.c_void_p),
    ]


class _AttnHead(ctypes.Structure):
    _fields_ = [
        ("n_ctx", ctypes.c_int32), ("d_attn", ctypes.c_int32), ("r", ctypes.c_int32),
        ("k", ctypes.c_int32), ("cdtype", ctypes.c_int32), ("group", ctypes.c_int32),
        ("k1c", ctypes.c_void_p), ("k2c", ctypes.c_void_p), ("vc", ctypes.c_void_p),
    ]


class Tuning(ctypes.Structure):
    """``spark_ffn_tuning``: choices pinned for one ``spark_ffn_decode_layers_tuned`` call (0 = automatic)."""
    _fields_ = [
        ("path", ctypes.c_int32), ("phases", ctypes.c_int32), ("rows_per_predict_block", ctypes.c_int32),
        ("neurons_per_gather_block", ctypes.c_int32), ("variant", ctypes.c_int32),
    ]


_lib = None


def load_library():
    """Loads ``libspark_hip.so``; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2506_06644_amd.build` "
            "(there is no CPU or PyTorch fallback)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i64, sz, c_int = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t, ctypes.c_int
    lib.spark_status_string.restype = ctypes.c_char_p
    lib.spark_status_string.argtypes = [c_int]
    lib.spark_version.restype = c_int
    lib.spark_normal_quantile.restype = ctypes.c_double
    lib.spark_normal_quantile.argtypes = [ctypes.c_double]
    lib.spark_stat_topk.restype = c_int
    lib.spark_stat_topk.argtypes = [vp, c_int, i64, i64, i64, i64, c_int, vp, i64, vp, vp, vp, i64, vp]
    lib.spark_stat_topk_huber.restype = c_int
    lib.spark_stat_topk_huber.argtypes = [vp, c_int, i64, i64, i64, i64, ctypes.c_float, vp, i64, vp, vp]
    lib.spark_stat_topk_huber_backward.restype = c_int
    lib.spark_stat_topk_huber_backward.argtypes = [vp, vp, c_int, i64, i64, i64, i64, i64, ctypes.c_float, vp, i64, vp]
    lib.spark_stat_topk_shard_stats.restype = c_int
    lib.spark_stat_topk_shard_stats.argtypes = [vp, c_int, i64, i64, i64, vp, vp]
    lib.spark_stat_topk_combine_stats.restype = c_int
    lib.spark_stat_topk_combine_stats.argtypes = [vp, ctypes.POINTER(i64), i32, i64, i64, vp, vp, vp, vp]
    lib.spark_stat_topk_apply.restype = c_int
    lib.spark_stat_topk_apply.argtypes = [vp, c_int, i64, i64, i64, vp, c_int, vp, i64, vp, vp, i64, vp]
    lib.spark_ffn_workspace_bytes.restype = sz
    lib.spark_ffn_workspace_bytes.argtypes = [i32, i32, i32]
    lib.spark_ffn_decode.restype = c_int
    lib.spark_ffn_decode.argtypes = [ctypes.POINTER(_Layer), vp, c_int, i32, i64, vp, vp, vp, vp, vp, vp,
                                     vp, sz, vp]
    lib.spark_ffn_decode_layers.restype = c_int
    lib.spark_ffn_decode_layers.argtypes = [ctypes.POINTER(_Layer), i32, vp, c_int, i32, i64, vp, vp, vp,
                                            vp, vp, vp, vp, sz, vp]
    lib.spark_ffn_prefill_workspace_bytes.restype = sz
    lib.spark_ffn_prefill_workspace_bytes.argtypes = [i32, i32, i32]
    lib.spark_ffn_prefill.restype = c_int
    lib.spark_ffn_prefill.argtypes = [ctypes.POINTER(_Layer), vp, c_int, i64, i32, i64, vp, vp, vp, vp, vp, vp,
                                      vp, sz, vp]
    lib.spark_ffn_dense_decode.restype = c_int
    lib.spark_ffn_dense_decode.argtypes = [ctypes.POINTER(_Layer), vp, c_int, i32, i64, vp, vp, sz, vp]
    lib.spark_attn_workspace_bytes.restype = sz
    lib.spark_attn_workspace_bytes.argtypes = [i32, i32, i32]
    lib.spark_attn_decode.restype = c_int
    lib.spark_attn_decode.argtypes = [ctypes.POINTER(_AttnHead), i32, vp, c_int, vp, vp, vp, vp, vp, sz, vp]
    lib.spark_ffn_dense_decode_layers.restype = c_int
    lib.spark_ffn_dense_decode_layers.argtypes = [ctypes.POINTER(_Layer), i32, vp, c_int, i32, i64, vp, vp, sz, vp]
    lib.spark_stat_topk_workspace_bytes.restype = sz
    lib.spark_stat_topk_workspace_bytes.argtypes = [i64, i64]
    lib.spark_ffn_decode_layers_tuned.restype = c_int
    lib.spark_ffn_decode_layers_tuned.argtypes = [ctypes.POINTER(_Layer), i32, vp, c_int, i32, i64, vp, vp, vp,
                                                  vp, vp, vp, vp, sz, ctypes.POINTER(Tuning), vp]
    lib.spark_ffn_decode_static.restype = c_int
    lib.spark_ffn_decode_static.argtypes = [ctypes.POINTER(_Layer), vp, c_int, i32, i64, vp, vp, vp, vp, vp, vp, vp]
    lib.spark_copy_bytes.restype = c_int
    lib.spark_copy_bytes.argtypes = [vp, vp, sz, vp]
    _lib = lib
    return lib


def status_string(code: int) -> str:
    return load_library().spark_status_string(int(code)).decode()


def normal_quantile(p: float) -> float:
    return float(load_library().spark_normal_quantile(float(p)))


def ffn_workspace_bytes(d_model: int, d_ff: int, batch: int) -> int:
    return int(load_library().spark_ffn_workspace_bytes(int(d_model), int(d_ff), int(batch)))


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    return -1


def _p(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(rc: int, what: str):
    if rc != 0:
        raise SparkError(rc, what)


def spark_stat_topk(x: torch.Tensor, k: int, fill: int = FILL_ZERO, y: Optional[torch.Tensor] = None,
                    theta: Optional[torch.Tensor] = None, count: Optional[torch.Tensor] = None,
                    idx: Optional[torch.Tensor] = None):
    """Row-wise statistical top-k of ``x[rows, n]`` (device tensor, fp32 or bf16)."""
    rows, n = x.shape
    idx_cap = 0 if idx is None else idx.shape[1]
    rc = load_library().spark_stat_topk(
        _p(x), _dt(x), rows, n, x.stride(0), int(k), int(fill), _p(y),
        0 if y is None else y.stride(0), _p(theta), _p(count), _p(idx), idx_cap, _stream())
    _check(rc, "spark_stat_topk")


def spark_stat_topk_huber(x: torch.Tensor, k: int, delta: float, y: torch.Tensor,
                          theta: Optional[torch.Tensor] = None):
    """``y = Huber(StatTop_k(x); delta) / delta`` row by row (``delta = 0``: StatTop_k itself)."""
    rows, n = x.shape
    rc = load_library().spark_stat_topk_huber(_p(x), _dt(x), rows, n, x.stride(0), int(k), float(delta), _p(y),
                                              y.stride(0), _p(theta), _stream())
    _check(rc, "spark_stat_topk_huber")


def spark_stat_topk_huber_backward(x: torch.Tensor, gy: torch.Tensor, k: int, delta: float, gx: torch.Tensor):
    """``gx = gy . dy/dx`` of :func:`spark_stat_topk_huber`, row by row (same dtype for all three)."""
    rows, n = x.shape
    if gy.dtype != x.dtype or gx.dtype != x.dtype or gy.shape != x.shape or gx.shape != x.shape:
        raise ValueError("x, gy and gx must share shape and dtype")
    rc = load_library().spark_stat_topk_huber_backward(_p(x), _p(gy), _dt(x), rows, n, x.stride(0), gy.stride(0),
                                                       int(k), float(delta), _p(gx), gx.stride(0), _stream())
    _check(rc, "spark_stat_topk_huber_backward")


def spark_stat_topk_shard_stats(x: torch.Tensor, stats: torch.Tensor):
    """(mean, centred sum of squares) of every row of the shard ``x[rows, n_shard]`` into ``stats[rows, 2]``."""
    rows, n = x.shape
    rc = load_library().spark_stat_topk_shard_stats(_p(x), _dt(x), rows, n, x.stride(0), _p(stats), _stream())
    _check(rc, "spark_stat_topk_shard_stats")


def spark_stat_topk_combine_stats(stats: torch.Tensor, n_shard, k: int, theta: torch.Tensor,
                                  mean: Optional[torch.Tensor] = None, std: Optional[torch.Tensor] = None):
    """Thresholds ``theta[rows]`` from the shards' statistics ``stats[n_shards, rows, 2]`` (contiguous)."""
    m, rows, _ = stats.shape
    ns = (ctypes.c_int64 * m)(*[int(v) for v in n_shard])
    rc = load_library().spark_stat_topk_combine_stats(_p(stats), ns, m, rows, int(k), _p(theta), _p(mean), _p(std),
                                                      _stream())
    _check(rc, "spark_stat_topk_combine_stats")


def spark_stat_topk_apply(x: torch.Tensor, theta: torch.Tensor, fill: int = FILL_ZERO, y: Optional[torch.Tensor] = None,
                          count: Optional[torch.Tensor] = None, idx: Optional[torch.Tensor] = None):
    """Soft thresholding of the shard ``x[rows, n_shard]`` with the given per-row thresholds."""
    rows, n = x.shape
    idx_cap = 0 if idx is None else idx.shape[1]
    rc = load_library().spark_stat_topk_apply(_p(x), _dt(x), rows, n, x.stride(0), _p(theta), int(fill), _p(y),
                                              0 if y is None else y.stride(0), _p(count), _p(idx), idx_cap, _stream())
    _check(rc, "spark_stat_topk_apply")


def make_layer(k1n: torch.Tensor, k2n: torch.Tensor, vn: torch.Tensor, k: int, gelu: int = GELU_ERF) -> _Layer:
    d_ff, r = k1n.shape
    d_model = vn.shape[1]
    if k2n.shape != (d_ff, d_model - r) or vn.shape[0] != d_ff:
        raise ValueError("inconsistent weight shapes")
    if not (k1n.is_contiguous() and k2n.is_contiguous() and vn.is_contiguous()):
        raise ValueError("weights must be contiguous neuron-major arrays")
    if not (k1n.dtype == k2n.dtype == vn.dtype):
        raise ValueError("the three weight arrays must share a dtype")
    return _Layer(d_model, d_ff, r, int(k), _dt(k1n), int(gelu), k1n.data_ptr(), k2n.data_ptr(),
                  vn.data_ptr())


def make_workspace(d_model: int, d_ff: int, batch: int, device) -> torch.Tensor:
    return torch.empty(ffn_workspace_bytes(d_model, d_ff, batch), dtype=torch.uint8, device=device)


def spark_ffn_decode(layer: _Layer, q: torch.Tensor, y: torch.Tensor, workspace: torch.Tensor,
                     theta=None, active_count=None, active_idx=None, union_count=None, union_idx=None):
    """One Spark-FFN layer over ``q[batch, d_model]``; ``y[batch, d_model]`` fp32 is overwritten."""
    rc = load_library().spark_ffn_decode(
        ctypes.byref(layer), _p(q), _dt(q), q.shape[0], q.stride(0), _p(y), _p(theta), _p(active_count),
        _p(active_idx), _p(union_count), _p(union_idx), _p(workspace), workspace.numel(), _stream())
    _check(rc, "spark_ffn_decode")


def spark_ffn_decode_static(layer: _Layer, q: torch.Tensor, y: torch.Tensor, theta=None, active_count=None,
                            active_idx=None, union_count=None, union_idx=None):
    """:func:`spark_ffn_decode` for one token on the library's built-in scratch array (no workspace, no
    allocation)."""
    rc = load_library().spark_ffn_decode_static(
        ctypes.byref(layer), _p(q), _dt(q), q.shape[0], q.stride(0), _p(y), _p(theta), _p(active_count),
        _p(active_idx), _p(union_count), _p(union_idx), _stream())
    _check(rc, "spark_ffn_decode_static")


def spark_ffn_decode_layers(layers: Sequence[_Layer], q: torch.Tensor, y: torch.Tensor,
                            workspace: torch.Tensor, theta=None, active_count=None, active_idx=None,
                            union_count=None, union_idx=None):
    """``len(layers)`` independent layers on the same ``q``; outputs carry a leading layer dim."""
    arr = (_Layer * len(layers))(*layers)
    rc = load_library().spark_ffn_decode_layers(
        arr, len(layers), _p(q), _dt(q), q.shape[0], q.stride(0), _p(y), _p(theta), _p(active_count),
        _p(active_idx), _p(union_count), _p(union_idx), _p(workspace), workspace.numel(), _stream())
    _check(rc, "spark_ffn_decode_layers")


def spark_ffn_decode_layers_tuned(layers: Sequence[_Layer], q: torch.Tensor, y: torch.Tensor,
                                  workspace: torch.Tensor, tuning: Optional[Tuning], theta=None, active_count=None,
                                  active_idx=None, union_count=None, union_idx=None):
    """:func:`spark_ffn_decode_layers` with the choices of ``tuning`` pinned (``None`` = automatic)."""
    arr = (_Layer * len(layers))(*layers)
    rc = load_library().spark_ffn_decode_layers_tuned(
        arr, len(layers), _p(q), _dt(q), q.shape[0], q.stride(0), _p(y), _p(theta), _p(active_count),
        _p(active_idx), _p(union_count), _p(union_idx), _p(workspace), workspace.numel(),
        None if tuning is None else ctypes.byref(tuning), _stream())
    _check(rc, "spark_ffn_decode_layers_tuned")


def stat_topk_workspace_bytes(rows: int, n: int) -> int:
    return int(load_library().spark_stat_topk_workspace_bytes(int(rows), int(n)))


def spark_copy_bytes(dst: torch.Tensor, src: torch.Tensor):
    """Plain device copy of ``src`` into ``dst`` (same byte size) by the library's reference copy kernel."""
    n = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != n:
        raise ValueError("dst and src must have the same size in bytes")
    _check(load_library().spark_copy_bytes(_p(dst), _p(src), n, _stream()), "spark_copy_bytes")


def pack_fp8_rows(codes: torch.Tensor, scales: torch.Tensor) -> torch.Tensor:
    """One 8-bit weight array as the library reads it: the codes ``[rows, cols]`` (E4M3 or int8 bytes, as uint8) followed
    by one fp32 scale per row, in one allocation (returned as a flat uint8 tensor)."""
    if codes.dtype != torch.uint8 or scales.dtype != torch.float32 or scales.shape != (codes.shape[0],):
        raise ValueError("codes must be uint8 [rows, cols] and scales float32 [rows]")
    if codes.shape[1] % 16:
        raise ValueError("rows of 8-bit weights must be multiples of 16 elements")
    return torch.cat([codes.contiguous().reshape(-1), scales.contiguous().view(torch.uint8).reshape(-1)])


def make_layer_fp8(k1n: torch.Tensor, k2n: torch.Tensor, vn: torch.Tensor, d_model: int, d_ff: int, r: int, k: int,
                   gelu: int = GELU_ERF, code_dtype: int = FP8_E4M3) -> _Layer:
    """Layer over three arrays packed by :func:`pack_fp8_rows` (the caller keeps them alive);
    ``code_dtype`` says how the bytes read: ``FP8_E4M3`` or ``INT8``."""
    need = (d_ff * (r + 4), d_ff * (d_model - r + 4), d_ff * (d_model + 4))
    for t, n in zip((k1n, k2n, vn), need):
        if t.dtype != torch.uint8 or t.numel() != n or not t.is_contiguous():
            raise ValueError("packed 8-bit weight array of the wrong size")
    return _Layer(int(d_model), int(d_ff), int(r), int(k), int(code_dtype), int(gelu), k1n.data_ptr(), k2n.data_ptr(),
                  vn.data_ptr())


def ffn_prefill_workspace_bytes(d_model: int, d_ff: int, chunk: int) -> int:
    return int(load_library().spark_ffn_prefill_workspace_bytes(int(d_model), int(d_ff), int(chunk)))


def make_prefill_workspace(d_model: int, d_ff: int, chunk: int, device) -> torch.Tensor:
    return torch.empty(ffn_prefill_workspace_bytes(d_model, d_ff, chunk), dtype=torch.uint8, device=device)


def spark_ffn_prefill(layer: _Layer, q: torch.Tensor, chunk: int, y: torch.Tensor, workspace: torch.Tensor,
                      theta=None, active_count=None, active_idx=None, union_count=None, union_idx=None,
                      n_tokens=None):
    """``q[n_tokens, d_model]`` through one layer in chunks of ``chunk`` tokens; ``y[n_tokens, d_model]``
    (``n_tokens`` defaults to all rows of ``q``)."""
    rc = load_library().spark_ffn_prefill(
        ctypes.byref(layer), _p(q), _dt(q), q.shape[0] if n_tokens is None else int(n_tokens), int(chunk), q.stride(0), _p(y), _p(theta),
        _p(active_count), _p(active_idx), _p(union_count), _p(union_idx), _p(workspace), workspace.numel(),
        _stream())
    _check(rc, "spark_ffn_prefill")


def spark_ffn_dense_decode(layer: _Layer, q: torch.Tensor, y: torch.Tensor, workspace: torch.Tensor):
    """Same layer with every K2 / V row read (the dense comparison point)."""
    rc = load_library().spark_ffn_dense_decode(
        ctypes.byref(layer), _p(q), _dt(q), q.shape[0], q.stride(0), _p(y), _p(workspace),
        workspace.numel(), _stream())
    _check(rc, "spark_ffn_dense_decode")


def spark_ffn_dense_decode_layers(layers: Sequence[_Layer], q: torch.Tensor, y: torch.Tensor, workspace: torch.Tensor):
    """``len(layers)`` independent layers, every K2 / V row read; ``y[L, batch, d_model]``."""
    arr = (_Layer * len(layers))(*layers)
    rc = load_library().spark_ffn_dense_decode_layers(
        arr, len(layers), _p(q), _dt(q), q.shape[0], q.stride(0), _p(y), _p(workspace), workspace.numel(), _stream())
    _check(rc, "spark_ffn_dense_decode_layers")


def make_attn_head(k1c: torch.Tensor, k2c: torch.Tensor, vc: torch.Tensor, k: int, group: int = 1) -> _AttnHead:
    """One key / value cache (token-major): k1c[n_ctx, r], k2c[n_ctx, d_attn - r], vc[n_ctx, d_attn]."""
    n_ctx, r = k1c.shape
    d_attn = vc.shape[1]
    if k2c.shape != (n_ctx, d_attn - r) or vc.shape[0] != n_ctx:
        raise ValueError("inconsistent cache shapes")
    if not (k1c.is_contiguous() and k2c.is_contiguous() and vc.is_contiguous()):
        raise ValueError("caches must be contiguous token-major arrays")
    if not (k1c.dtype == k2c.dtype == vc.dtype):
        raise ValueError("the three caches must share a dtype")
    return _AttnHead(n_ctx, d_attn, r, int(k), _dt(k1c), int(group), k1c.data_ptr(), k2c.data_ptr(), vc.data_ptr())


def attn_workspace_bytes(n_heads: int, group: int, n_ctx: int) -> int:
    return int(load_library().spark_attn_workspace_bytes(int(n_heads), int(group), int(n_ctx)))


def spark_attn_decode(heads: Sequence[_AttnHead], q: torch.Tensor, y: torch.Tensor, workspace: torch.Tensor,
                      theta=None, kept_count=None, kept_idx=None):
    """One decode step of Spark attention: q[n_heads, group, d_attn] -> y[n_heads, group, d_attn] (fp32)."""
    if not q.is_contiguous():
        raise ValueError("q must be contiguous")
    arr = (_AttnHead * len(heads))(*heads)
    rc = load_library().spark_attn_decode(arr, len(heads), _p(q), _dt(q), _p(y), _p(theta), _p(kept_count),
                                          _p(kept_idx), _p(workspace), workspace.numel(), _stream())
    _check(rc, "spark_attn_decode")
