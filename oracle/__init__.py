"""CPU oracle of the Spark-FFN sparse decode path -- TEST INFRASTRUCTURE ONLY.

Thin ctypes access to ``spark_oracle.c`` (plain C, double precision, written from the
paper's definitions: Eq.2, Eq.9-11 of arXiv 2506.06644) plus the two set-level steps that
need no arithmetic (union of per-token active sets, batching = one token at a time).

Nothing in the product imports this package; only tests/, the smoke check and the
benchmark's ``cpu_baseline`` leg do.  It imports nothing from the HIP library or its
binding.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "spark_oracle.c")
_LIB = os.path.join(_HERE, "libspark_oracle.so")

FILL_ZERO, FILL_NEG_INF = 0, 1
GELU_ERF, GELU_TANH = 0, 1

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (``-O2 -fopenmp``); returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build()
    lib = ctypes.CDLL(_LIB)
    c_d, c_i64, c_int = ctypes.c_double, ctypes.c_int64, ctypes.c_int
    vp = ctypes.c_void_p
    lib.spark_ref_max_threads.restype = c_int
    lib.spark_ref_normal_cdf.restype = c_d
    lib.spark_ref_normal_cdf.argtypes = [c_d]
    lib.spark_ref_normal_quantile.restype = c_d
    lib.spark_ref_normal_quantile.argtypes = [c_d]
    lib.spark_ref_gelu.restype = c_d
    lib.spark_ref_gelu.argtypes = [c_d, c_int]
    lib.spark_ref_stat_topk.restype = c_int
    lib.spark_ref_stat_topk.argtypes = [vp, c_i64, c_i64, c_int, vp, vp, vp, vp]
    lib.spark_ref_stat_topk_rows.restype = c_int
    lib.spark_ref_stat_topk_rows.argtypes = [vp, c_i64, c_i64, c_i64, c_i64, c_int, vp, c_i64,
                                             vp, vp, vp, vp, c_i64, c_int]
    lib.spark_ref_huber.restype = c_d
    lib.spark_ref_huber.argtypes = [c_d, c_d]
    lib.spark_ref_huber_stat_topk_rows.restype = c_int
    lib.spark_ref_huber_stat_topk_rows.argtypes = [vp, c_i64, c_i64, c_i64, c_d, vp, vp, c_int]
    lib.spark_ref_huber_stat_topk_vjp_rows.restype = c_int
    lib.spark_ref_huber_stat_topk_vjp_rows.argtypes = [vp, vp, c_i64, c_i64, c_i64, c_d, vp, c_int]
    lib.spark_ref_exact_topk.restype = c_int
    lib.spark_ref_exact_topk.argtypes = [vp, c_i64, c_i64, vp]
    lib.spark_ref_exact_topk_rows.restype = c_int
    lib.spark_ref_exact_topk_rows.argtypes = [vp, c_i64, c_i64, c_i64, c_i64, vp, c_int]
    lib.spark_ref_fp8_e4m3_value.restype = c_d
    lib.spark_ref_fp8_e4m3_value.argtypes = [ctypes.c_uint]
    lib.spark_ref_fp8_dequantize_rows.restype = c_int
    lib.spark_ref_fp8_dequantize_rows.argtypes = [vp, vp, c_i64, c_i64, vp]
    lib.spark_ref_int8_dequantize_rows.restype = c_int
    lib.spark_ref_int8_dequantize_rows.argtypes = [vp, vp, c_i64, c_i64, vp]
    lib.spark_ref_spark_ffn.restype = c_int
    lib.spark_ref_spark_ffn.argtypes = [vp, vp, vp, vp, c_i64, c_i64, c_i64, c_i64, c_int, c_int,
                                        vp, vp, vp, vp, vp, vp, vp, vp, c_int]
    lib.spark_ref_softplus.restype = c_d
    lib.spark_ref_softplus.argtypes = [c_d]
    lib.spark_ref_spark_attention.restype = c_int
    lib.spark_ref_spark_attention.argtypes = [vp, vp, vp, vp, c_i64, c_i64, c_i64, c_i64, c_int,
                                              vp, vp, vp, vp, vp, vp, vp]
    lib.spark_ref_spark_attention_on_set.restype = c_int
    lib.spark_ref_spark_attention_on_set.argtypes = [vp, vp, vp, vp, c_i64, c_i64, c_i64, vp, c_i64, vp]
    _lib = lib
    return lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _check(rc: int, what: str):
    if rc != 0:
        names = {1: "null pointer", 2: "bad shape", 3: "k out of range"}
        raise ValueError(f"{what}: {names.get(rc, rc)}")


def max_threads() -> int:
    return int(_load().spark_ref_max_threads())


def normal_cdf(z: float) -> float:
    return float(_load().spark_ref_normal_cdf(float(z)))


def normal_quantile(p: float) -> float:
    """Q(p) of the standard Gaussian (text after Eq.11)."""
    return float(_load().spark_ref_normal_quantile(float(p)))


def gelu(x: float, kind: int = GELU_ERF) -> float:
    return float(_load().spark_ref_gelu(float(x), int(kind)))


@dataclass
class StatTopK:
    y: np.ndarray        # [d] float64, Eq.10 output
    mean: float
    std: float
    z: float             # Q(1 - k/d)
    theta: float         # Eq.11
    idx: np.ndarray      # ascending active indices, int32
    count: int


def stat_topk(x, k: int, fill: int = FILL_ZERO) -> StatTopK:
    """Statistical top-k of one vector (Eq.9-11)."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    if x.ndim != 1:
        raise ValueError("stat_topk takes one vector")
    d = x.shape[0]
    y = np.empty(d, np.float64)
    stats = np.empty(4, np.float64)
    idx = np.empty(max(d, 1), np.int32)
    cnt = np.zeros(1, np.int64)
    rc = _load().spark_ref_stat_topk(_ptr(x), d, int(k), int(fill), _ptr(y), _ptr(stats),
                                     _ptr(idx), _ptr(cnt))
    _check(rc, "stat_topk")
    m = int(cnt[0])
    return StatTopK(y, float(stats[0]), float(stats[1]), float(stats[2]), float(stats[3]),
                    idx[:m].copy(), m)


@dataclass
class StatTopKRows:
    y: np.ndarray | None      # [rows, d] float64
    theta: np.ndarray         # [rows] float64
    std: np.ndarray           # [rows] float64
    count: np.ndarray         # [rows] int64
    idx: np.ndarray | None    # [rows, d] int32, first count[row] entries valid


def stat_topk_rows(x, k: int, fill: int = FILL_ZERO, want_y: bool = True, want_idx: bool = True,
                   threads: int = 0) -> StatTopKRows:
    """Row-wise statistical top-k over x[rows, d]."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    if x.ndim != 2:
        raise ValueError("stat_topk_rows takes a matrix")
    rows, d = x.shape
    y = np.empty((rows, d), np.float64) if want_y else None
    theta = np.empty(rows, np.float64)
    std = np.empty(rows, np.float64)
    count = np.zeros(rows, np.int64)
    idx = np.full((rows, d), -1, np.int32) if want_idx else None
    rc = _load().spark_ref_stat_topk_rows(_ptr(x), rows, d, d, int(k), int(fill), _ptr(y), d,
                                          _ptr(theta), _ptr(std), _ptr(count), _ptr(idx), d,
                                          int(threads))
    _check(rc, "stat_topk_rows")
    return StatTopKRows(y, theta, std, count, idx)


def shard_stats(x_shard):
    """What one device computes on its shard of the activations (Appendix D.2, global variant): the mean
    and the (population) variance of its entries, per row.  x_shard[rows, n_s] -> (mean[rows], var[rows])."""
    x = np.asarray(x_shard, dtype=np.float64)
    if x.ndim != 2 or x.shape[1] < 1:
        raise ValueError("shard_stats takes a matrix with at least one column")
    return x.mean(axis=1), x.var(axis=1)


def combine_shard_stats(ns, means, variances):
    """What every device does with the m (mean, variance) pairs it holds after the exchange (Appendix
    D.2): the mean and the sample standard deviation (ddof = 1, Eq.11's convention) of the whole vector.
    ns[m] entries per shard, means[m][rows], variances[m][rows] -> (mean[rows], std[rows]).
    mean = sum n_s mean_s / N;  sum of squares about it = sum n_s (var_s + (mean_s - mean)^2)."""
    ns = np.asarray(ns, dtype=np.float64)
    means = np.asarray(means, dtype=np.float64)
    variances = np.asarray(variances, dtype=np.float64)
    if means.shape != variances.shape or means.shape[0] != ns.shape[0]:
        raise ValueError("one (mean, variance) pair per shard and row")
    total = ns.sum()
    if total < 2:
        raise ValueError("at least two entries in all")
    mean = (ns[:, None] * means).sum(axis=0) / total
    ss = (ns[:, None] * (variances + (means - mean[None, :]) ** 2)).sum(axis=0)
    return mean, np.sqrt(ss / (total - 1.0))


def stat_topk_sharded(x, k: int, bounds, fill: int = FILL_ZERO, local: bool = False) -> StatTopKRows:
    """Statistical top-k of every row of x[rows, N] whose columns are sharded at `bounds` (column
    offsets 0 = b_0 < b_1 < ... < b_m = N), Appendix D.2.
    Global (local = False): every shard contributes (mean, variance), the combined statistics give one
    threshold theta = mean + std Q(1 - k / N) per row, and each shard is soft-thresholded with it: the
    result is that of the unsharded operator.
    Local (local = True): each shard runs the operator by itself with k' = k n_s / N (k / m for equal
    shards; rounded to the nearest integer, at least 1): no exchange, a different result.  theta and
    std then hold the first shard's values."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    rows, n = x.shape
    bounds = [int(b) for b in bounds]
    if bounds[0] != 0 or bounds[-1] != n or any(b1 <= b0 for b0, b1 in zip(bounds, bounds[1:])):
        raise ValueError("bounds must run from 0 to N, increasing")
    if not 1 <= k <= n - 1:
        raise ValueError("k out of range")
    fillv = -np.inf if fill == FILL_NEG_INF else 0.0
    y = np.empty_like(x)
    count = np.zeros(rows, np.int64)
    idx = np.full((rows, n), -1, np.int32)
    if local:
        theta0 = std0 = None
        for b0, b1 in zip(bounds, bounds[1:]):
            ks = min(max(int(round(k * (b1 - b0) / n)), 1), b1 - b0 - 1)
            part = stat_topk_rows(x[:, b0:b1], ks, fill)
            y[:, b0:b1] = part.y
            for r in range(rows):
                c = int(part.count[r])
                idx[r, count[r]:count[r] + c] = part.idx[r, :c] + b0
                count[r] += c
            if theta0 is None:
                theta0, std0 = part.theta, part.std
        return StatTopKRows(y, theta0, std0, count, idx)
    ns = [b1 - b0 for b0, b1 in zip(bounds, bounds[1:])]
    stats = [shard_stats(x[:, b0:b1]) for b0, b1 in zip(bounds, bounds[1:])]
    mean, std = combine_shard_stats(ns, [s[0] for s in stats], [s[1] for s in stats])
    theta = mean + std * normal_quantile(1.0 - k / n)
    for r in range(rows):
        keep = x[r] > theta[r]
        y[r] = np.where(keep, x[r] - theta[r], fillv)
        where = np.nonzero(keep)[0]
        count[r] = where.size
        idx[r, :where.size] = where
    return StatTopKRows(y, theta, std, count, idx)


def huber(x: float, delta: float) -> float:
    """Huber loss (Section 3.2, Eq.13) for one number."""
    return float(_load().spark_ref_huber(float(x), float(delta)))


def huber_stat_topk(x, k: int, delta: float, threads: int = 0):
    """Huber(StatTop_k(x); delta) / delta (Section 3.2, Eq.14, Theorem 2) of a vector or of every row of a
    matrix; delta = 0 gives StatTop_k itself.  Returns (y, theta) as float64 arrays."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    x2 = x.reshape(1, -1) if x.ndim == 1 else x
    rows, d = x2.shape
    y = np.empty((rows, d), np.float64)
    theta = np.empty(rows, np.float64)
    rc = _load().spark_ref_huber_stat_topk_rows(_ptr(x2), rows, d, int(k), float(delta), _ptr(y), _ptr(theta),
                                                int(threads))
    _check(rc, "huber_stat_topk")
    return (y[0], theta) if x.ndim == 1 else (y, theta)


def huber_stat_topk_vjp(x, gy, k: int, delta: float, threads: int = 0) -> np.ndarray:
    """gx = gy . d(Huber(StatTop_k(x); delta) / delta)/dx, per vector or per row, float64."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    gy = np.ascontiguousarray(gy, dtype=np.float64)
    if gy.shape != x.shape:
        raise ValueError("gy must have the shape of x")
    x2 = x.reshape(1, -1) if x.ndim == 1 else x
    rows, d = x2.shape
    gx = np.empty((rows, d), np.float64)
    rc = _load().spark_ref_huber_stat_topk_vjp_rows(_ptr(x2), _ptr(gy.reshape(rows, d)), rows, d, int(k),
                                                    float(delta), _ptr(gx), int(threads))
    _check(rc, "huber_stat_topk_vjp")
    return gx[0] if x.ndim == 1 else gx


def exact_topk(x, k: int) -> np.ndarray:
    """Indices of the k largest entries by sorting (ties: lower index), ascending."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    idx = np.empty(max(int(k), 1), np.int32)
    rc = _load().spark_ref_exact_topk(_ptr(x), x.shape[0], int(k), _ptr(idx))
    _check(rc, "exact_topk")
    return idx[: int(k)].copy()


def exact_topk_rows(x, k: int, threads: int = 0) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float64)
    rows, d = x.shape
    idx = np.empty((rows, int(k)), np.int32)
    rc = _load().spark_ref_exact_topk_rows(_ptr(x), rows, d, d, int(k), _ptr(idx), int(threads))
    _check(rc, "exact_topk_rows")
    return idx


def fp8_e4m3_value(code: int) -> float:
    """Value of one OCP E4M3 code (0..255)."""
    return float(_load().spark_ref_fp8_e4m3_value(int(code)))


def fp8_dequantize_rows(codes, scales) -> np.ndarray:
    """float32 weights ``scales[row] * value(codes[row, c])`` of a matrix of E4M3 codes (uint8)."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    scales = np.ascontiguousarray(scales, dtype=np.float32)
    rows, cols = codes.shape
    if scales.shape != (rows,):
        raise ValueError("one scale per row")
    out = np.empty((rows, cols), np.float32)
    _check(_load().spark_ref_fp8_dequantize_rows(_ptr(codes), _ptr(scales), rows, cols, _ptr(out)), "fp8_dequantize_rows")
    return out


def int8_dequantize_rows(codes, scales) -> np.ndarray:
    """float32 weights ``scales[row] * codes[row, c]`` of a matrix of signed 8-bit codes."""
    codes = np.ascontiguousarray(codes).view(np.int8)
    scales = np.ascontiguousarray(scales, dtype=np.float32)
    rows, cols = codes.shape
    if scales.shape != (rows,):
        raise ValueError("one scale per row")
    out = np.empty((rows, cols), np.float32)
    _check(_load().spark_ref_int8_dequantize_rows(_ptr(codes), _ptr(scales), rows, cols, _ptr(out)), "int8_dequantize_rows")
    return out


@dataclass
class SparkFFN:
    y: np.ndarray        # [d_model] float64
    s: np.ndarray        # [d_ff] predictor scores
    a: np.ndarray        # [d_ff] StatTop_k(s)
    u: np.ndarray        # [d_ff] GELU(a) * (K2^T q[r:])
    mean: float
    std: float
    z: float
    theta: float
    idx: np.ndarray      # ascending active set
    count: int
    macs: tuple          # multiply-adds spent on (K1, K2, V)


def spark_ffn(k1n, k2n, vn, q, k: int, gelu_kind: int = GELU_ERF, skip_inactive: bool = False,
              threads: int = 0) -> SparkFFN:
    """One Spark-FFN layer for one token (Eq.2); weights neuron-major float32 arrays."""
    k1n = np.ascontiguousarray(k1n, dtype=np.float32)
    k2n = np.ascontiguousarray(k2n, dtype=np.float32)
    vn = np.ascontiguousarray(vn, dtype=np.float32)
    q = np.ascontiguousarray(q, dtype=np.float32)
    d_ff, r = k1n.shape
    d_model = vn.shape[1]
    if k2n.shape != (d_ff, d_model - r) or vn.shape[0] != d_ff or q.shape != (d_model,):
        raise ValueError("spark_ffn: inconsistent shapes")
    y = np.empty(d_model, np.float64)
    s = np.empty(d_ff, np.float64)
    a = np.empty(d_ff, np.float64)
    u = np.empty(d_ff, np.float64)
    stats = np.empty(4, np.float64)
    idx = np.empty(d_ff, np.int32)
    cnt = np.zeros(1, np.int64)
    macs = np.zeros(3, np.int64)
    rc = _load().spark_ref_spark_ffn(_ptr(k1n), _ptr(k2n), _ptr(vn), _ptr(q), d_model, d_ff, r,
                                     int(k), int(gelu_kind), int(bool(skip_inactive)), _ptr(y),
                                     _ptr(s), _ptr(a), _ptr(u), _ptr(stats), _ptr(idx),
                                     _ptr(cnt), _ptr(macs), int(threads))
    _check(rc, "spark_ffn")
    m = int(cnt[0])
    return SparkFFN(y, s, a, u, float(stats[0]), float(stats[1]), float(stats[2]),
                    float(stats[3]), idx[:m].copy(), m, tuple(int(v) for v in macs))


def spark_ffn_batch(k1n, k2n, vn, q, k: int, gelu_kind: int = GELU_ERF,
                    skip_inactive: bool = True, threads: int = 0):
    """Batch of tokens: every token is evaluated on its own (Appendix B: individual masks
    decide the computation); the union of the active sets only says which rows a batched
    kernel has to load and never changes any y_b.  Returns (list of SparkFFN, union idx)."""
    q = np.asarray(q, dtype=np.float32)
    outs = [spark_ffn(k1n, k2n, vn, q[b], k, gelu_kind, skip_inactive, threads)
            for b in range(q.shape[0])]
    return outs, union_of([o.idx for o in outs])


@dataclass
class SparkAttention:
    y: np.ndarray        # [d_attn] float64
    s: np.ndarray        # [n_ctx] predictor scores
    p: np.ndarray        # [n_ctx] softmax over the kept keys (0 elsewhere)
    g: np.ndarray        # [n_ctx] softplus(K2^T q[r:])
    mean: float
    std: float
    z: float
    theta: float         # -inf when n_ctx <= k (every key kept)
    idx: np.ndarray      # ascending kept keys
    count: int


def softplus(x: float) -> float:
    return float(_load().spark_ref_softplus(float(x)))


def spark_attention(k1c, k2c, vc, q, k: int, skip_inactive: bool = False) -> SparkAttention:
    """One head of Spark attention for one query (Eq.7); caches token-major float32 arrays
    k1c[n_ctx, r], k2c[n_ctx, d_attn - r], vc[n_ctx, d_attn]."""
    k1c = np.ascontiguousarray(k1c, dtype=np.float32)
    k2c = np.ascontiguousarray(k2c, dtype=np.float32)
    vc = np.ascontiguousarray(vc, dtype=np.float32)
    q = np.ascontiguousarray(q, dtype=np.float32)
    n_ctx, r = k1c.shape
    d_attn = vc.shape[1]
    if k2c.shape != (n_ctx, d_attn - r) or vc.shape[0] != n_ctx or q.shape != (d_attn,):
        raise ValueError("spark_attention: inconsistent shapes")
    y = np.empty(d_attn, np.float64)
    s = np.empty(n_ctx, np.float64)
    p = np.empty(n_ctx, np.float64)
    g = np.empty(n_ctx, np.float64)
    stats = np.empty(4, np.float64)
    idx = np.empty(n_ctx, np.int32)
    cnt = np.zeros(1, np.int64)
    rc = _load().spark_ref_spark_attention(_ptr(k1c), _ptr(k2c), _ptr(vc), _ptr(q), n_ctx, d_attn, r,
                                           int(k), int(bool(skip_inactive)), _ptr(y), _ptr(s), _ptr(p),
                                           _ptr(g), _ptr(stats), _ptr(idx), _ptr(cnt))
    _check(rc, "spark_attention")
    m = int(cnt[0])
    return SparkAttention(y, s, p, g, float(stats[0]), float(stats[1]), float(stats[2]),
                          float(stats[3]), idx[:m].copy(), m)


def spark_attention_on_set(k1c, k2c, vc, q, kept) -> np.ndarray:
    """Eq.7 evaluated on a given kept set (softmax over exactly those keys): y[d_attn] float64."""
    k1c = np.ascontiguousarray(k1c, dtype=np.float32)
    k2c = np.ascontiguousarray(k2c, dtype=np.float32)
    vc = np.ascontiguousarray(vc, dtype=np.float32)
    q = np.ascontiguousarray(q, dtype=np.float32)
    kept = np.ascontiguousarray(kept, dtype=np.int32)
    n_ctx, r = k1c.shape
    d_attn = vc.shape[1]
    if k2c.shape != (n_ctx, d_attn - r) or vc.shape[0] != n_ctx or q.shape != (d_attn,):
        raise ValueError("spark_attention_on_set: inconsistent shapes")
    y = np.empty(d_attn, np.float64)
    rc = _load().spark_ref_spark_attention_on_set(_ptr(k1c), _ptr(k2c), _ptr(vc), _ptr(q), n_ctx, d_attn, r,
                                                  _ptr(kept), kept.shape[0], _ptr(y))
    _check(rc, "spark_attention_on_set")
    return y


def union_of(index_sets) -> np.ndarray:
    """Ascending union of active index sets."""
    u = set()
    for s in index_sets:
        u.update(int(i) for i in s)
    return np.array(sorted(u), dtype=np.int32)
