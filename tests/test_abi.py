"""The C-ABI library loads, exports every symbol include/spark.h declares, and rejects
invalid calls on the host before anything is launched (no GPU needed)."""
import ctypes
import os
import re

import pytest

from paper_2506_06644_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "spark.h")).read()
    declared = set(re.findall(r"\b(spark_[a-z_0-9]+)\s*\(", header))
    declared -= {"spark_status", "spark_dtype", "spark_fill", "spark_gelu", "spark_ffn_layer"}
    assert declared == set(binding.EXPORTS)
    lib = binding.load_library()
    for name in declared:
        assert hasattr(lib, name), name
    assert lib.spark_version() == 100


def test_status_strings():
    for code in range(8):
        assert binding.status_string(code) not in ("", "unknown status")
    assert binding.status_string(99) == "unknown status"


def test_library_quantile_agrees_with_statistics_module():
    import statistics
    nd = statistics.NormalDist()
    for p in [1e-9, 0.001, 0.08, 0.5, 0.7, 1 - 737 / 9216, 0.999999]:
        assert binding.normal_quantile(p) == pytest.approx(nd.inv_cdf(p), rel=1e-12, abs=1e-13)
    assert binding.normal_quantile(0.0) == float("-inf") and binding.normal_quantile(1.0) == float("inf")
    assert binding.normal_quantile(2.0) != binding.normal_quantile(2.0)


def _layer(d_model=256, d_ff=1024, r=128, k=82, wd=binding.BF16, gelu=0, k1=0x1000, k2=0x2000, v=0x3000):
    return binding._Layer(d_model, d_ff, r, k, wd, gelu, k1, k2, v)


def _decode(layer, q=0x4000, qd=binding.BF16, batch=1, ldq=256, y=0x5000, ws=0x10000, ws_bytes=None):
    lib = binding.load_library()
    if ws_bytes is None:
        ws_bytes = binding.ffn_workspace_bytes(layer.d_model, layer.d_ff, max(1, min(batch, 64)))
    vp = ctypes.c_void_p
    return lib.spark_ffn_decode(ctypes.byref(layer), vp(q), qd, batch, ldq, vp(y), None, None, None, None,
                                None, vp(ws), ws_bytes, None)


def test_decode_rejects_bad_arguments_before_launch():
    # every call below carries fake (never dereferenced) device addresses
    assert _decode(_layer(k1=0)) == 1                        # NULL weights
    assert _decode(_layer(), q=0) == 1
    assert _decode(_layer(), y=0) == 1
    assert _decode(_layer(d_ff=1)) == 2
    assert _decode(_layer(r=0)) == 2
    assert _decode(_layer(r=256)) == 2
    assert _decode(_layer(), batch=0) == 2
    assert _decode(_layer(), batch=65) == 2
    assert _decode(_layer(), ldq=128) == 2
    assert _decode(_layer(k=0)) == 3
    assert _decode(_layer(k=1024)) == 3
    assert _decode(_layer(wd=7)) == 4
    assert _decode(_layer(gelu=5)) == 4
    assert _decode(_layer(), qd=9) == 4
    assert _decode(_layer(r=100)) == 5                       # 200-byte rows
    assert _decode(_layer(k1=0x1004)) == 5
    assert _decode(_layer(), q=0x4002) == 5
    assert _decode(_layer(), ws=0) == 6
    assert _decode(_layer(), ws=0x10010) == 6
    assert _decode(_layer(), ws_bytes=1024) == 6


def test_stat_topk_rejects_bad_arguments_before_launch():
    lib = binding.load_library()
    vp = ctypes.c_void_p

    def call(x=0x1000, dt=0, rows=4, n=64, ldx=64, k=5, fill=0, y=0x2000, ldy=64, cap=0):
        return lib.spark_stat_topk(vp(x), dt, rows, n, ldx, k, fill, vp(y), ldy, None, None, None, cap, None)

    assert call(x=0) == 1
    assert call(n=1) == 2
    assert call(rows=-1) == 2
    assert call(ldx=60) == 2
    assert call(ldy=32) == 2
    assert call(k=0) == 3 and call(k=64) == 3
    assert call(dt=3) == 4 and call(fill=2) == 4
    assert call(x=0x1008) == 5
    assert call(ldx=66, ldy=66) == 5
    assert call(rows=0) == 0                                  # empty input: nothing to do


def test_workspace_query():
    assert binding.ffn_workspace_bytes(2304, 9216, 1) > 9216 * 4 * 4
    assert binding.ffn_workspace_bytes(2304, 9216, 64) > binding.ffn_workspace_bytes(2304, 9216, 1)
    assert binding.ffn_workspace_bytes(2304, 9216, 0) == 0
    assert binding.ffn_workspace_bytes(2304, 9216, 65) == 0


def test_huber_entries_reject_bad_arguments_before_launch():
    lib = binding.load_library()
    vp = ctypes.c_void_p

    def fwd(x=0x1000, dt=0, rows=4, n=64, ldx=64, k=5, delta=0.25, y=0x2000, ldy=64):
        return lib.spark_stat_topk_huber(vp(x), dt, rows, n, ldx, k, delta, vp(y), ldy, None, None)

    def bwd(x=0x1000, gy=0x2000, dt=0, rows=4, n=64, ldx=64, ldgy=64, k=5, delta=0.25, gx=0x3000, ldgx=64):
        return lib.spark_stat_topk_huber_backward(vp(x), vp(gy), dt, rows, n, ldx, ldgy, k, delta, vp(gx), ldgx, None)

    assert fwd(x=0) == 1 and fwd(y=0) == 1
    assert fwd(n=1) == 2 and fwd(ldy=32) == 2 and fwd(delta=-1.0) == 2 and fwd(delta=float("nan")) == 2
    assert fwd(k=0) == 3 and fwd(k=64) == 3
    assert fwd(dt=2) == 4 and fwd(dt=3) == 4                  # the 8-bit code types are weight types only
    assert fwd(x=0x1004) == 5 and fwd(dt=1, ldx=68, ldy=68) == 5
    assert fwd(rows=0) == 0
    assert bwd(gy=0) == 1 and bwd(gx=0) == 1
    assert bwd(ldgy=60) == 2 and bwd(ldgx=60) == 2 and bwd(delta=float("inf")) == 2
    assert bwd(k=64) == 3 and bwd(dt=5) == 4 and bwd(gy=0x2008) == 5
    assert bwd(rows=0) == 0


def test_prefill_and_8bit_weights_reject_bad_arguments_before_launch():
    lib = binding.load_library()
    vp = ctypes.c_void_p

    def prefill(layer, n_tokens=100, chunk=16, q=0x4000, qd=binding.BF16, ldq=256, y=0x5000, ws=0x10000, ws_bytes=None):
        if ws_bytes is None:
            ws_bytes = binding.ffn_prefill_workspace_bytes(layer.d_model, layer.d_ff, max(1, min(chunk, 64)))
        return lib.spark_ffn_prefill(ctypes.byref(layer), vp(q), qd, n_tokens, chunk, ldq, vp(y), None, None, None,
                                     None, None, vp(ws), ws_bytes, None)

    assert prefill(_layer(), n_tokens=-1) == 2
    assert prefill(_layer(), chunk=0) == 2 and prefill(_layer(), chunk=65) == 2
    assert prefill(_layer(), q=0) == 1
    assert prefill(_layer(), ws_bytes=4096) == 6
    assert prefill(_layer(), n_tokens=0) == 0                 # nothing to do
    assert binding.ffn_prefill_workspace_bytes(256, 1024, 16) >= binding.ffn_workspace_bytes(256, 1024, 16)
    assert binding.ffn_prefill_workspace_bytes(256, 1024, 16) >= binding.ffn_workspace_bytes(256, 1024, 1)
    # 8-bit weight codes: rows of whole 16-byte chunks, tokens cannot be codes, the dense comparison takes one token
    f8 = binding.FP8_E4M3
    assert _decode(_layer(wd=f8, r=136, d_model=328), ldq=328) == 5
    assert _decode(_layer(wd=f8), qd=f8) == 4
    assert _decode(_layer(wd=binding.INT8), qd=binding.INT8) == 4
    for wd in (f8, binding.INT8):
        layer = _layer(wd=wd)
        ws_bytes = binding.ffn_workspace_bytes(256, 1024, 2)
        assert lib.spark_ffn_dense_decode_layers(ctypes.byref(layer), 1, vp(0x4000), binding.BF16, 2, 256, vp(0x5000),
                                                 vp(0x10000), ws_bytes, None) == 4
        assert lib.spark_ffn_dense_decode(ctypes.byref(layer), vp(0x4000), binding.BF16, 1, 256, vp(0x5000),
                                          vp(0x10000), ws_bytes, None) == 4


def test_stat_topk_needs_no_workspace_and_copy_validates():
    assert binding.stat_topk_workspace_bytes(8192, 9216) == 0
    lib = binding.load_library()
    vp = ctypes.c_void_p
    assert lib.spark_copy_bytes(vp(0x1000), vp(0x2000), 0, None) == 0       # nothing to do
    assert lib.spark_copy_bytes(None, vp(0x2000), 64, None) == 1
    assert lib.spark_copy_bytes(vp(0x1008), vp(0x2000), 64, None) == 5
    assert lib.spark_copy_bytes(vp(0x1000), vp(0x2000), 40, None) == 5


def test_tuned_entry_point_validates_like_the_plain_one():
    lib = binding.load_library()
    vp = ctypes.c_void_p
    layer = _layer()
    ws_bytes = binding.ffn_workspace_bytes(256, 1024, 1)
    tune = binding.Tuning(path=1)
    args = lambda n, ws: (ctypes.byref(layer), n, vp(0x4000), binding.BF16, 1, 256, vp(0x5000), None, None, None,
                          None, None, vp(0x10000), ws, ctypes.byref(tune), None)
    assert lib.spark_ffn_decode_layers_tuned(*args(0, ws_bytes)) == 2
    assert lib.spark_ffn_decode_layers_tuned(*args(1, ws_bytes - 1)) == 6


def test_static_scratch_entry_point_rejects_on_the_host():
    """Validation happens before the built-in array is looked up, so these need no GPU."""
    lib = binding.load_library()
    vp = ctypes.c_void_p
    call = lambda layer, batch=1, y=0x5000: lib.spark_ffn_decode_static(
        ctypes.byref(layer), vp(0x4000), binding.BF16, batch, 256, vp(y) if y else None, None, None, None, None, None, None)
    assert call(_layer(), y=0) == 1
    assert call(_layer(), batch=2) == 2                       # one token only
    assert call(_layer(k=0)) == 3
    assert call(_layer(d_ff=600000)) == 6                     # scratch need beyond the built-in array
    assert call(_layer(d_model=328, r=136, wd=binding.F32)) in (2, 5)


def test_sharded_top_k_entries_reject_bad_arguments_before_launch():
    lib = binding.load_library()
    vp = ctypes.c_void_p
    i64 = ctypes.c_int64

    def stats(x=0x1000, dt=0, rows=4, n=64, ldx=256, out=0x2000):
        return lib.spark_stat_topk_shard_stats(vp(x), dt, rows, n, ldx, vp(out) if out else None, None)

    def combine(st=0x1000, ns=(64, 64, 128), rows=4, k=20, theta=0x2000):
        arr = (i64 * max(1, len(ns)))(*ns)
        return lib.spark_stat_topk_combine_stats(vp(st) if st else None, arr, len(ns), rows, k, vp(theta) if theta else None,
                                                 None, None, None)

    def apply(x=0x1000, dt=0, rows=4, n=64, ldx=256, theta=0x3000, fill=0, y=0x2000, ldy=256, cap=0):
        return lib.spark_stat_topk_apply(vp(x), dt, rows, n, ldx, vp(theta) if theta else None, fill, vp(y), ldy, None, None,
                                         cap, None)

    assert stats(x=0) == 1 and stats(out=0) == 1
    assert stats(n=0) == 2 and stats(ldx=32) == 2 and stats(rows=-1) == 2
    assert stats(dt=2) == 4 and stats(x=0x1004) == 5 and stats(dt=1, ldx=260) == 5
    assert stats(rows=0) == 0 and stats(n=1, rows=0) == 0
    assert combine(st=0) == 1 and combine(theta=0) == 1
    assert combine(ns=()) == 2 and combine(ns=(64, 0)) == 2 and combine(ns=(1,)) == 2 and combine(ns=(1,) * 65) == 2
    assert combine(k=0) == 3 and combine(k=256) == 3
    assert combine(rows=0) == 0
    assert apply(x=0) == 1 and apply(theta=0) == 1
    assert apply(n=0) == 2 and apply(ldy=32) == 2 and apply(dt=3) == 4 and apply(fill=2) == 4
    assert apply(x=0x1008) == 5 and apply(rows=0) == 0
