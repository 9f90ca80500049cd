"""GPU parity of the Spark-FFN decode path with 8-bit (OCP E4M3 or signed integer) weight rows and per-row scales
(the quantisation synergy of Appendix D.4) against the CPU oracle.

The synthetic quantiser keeps scales to 8 significant bits, so the oracle's float weights
scale * value(code) are exactly the stored weights; the kernels widen the codes exactly, multiply
and add in fp32 and apply the row's scale to the finished dot product.  Bars as for bf16 weights:
index sets exact outside the 1e-3 std band, y within 5e-5 relative L2 (1e-2 is the stated bar).
"""
import numpy as np
import pytest
import torch

import oracle
import synth
from paper_2506_06644_amd import binding
from parity_util import TOL_BF16_TIGHT, check_ffn_against_oracle

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


KINDS = {"fp8": (binding.FP8_E4M3, synth.quantize_rows_fp8, oracle.fp8_dequantize_rows),
         "int8": (binding.INT8, synth.quantize_rows_int8, oracle.int8_dequantize_rows)}


def _quantised_stack(shape, n_layers, seed, kind="fp8"):
    """(packed device arrays per layer, dequantised float32 CPU weights per layer)."""
    _, quantize, dequantize = KINDS[kind]
    packed, deq = [], []
    for l in range(n_layers):
        w = synth.ffn_layer(shape, seed + l, torch.float32)
        pk, dq = [], []
        for t in w:
            codes, scales = quantize(t)
            pk.append(binding.pack_fp8_rows(codes, scales).to(DEV))
            dq.append(torch.from_numpy(dequantize(codes.numpy(), scales.numpy())))
        packed.append(pk)
        deq.append(tuple(dq))
    return packed, deq


def _run(shape, packed, q, via_layers, dense=False, gelu=binding.GELU_ERF, kind="fp8"):
    L, B = len(packed), q.shape[0]
    layers = [binding.make_layer_fp8(p[0], p[1], p[2], shape.d_model, shape.d_ff, shape.r, shape.k, gelu, KINDS[kind][0])
              for p in packed]
    qd = q.to(DEV)
    ws = binding.make_workspace(shape.d_model, shape.d_ff, B, DEV)
    y = torch.full((L, B, shape.d_model), float("nan"), device=DEV)
    theta = torch.zeros(L, B, device=DEV)
    cnt = torch.zeros(L, B, dtype=torch.int32, device=DEV)
    idx = torch.full((L, B, shape.d_ff), -1, dtype=torch.int32, device=DEV)
    ucnt = torch.zeros(L, dtype=torch.int32, device=DEV)
    uidx = torch.full((L, shape.d_ff), -1, dtype=torch.int32, device=DEV)
    if dense:
        binding.spark_ffn_dense_decode_layers(layers, qd, y, ws)
    elif via_layers:
        binding.spark_ffn_decode_layers(layers, qd, y, ws, theta, cnt, idx, ucnt, uidx)
    else:
        for l in range(L):
            binding.spark_ffn_decode(layers[l], qd, y[l], ws, theta[l], cnt[l], idx[l], ucnt[l:l + 1], uidx[l])
    torch.cuda.synchronize()
    return dict(y=y.cpu().numpy(), theta=theta.cpu().numpy(), count=cnt.cpu().numpy(), idx=idx.cpu().numpy(),
                ucount=ucnt.cpu().numpy(), uidx=uidx.cpu().numpy())


@pytest.mark.parametrize("kind", ["fp8", "int8"])
@pytest.mark.parametrize("qdtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("via_layers", [False, True])
def test_tiny_layers(qdtype, via_layers, kind):
    sh = synth.TINY
    packed, deq = _quantised_stack(sh, 3, 300, kind)
    q = synth.tokens(sh, 1, 301, qdtype)
    out = _run(sh, packed, q, via_layers, kind=kind)
    worst = check_ffn_against_oracle(sh, deq, q, out, TOL_BF16_TIGHT, what=f"fp8 tiny {qdtype}")
    assert worst < TOL_BF16_TIGHT


@pytest.mark.parametrize("kind", ["fp8", "int8"])
@pytest.mark.parametrize("shape", [synth.GEMMA2_2B, synth.GEMMA2_9B, synth.FFNShape("odd", 1040, 1000, 272, 77)])
def test_model_shapes_and_a_ragged_one(shape, kind):
    """The 2B and 9B layer shapes (two layers in one call) and a shape whose rows do not fill the last
    16-byte chunks of a wave and whose d_ff is ragged."""
    packed, deq = _quantised_stack(shape, 2, 310, kind)
    q = synth.tokens(shape, 1, 311, torch.bfloat16)
    out = _run(shape, packed, q, True, kind=kind)
    check_ffn_against_oracle(shape, deq, q, out, TOL_BF16_TIGHT, what=f"fp8 {shape.name}")
    assert np.all(np.abs(out["count"] - shape.k) < 6 * np.sqrt(shape.k) + 6)


@pytest.mark.parametrize("kind", ["fp8", "int8"])
def test_dense_evaluation_and_tanh_gelu(kind):
    sh = synth.TINY
    packed, deq = _quantised_stack(sh, 2, 320, kind)
    q = synth.tokens(sh, 1, 321, torch.bfloat16)
    out = _run(sh, packed, q, True, dense=True, kind=kind)
    check_ffn_against_oracle(sh, deq, q, out, TOL_BF16_TIGHT, dense=True, what="fp8 dense")
    out = _run(sh, packed, q, True, gelu=binding.GELU_TANH, kind=kind)
    check_ffn_against_oracle(sh, deq, q, out, TOL_BF16_TIGHT, gelu=oracle.GELU_TANH, what="fp8 tanh")


@pytest.mark.parametrize("kind", ["fp8", "int8"])
@pytest.mark.parametrize("shape,batch", [(synth.TINY, 2), (synth.TINY, 16), (synth.FFNShape("odd", 1040, 1000, 272, 77), 5),
                                         (synth.GEMMA2_2B, 4), (synth.TINY, 64)])
def test_batches_take_the_general_kernels(shape, batch, kind):
    """More than one token with 8-bit weight rows, on shapes, token types and batch sizes that the
    whole-row kernels do not take (and the 2B shape with bf16 tokens, which they do): every token against
    the oracle on the dequantised weights, the union list against the oracle's, and y[b] equal to the
    one-token result."""
    packed, deq = _quantised_stack(shape, 2, 340, kind)
    for qdtype in (torch.bfloat16, torch.float32):
        q = synth.tokens(shape, batch, 341 + batch, qdtype)
        for via_layers in (False, True):
            out = _run(shape, packed, q, via_layers, kind=kind)
            check_ffn_against_oracle(shape, deq, q, out, TOL_BF16_TIGHT, what=f"{kind} B={batch} {qdtype}")
        solo = _run(shape, packed, q[1:2], True, kind=kind)
        assert np.array_equal(solo["idx"][:, 0], out["idx"][:, 1])
        assert np.linalg.norm(solo["y"][:, 0] - out["y"][:, 1]) <= 1e-6 * np.linalg.norm(solo["y"][:, 0])


@pytest.mark.parametrize("kind", ["fp8", "int8"])
@pytest.mark.parametrize("d_model,d_ff,r,k", [(2304, 1000, 1024, 77), (3072, 600, 1536, 48), (3584, 200, 1536, 20),
                                              (2048, 2085, 1024, 160)])
@pytest.mark.parametrize("batch", [2, 7, 12, 16])
def test_batches_on_the_whole_row_kernels(d_model, d_ff, r, k, batch, kind):
    """Two to sixteen bf16 tokens with rows of whole 256-code multiples: the whole-row matrix-core kernels
    widen the codes to bf16 in registers (predict, k2) and on the way into LDS (V).  Every compiled row
    length (1024 .. 2048 codes), one to four groups of four tokens, ragged numbers of neurons, one and
    several layers; against the oracle on the dequantised weights and against the one-token path."""
    sh = synth.FFNShape("rows4-8bit", d_model, d_ff, r, k)
    for n_layers in (1, 3):
        packed, deq = _quantised_stack(sh, n_layers, 360 + n_layers, kind)
        q = synth.tokens(sh, batch, 370 + batch, torch.bfloat16)
        out = _run(sh, packed, q, True, kind=kind)
        check_ffn_against_oracle(sh, deq, q, out, TOL_BF16_TIGHT, what=f"{kind} whole rows B={batch} L={n_layers}")
        solo = _run(sh, packed, q[batch - 1:batch], True, kind=kind)
        assert np.linalg.norm(solo["y"][:, 0] - out["y"][:, batch - 1]) <= 1e-5 * np.linalg.norm(solo["y"][:, 0])


@pytest.mark.parametrize("kind", ["fp8", "int8"])
@pytest.mark.parametrize("d_model,d_ff,r,k", [(2048, 600, 1024, 48), (2304, 1000, 1024, 77), (3072, 200, 1536, 20)])
@pytest.mark.parametrize("batch", [17, 40, 64])
def test_batches_on_the_staged_kernels(d_model, d_ff, r, k, batch, kind):
    """Seventeen to sixty-four bf16 tokens: tiles of 16 rows of codes are widened to bf16 on the way into
    LDS (predict, k2; the rows' scales travel with them) and in the V step.  Two, three and four token
    blocks, every compiled row length, ragged numbers of neurons (the 2B-like shape with two token blocks
    is one the staged kernels do not take: it goes through the general ones); against the oracle."""
    sh = synth.FFNShape("staged-8bit", d_model, d_ff, r, k)
    for n_layers in (1, 3):
        packed, deq = _quantised_stack(sh, n_layers, 390 + n_layers, kind)
        q = synth.tokens(sh, batch, 395 + batch, torch.bfloat16)
        out = _run(sh, packed, q, True, kind=kind)
        check_ffn_against_oracle(sh, deq, q, out, TOL_BF16_TIGHT, what=f"{kind} staged B={batch} L={n_layers}")


@pytest.mark.parametrize("kind", ["fp8", "int8"])
def test_prefill_in_chunks_on_the_whole_row_kernels(kind):
    """A prompt through a 2B-shaped layer with 8-bit weights in chunks of 8 (the full chunks share one set
    of batched launches, the shorter last chunk takes a call of its own): sampled tokens and every
    chunk's union size against the oracle."""
    sh = synth.FFNShape("prefill-8bit", 2304, 1000, 1024, 77)
    packed, deq = _quantised_stack(sh, 1, 380, kind)
    layer = binding.make_layer_fp8(*packed[0], sh.d_model, sh.d_ff, sh.r, sh.k, code_dtype=KINDS[kind][0])
    T, chunk = 29, 8
    q = synth.tokens(sh, T, 381, torch.bfloat16)
    ws = binding.make_prefill_workspace(sh.d_model, sh.d_ff, chunk, DEV)
    nch = (T + chunk - 1) // chunk
    y = torch.full((T, sh.d_model), float("nan"), device=DEV)
    theta = torch.zeros(T, device=DEV)
    cnt = torch.zeros(T, dtype=torch.int32, device=DEV)
    idx = torch.full((T, sh.d_ff), -1, dtype=torch.int32, device=DEV)
    ucnt = torch.zeros(nch, dtype=torch.int32, device=DEV)
    uidx = torch.full((nch, sh.d_ff), -1, dtype=torch.int32, device=DEV)
    binding.spark_ffn_prefill(layer, q.to(DEV), chunk, y, ws, theta, cnt, idx, ucnt, uidx)
    torch.cuda.synchronize()
    for c in range(nch):
        t0, t1 = c * chunk, min(T, (c + 1) * chunk)
        sub = dict(y=y[None, t0:t1].cpu().numpy(), theta=theta[None, t0:t1].cpu().numpy(),
                   count=cnt[None, t0:t1].cpu().numpy(), idx=idx[None, t0:t1].cpu().numpy(),
                   ucount=ucnt[c:c + 1].cpu().numpy(), uidx=uidx[c:c + 1].cpu().numpy())
        check_ffn_against_oracle(sh, deq, q[t0:t1], sub, TOL_BF16_TIGHT, what=f"{kind} prefill chunk {c}")


@pytest.mark.parametrize("kind", ["fp8", "int8"])
def test_prefill_in_chunks(kind):
    """A prompt through a layer with 8-bit weights in chunks of 4 (last chunk shorter): every token and
    every chunk's union against the oracle."""
    sh = synth.TINY
    packed, deq = _quantised_stack(sh, 1, 350, kind)
    layer = binding.make_layer_fp8(*packed[0], sh.d_model, sh.d_ff, sh.r, sh.k, code_dtype=KINDS[kind][0])
    T, chunk = 11, 4
    q = synth.tokens(sh, T, 351, torch.bfloat16)
    ws = binding.make_prefill_workspace(sh.d_model, sh.d_ff, chunk, DEV)
    nch = (T + chunk - 1) // chunk
    y = torch.full((T, sh.d_model), float("nan"), device=DEV)
    theta = torch.zeros(T, device=DEV)
    cnt = torch.zeros(T, dtype=torch.int32, device=DEV)
    idx = torch.full((T, sh.d_ff), -1, dtype=torch.int32, device=DEV)
    ucnt = torch.zeros(nch, dtype=torch.int32, device=DEV)
    uidx = torch.full((nch, sh.d_ff), -1, dtype=torch.int32, device=DEV)
    binding.spark_ffn_prefill(layer, q.to(DEV), chunk, y, ws, theta, cnt, idx, ucnt, uidx)
    torch.cuda.synchronize()
    for c in range(nch):
        t0, t1 = c * chunk, min(T, (c + 1) * chunk)
        sub = dict(y=y[None, t0:t1].cpu().numpy(), theta=theta[None, t0:t1].cpu().numpy(),
                   count=cnt[None, t0:t1].cpu().numpy(), idx=idx[None, t0:t1].cpu().numpy(),
                   ucount=ucnt[c:c + 1].cpu().numpy(), uidx=uidx[c:c + 1].cpu().numpy())
        check_ffn_against_oracle(sh, deq, q[t0:t1], sub, TOL_BF16_TIGHT, what=f"{kind} prefill chunk {c}")


def test_prefill_token_by_token_and_unsupported_uses():
    sh = synth.TINY
    packed, deq = _quantised_stack(sh, 1, 330)
    layer = binding.make_layer_fp8(*packed[0], sh.d_model, sh.d_ff, sh.r, sh.k)
    q = synth.tokens(sh, 5, 331, torch.bfloat16)
    qd = q.to(DEV)
    ws = binding.make_prefill_workspace(sh.d_model, sh.d_ff, 4, DEV)
    y = torch.empty(5, sh.d_model, device=DEV)
    binding.spark_ffn_prefill(layer, qd, 1, y, ws)
    torch.cuda.synchronize()
    for t in range(5):
        o = oracle.spark_ffn(*(synth.to_oracle(a) for a in deq[0]), synth.to_oracle(q)[t], sh.k, skip_inactive=True)
        assert np.linalg.norm(y[t].cpu().numpy() - o.y) <= TOL_BF16_TIGHT * np.linalg.norm(o.y)
    # the dense comparison calls take one token, and only through the layers entry point
    for call in (lambda: binding.spark_ffn_dense_decode_layers([layer], qd[:2], y[None, :2], ws),
                 lambda: binding.spark_ffn_dense_decode(layer, qd[:1], y[:1], ws)):
        with pytest.raises(binding.SparkError) as e:
            call()
        assert e.value.code == 4          # SPARK_ERR_DTYPE
    # rows must be multiples of 16 codes
    bad = binding._Layer(328, 1000, 136, 77, binding.FP8_E4M3, 0, packed[0][0].data_ptr(), packed[0][1].data_ptr(),
                         packed[0][2].data_ptr())
    with pytest.raises(binding.SparkError) as e:
        binding.spark_ffn_decode(bad, torch.zeros(1, 328, device=DEV), torch.zeros(1, 328, device=DEV), ws)
    assert e.value.code == 5              # SPARK_ERR_ALIGN


@pytest.mark.parametrize("kind,batch", [("fp8", 1), ("int8", 1), ("fp8", 4), ("int8", 16), ("fp8", 64)])
def test_stack_as_benchmarked_52_layers(kind, batch):
    """The benchmark's launch configurations (52 quantised 2B-shaped layers in one call, with 1, 4, 16
    or 64 tokens): y of the first, a middle and the last layer, and every layer's index sets, against
    the oracle."""
    sh, L = synth.GEMMA2_2B, 52
    _, quantize, dequantize = KINDS[kind]
    packed, host = [], {}
    for l in range(L):
        w = synth.ffn_layer(sh, 1000 + l, torch.float32, DEV)
        arrays = []
        for i, t in enumerate(w):
            codes, scales = quantize(t)
            arrays.append(binding.pack_fp8_rows(codes, scales))
            if i == 0 or l in (0, 25, 51):
                host[(l, i)] = dequantize(codes.cpu().numpy(), scales.cpu().numpy())
        packed.append(arrays)
        del w
    q = synth.tokens(sh, batch, 2001, torch.bfloat16)
    out = _run(sh, packed, q, True, kind=kind)
    qs = synth.to_oracle(q)
    pick = [0, 25, 51]
    sub = {k: (v[pick] if v.shape[0] == L else v) for k, v in out.items()}
    deq = [tuple(torch.from_numpy(host[(l, i)]) for i in range(3)) for l in pick]
    check_ffn_against_oracle(sh, deq, q, sub, TOL_BF16_TIGHT, what=f"{kind} stack, {batch} tokens")
    from parity_util import assert_active_set
    for l in range(L):
        S = qs[:, :sh.r].astype(np.float64) @ host[(l, 0)].astype(np.float64).T
        ref = oracle.stat_topk_rows(S, sh.k)
        for b in range(batch):
            assert abs(out["theta"][l, b] - ref.theta[b]) <= 1e-5 * ref.std[b] + 1e-6 * abs(ref.theta[b])
            m = int(out["count"][l, b])
            assert_active_set(out["idx"][l, b, :m], S[b], ref.theta[b], ref.std[b], f"layer {l} token {b}")
