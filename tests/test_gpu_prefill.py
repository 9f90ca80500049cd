"""GPU parity of the chunked prefill entry point (a prompt through one Spark-FFN layer in
chunks of consecutive tokens) against the CPU oracle, token by token and chunk by chunk."""
import numpy as np
import pytest
import torch

import synth
from paper_2506_06644_amd import binding
from parity_util import TOL_BF16_TIGHT, TOL_F32, check_ffn_against_oracle, rel_l2

pytestmark = pytest.mark.gpu


def _run_prefill(shape, w, q, chunk, gelu=binding.GELU_ERF):
    dev = torch.device("cuda:0")
    T = q.shape[0]
    nch = (T + chunk - 1) // chunk
    wd = [t.to(dev) for t in w]
    qd = q.to(dev)
    layer = binding.make_layer(wd[0], wd[1], wd[2], shape.k, gelu)
    ws = binding.make_prefill_workspace(shape.d_model, shape.d_ff, chunk, dev)
    y = torch.full((T, shape.d_model), float("nan"), dtype=torch.float32, device=dev)
    theta = torch.zeros(T, dtype=torch.float32, device=dev)
    cnt = torch.zeros(T, dtype=torch.int32, device=dev)
    idx = torch.full((T, shape.d_ff), -1, dtype=torch.int32, device=dev)
    ucnt = torch.zeros(max(nch, 1), dtype=torch.int32, device=dev)
    uidx = torch.full((max(nch, 1), shape.d_ff), -1, dtype=torch.int32, device=dev)
    binding.spark_ffn_prefill(layer, qd, chunk, y, ws, theta, cnt, idx, ucnt, uidx)
    torch.cuda.synchronize()
    return dict(y=y.cpu().numpy(), theta=theta.cpu().numpy(), count=cnt.cpu().numpy(), idx=idx.cpu().numpy(),
                ucount=ucnt.cpu().numpy(), uidx=uidx.cpu().numpy())


def _check_chunks(shape, w, q, chunk, out, tol, chunks=None, what=""):
    """Every token of the listed chunks (all by default) and each chunk's union against the oracle."""
    T = q.shape[0]
    nch = (T + chunk - 1) // chunk
    worst = 0.0
    for c in (range(nch) if chunks is None else chunks):
        t0, t1 = c * chunk, min(T, (c + 1) * chunk)
        sub = dict(y=out["y"][None, t0:t1], theta=out["theta"][None, t0:t1], count=out["count"][None, t0:t1],
                   idx=out["idx"][None, t0:t1], ucount=out["ucount"][c:c + 1], uidx=out["uidx"][c:c + 1])
        worst = max(worst, check_ffn_against_oracle(shape, [w], q[t0:t1], sub, tol, what=f"{what} chunk {c}"))
    return worst


@pytest.mark.parametrize("n_tokens,chunk", [(53, 16), (17, 8), (141, 2), (5, 16), (64, 64), (40, 1)])
def test_prefill_tiny_layer_bf16(n_tokens, chunk):
    """Full chunks through the batched launch (more chunks than one launch holds for chunk 2),
    a shorter last chunk, a last chunk of one token, a prompt shorter than a chunk."""
    sh = synth.TINY
    w = synth.ffn_layer(sh, 77, torch.bfloat16)
    q = synth.tokens(sh, n_tokens, 9000 + n_tokens, torch.bfloat16)
    out = _run_prefill(sh, w, q, chunk)
    _check_chunks(sh, w, q, chunk, out, TOL_BF16_TIGHT, what=f"T={n_tokens} chunk={chunk}")


def test_prefill_other_types_and_shapes_go_chunk_by_chunk():
    """fp32 weights and a shape the batched launch does not take: one call per chunk inside."""
    sh = synth.TINY
    w = synth.ffn_layer(sh, 78, torch.float32)
    q = synth.tokens(sh, 11, 9100, torch.float32)
    out = _run_prefill(sh, w, q, 4)
    _check_chunks(sh, w, q, 4, out, TOL_F32, what="fp32")
    sh = synth.RAGGED
    w = synth.ffn_layer(sh, 79, torch.bfloat16)
    q = synth.tokens(sh, 19, 9101, torch.bfloat16)
    out = _run_prefill(sh, w, q, 8)
    _check_chunks(sh, w, q, 8, out, TOL_BF16_TIGHT, what="ragged")


def test_prefill_equals_chunk_by_chunk_calls_of_the_general_path():
    from parity_util import run_gpu_ffn
    sh = synth.TINY
    w = synth.ffn_layer(sh, 80, torch.bfloat16)
    q = synth.tokens(sh, 37, 9200, torch.bfloat16)
    a = _run_prefill(sh, w, q, 16)
    for c, t0 in enumerate(range(0, 37, 16)):
        t1 = min(37, t0 + 16)
        b = run_gpu_ffn(sh, [w], q[t0:t1], force_general=True)
        assert rel_l2(a["y"][t0:t1], b["y"][0]) < 1e-6
        mu = int(b["ucount"][0])
        assert a["ucount"][c] == mu and np.array_equal(a["uidx"][c, :mu], b["uidx"][0, :mu])
        assert np.array_equal(a["count"][t0:t1], b["count"][0]) and np.array_equal(a["idx"][t0:t1], b["idx"][0])


def test_prefill_token_results_do_not_depend_on_the_chunking():
    """y[t] is a function of token t alone (Appendix B: individual masks decide the arithmetic)."""
    sh = synth.TINY
    w = synth.ffn_layer(sh, 81, torch.bfloat16)
    q = synth.tokens(sh, 48, 9300, torch.bfloat16)
    a = _run_prefill(sh, w, q, 16)
    b = _run_prefill(sh, w, q, 6)
    assert np.array_equal(a["count"], b["count"]) and np.array_equal(a["idx"], b["idx"])
    assert np.array_equal(a["theta"], b["theta"])
    assert rel_l2(a["y"], b["y"]) < 1e-6


def test_prefill_gemma2_2b_layer_chunks_of_64():
    """The benchmarked configuration's chunk size on the 2B layer shape: 5 full chunks and a
    last one of 10 tokens; the first, a middle and the last chunk token by token."""
    sh = synth.GEMMA2_2B
    w = synth.ffn_layer(sh, 1000, torch.bfloat16)
    q = synth.tokens(sh, 5 * 64 + 10, 9400, torch.bfloat16)
    out = _run_prefill(sh, w, q, 64)
    assert np.isfinite(out["y"]).all()
    _check_chunks(sh, w, q, 64, out, TOL_BF16_TIGHT, chunks=[0, 3, 5], what="2b")
    # every chunk's union is the union of its tokens' own index sets
    for c in range(6):
        t0, t1 = c * 64, min(q.shape[0], (c + 1) * 64)
        un = np.unique(np.concatenate([out["idx"][t, :out["count"][t]] for t in range(t0, t1)]))
        assert out["ucount"][c] == len(un) and np.array_equal(out["uidx"][c, :len(un)], un)


def test_prefill_argument_errors_and_empty_prompt():
    dev = torch.device("cuda:0")
    sh = synth.TINY
    w = [t.to(dev) for t in synth.ffn_layer(sh, 82, torch.bfloat16)]
    layer = binding.make_layer(w[0], w[1], w[2], sh.k)
    q = synth.tokens(sh, 8, 9500, torch.bfloat16).to(dev)
    y = torch.full((8, sh.d_model), 7.0, device=dev)
    ws = binding.make_prefill_workspace(sh.d_model, sh.d_ff, 4, dev)
    assert binding.ffn_prefill_workspace_bytes(sh.d_model, sh.d_ff, 0) == 0
    assert binding.ffn_prefill_workspace_bytes(sh.d_model, sh.d_ff, 65) == 0
    for chunk in (0, 65):
        with pytest.raises(binding.SparkError) as e:
            binding.spark_ffn_prefill(layer, q, chunk, y, ws)
        assert e.value.code == 2          # SPARK_ERR_SHAPE
    with pytest.raises(binding.SparkError) as e:
        binding.spark_ffn_prefill(layer, q, 4, y, ws[:1024])
    assert e.value.code == 6              # SPARK_ERR_WORKSPACE
    binding.spark_ffn_prefill(layer, q, 4, y, ws, n_tokens=0)   # nothing to do, nothing written
    torch.cuda.synchronize()
    assert torch.all(y == 7.0)


def test_prefill_as_benchmarked_4096_tokens():
    """The benchmark's launch configuration (4096 tokens, chunks of 64: two sets of 32 chunk slots):
    sampled tokens against the oracle, every chunk's union against its tokens' own index sets."""
    sh = synth.GEMMA2_2B
    T, chunk = 4096, 64
    w = synth.ffn_layer(sh, 1000, torch.bfloat16)
    dev = torch.device("cuda:0")
    q = synth.tokens(sh, T, 7000, torch.bfloat16, dev)
    wd = [t.to(dev) for t in w]
    layer = binding.make_layer(wd[0], wd[1], wd[2], sh.k)
    ws = binding.make_prefill_workspace(sh.d_model, sh.d_ff, chunk, dev)
    y = torch.full((T, sh.d_model), float("nan"), device=dev)
    cnt = torch.zeros(T, dtype=torch.int32, device=dev)
    idx = torch.full((T, sh.d_ff), -1, dtype=torch.int32, device=dev)
    ucnt = torch.zeros(T // chunk, dtype=torch.int32, device=dev)
    uidx = torch.full((T // chunk, sh.d_ff), -1, dtype=torch.int32, device=dev)
    binding.spark_ffn_prefill(layer, q, chunk, y, ws, None, cnt, idx, ucnt, uidx)
    torch.cuda.synchronize()
    assert torch.isfinite(y).all()
    import oracle
    k1n, k2n, vn = (synth.to_oracle(t) for t in w)
    qs = synth.to_oracle(q)
    for t in (0, 63, 64, 2047, 2048, 2111, 4032, 4095):
        o = oracle.spark_ffn(k1n, k2n, vn, qs[t], sh.k, skip_inactive=True)
        assert rel_l2(y[t].cpu().numpy(), o.y) <= TOL_BF16_TIGHT, t
        m = int(cnt[t])
        got = set(idx[t, :m].cpu().tolist())
        for j in got ^ set(o.idx.tolist()):
            assert abs(o.s[j] - o.theta) < 1e-3 * o.std
    cnt_h, ucnt_h = cnt.cpu().numpy(), ucnt.cpu().numpy()
    for c in (0, 31, 32, 63):
        rows = idx[c * chunk:(c + 1) * chunk].cpu().numpy()
        un = np.unique(np.concatenate([rows[i, :cnt_h[c * chunk + i]] for i in range(chunk)]))
        assert ucnt_h[c] == len(un) and np.array_equal(uidx[c, :len(un)].cpu().numpy(), un)
