"""GPU parity of the Huber statistical top-k (Section 3.2, Eq.13 / Eq.14) and of its backward pass
(gradient through theta, Appendix A.2) against the CPU oracle.

Tolerances, from the arithmetic: the kernels form theta in fp32 in one pass, within
2e-6 (std + |theta|) of the oracle's double two-pass value (the bound the forward tests use); y has
slope <= 1 in theta, so y is within that plus one rounding to the storage type.  In the backward
pass the slope a / delta of the Huber zone moves by that theta error over delta, and the sums over
~k terms add a few fp32 roundings: with delta >= 0.1 std a row's gx is within 5e-5 of the oracle in
relative L2 for fp32 storage, and within the rounding of its bf16 storage (2^-9 rms, 4e-3 allowed)
otherwise.  With delta = 0 an entry within 1e-5 std of theta may fall on the other side (its whole
gy_i moves): such rows are left out and must be rare.
"""
import numpy as np
import pytest
import torch

import oracle
import synth
from paper_2506_06644_amd import binding
from parity_util import rel_l2

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

SHAPES = [(5, 1024, 82), (33, 9216, 737), (7, 1000, 77), (3, 14336, 1147), (2, 20000, 1500), (2, 40000, 3000),
          (4, 24, 3)]


def _padded(t, ld, fillv=0.0):
    rows, n = t.shape
    buf = torch.full((rows, ld), fillv, dtype=t.dtype, device=DEV)
    buf[:, :n] = t.to(DEV)
    return buf[:, :n], buf


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("rows,n,k", SHAPES)
@pytest.mark.parametrize("delta", [0.0, 0.3, 4.0])
def test_huber_forward_matches_oracle(rows, n, k, dtype, delta):
    x = synth.topk_rows(rows, n, seed=4300 + n, dtype=dtype)
    ld = (n + 15) // 8 * 8
    xv, _ = _padded(x, ld)
    y, ybuf = _padded(torch.full((rows, n), 7.0, dtype=dtype), ld, 7.0)
    theta = torch.zeros(rows, dtype=torch.float32, device=DEV)
    binding.spark_stat_topk_huber(xv, k, delta, y, theta)
    torch.cuda.synchronize()
    xs = synth.to_oracle(x).astype(np.float64)
    ref_y, ref_theta = oracle.huber_stat_topk(xs, k, delta)
    st = oracle.stat_topk_rows(xs, k, want_y=False, want_idx=False)
    yg = y.float().cpu().numpy().astype(np.float64)
    ulp = 2.0 ** -8 if dtype == torch.bfloat16 else 2.0 ** -22
    for r in range(rows):
        eps = 2e-6 * (st.std[r] + abs(ref_theta[r]))
        assert abs(theta[r].item() - ref_theta[r]) <= eps
        assert np.all(np.abs(yg[r] - ref_y[r]) <= ulp * np.abs(ref_y[r]) + 2 * eps), f"row {r}"
    assert torch.all(ybuf[:, n:] == 7.0)   # nothing written past the row


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("rows,n,k", SHAPES)
@pytest.mark.parametrize("delta", [0.0, 0.3, 4.0])
def test_backward_matches_oracle(rows, n, k, dtype, delta):
    x = synth.topk_rows(rows, n, seed=4400 + n, dtype=dtype)
    gy = synth.grad_rows(rows, n, seed=4500 + n, dtype=dtype)
    ld = (n + 15) // 8 * 8
    (xv, _), (gv, _) = _padded(x, ld), _padded(gy, ld + 8)
    gx, gxbuf = _padded(torch.full((rows, n), 7.0, dtype=dtype), ld + 16, 7.0)
    binding.spark_stat_topk_huber_backward(xv, gv, k, delta, gx)
    torch.cuda.synchronize()
    xs = synth.to_oracle(x).astype(np.float64)
    gs = synth.to_oracle(gy).astype(np.float64)
    ref = oracle.huber_stat_topk_vjp(xs, gs, k, delta)
    st = oracle.stat_topk_rows(xs, k, want_y=False, want_idx=False)
    got = gx.float().cpu().numpy().astype(np.float64)
    tol = 4e-3 if dtype == torch.bfloat16 else 5e-5
    skipped = 0
    for r in range(rows):
        if delta == 0.0 and np.min(np.abs(xs[r] - st.theta[r])) < 1e-5 * st.std[r]:
            skipped += 1
            continue
        assert rel_l2(got[r], ref[r]) <= tol, f"row {r}: {rel_l2(got[r], ref[r]):.3e}"
        if dtype == torch.float32:      # the small common term of the entries that were dropped
            drop = xs[r] <= st.theta[r]
            assert np.allclose(got[r][drop], ref[r][drop], rtol=2e-3, atol=1e-4 * np.max(np.abs(ref[r])))
    assert skipped <= max(1, rows // 10)
    assert torch.all(gxbuf[:, n:] == 7.0)


def test_backward_in_place_and_degenerate_rows():
    """gx may overwrite gy; a constant row and a row with one outlier."""
    n, k = 2048, 100
    x = synth.topk_rows(4, n, seed=4600, dtype=torch.float32)
    x[1] = 3.25
    x[2] = 0.0
    x[2, 17] = 1.0
    gy = synth.grad_rows(4, n, seed=4601, dtype=torch.float32)
    ref = oracle.huber_stat_topk_vjp(x.numpy().astype(np.float64), gy.numpy().astype(np.float64), k, 0.2)
    xd, gd = x.to(DEV), gy.to(DEV)
    binding.spark_stat_topk_huber_backward(xd, gd, k, 0.2, gd)
    torch.cuda.synchronize()
    got = gd.cpu().numpy().astype(np.float64)
    assert np.all(got[1] == 0.0) and np.all(ref[1] == 0.0)
    for r in (0, 2, 3):
        assert rel_l2(got[r], ref[r]) <= 5e-5
    # forward in place as well
    y_ref, _ = oracle.huber_stat_topk(x.numpy().astype(np.float64), k, 0.2)
    binding.spark_stat_topk_huber(xd, k, 0.2, xd)
    torch.cuda.synchronize()
    assert np.allclose(xd.cpu().numpy(), y_ref, rtol=1e-5, atol=1e-5)


def test_prefill_shape_sampled_rows():
    """The benchmarked shape (8192 x 9216, k = 737, bf16 and fp32): sampled rows against the oracle."""
    rows, n, k, delta = 8192, 9216, 737, 0.25
    for dtype in (torch.bfloat16, torch.float32):
        x = synth.topk_rows(rows, n, seed=4242, dtype=dtype, device=DEV)
        gy = synth.grad_rows(rows, n, seed=4243, dtype=dtype, device=DEV)
        gx = torch.empty_like(x)
        y = torch.empty_like(x)
        binding.spark_stat_topk_huber_backward(x, gy, k, delta, gx)
        binding.spark_stat_topk_huber(x, k, delta, y)
        torch.cuda.synchronize()
        pick = [0, 1, 4095, 4096, 8190, 8191] + list(range(37, rows, 911))
        xs = synth.to_oracle(x[pick]).astype(np.float64)
        gs = synth.to_oracle(gy[pick]).astype(np.float64)
        ref = oracle.huber_stat_topk_vjp(xs, gs, k, delta)
        ref_y, _ = oracle.huber_stat_topk(xs, k, delta)
        got = gx[pick].float().cpu().numpy().astype(np.float64)
        got_y = y[pick].float().cpu().numpy().astype(np.float64)
        tol = 4e-3 if dtype == torch.bfloat16 else 5e-5
        for i in range(len(pick)):
            assert rel_l2(got[i], ref[i]) <= tol
            assert rel_l2(got_y[i], ref_y[i]) <= tol
        del x, gy, gx, y


def test_argument_errors():
    x = torch.zeros(2, 64, device=DEV)
    for bad in (-1.0, float("nan"), float("inf")):
        with pytest.raises(binding.SparkError) as e:
            binding.spark_stat_topk_huber(x, 5, bad, x)
        assert e.value.code == 2
        with pytest.raises(binding.SparkError) as e:
            binding.spark_stat_topk_huber_backward(x, x, 5, bad, x)
        assert e.value.code == 2
    with pytest.raises(binding.SparkError) as e:
        binding.spark_stat_topk_huber_backward(x, x, 64, 0.1, x)
    assert e.value.code == 3
