"""GPU parity of the sharded statistical top-k (Appendix D.2): one device's three calls (shard
statistics, combination, thresholding with the combined threshold) against the CPU oracle's global
variant, which equals the unsharded operator; the local variant (the plain call on a shard with
k / m) against the oracle's local variant."""
import numpy as np
import pytest
import torch

import oracle
import synth
from paper_2506_06644_amd import binding
from parity_util import assert_active_set

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _global_on_gpu(x, k, bounds, fill=binding.FILL_ZERO):
    """The three calls, shard by shard, on views of one device tensor (row pitch = the full row)."""
    rows, n = x.shape
    m = len(bounds) - 1
    stats = torch.full((m, rows, 2), float("nan"), device=DEV)
    for s, (b0, b1) in enumerate(zip(bounds, bounds[1:])):
        binding.spark_stat_topk_shard_stats(x[:, b0:b1], stats[s])
    theta = torch.empty(rows, device=DEV)
    mean = torch.empty(rows, device=DEV)
    std = torch.empty(rows, device=DEV)
    binding.spark_stat_topk_combine_stats(stats, [b1 - b0 for b0, b1 in zip(bounds, bounds[1:])], k, theta, mean, std)
    y = torch.full_like(x, 7.0)
    counts, lists = [], []
    for b0, b1 in zip(bounds, bounds[1:]):
        cnt = torch.zeros(rows, dtype=torch.int32, device=DEV)
        idx = torch.full((rows, b1 - b0), -1, dtype=torch.int32, device=DEV)
        binding.spark_stat_topk_apply(x[:, b0:b1], theta, fill, y[:, b0:b1], cnt, idx)
        counts.append(cnt)
        lists.append(idx)
    torch.cuda.synchronize()
    return dict(theta=theta.cpu().numpy(), mean=mean.cpu().numpy(), std=std.cpu().numpy(), y=y.float().cpu().numpy(),
                counts=[c.cpu().numpy() for c in counts], lists=[l.cpu().numpy() for l in lists])


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("n,k,bounds", [(9216, 737, [0, 2304, 4608, 6912, 9216]), (9216, 737, [0, 1000, 6000, 9216]),
                                        (9216, 737, [0, 9208, 9216]), (1000, 77, [0, 504, 1000]),
                                        (40000, 3000, [0, 24000, 40000])])
def test_global_variant_matches_the_oracle_and_the_unsharded_call(n, k, bounds, dtype):
    rows = 19
    x = synth.topk_rows(rows, n, seed=6100 + n, dtype=dtype, device=torch.device(DEV))
    x[:, :bounds[1]] += 0.75          # shards of different levels
    out = _global_on_gpu(x, k, bounds)
    xs = synth.to_oracle(x.cpu())
    ref = oracle.stat_topk_sharded(xs, k, bounds)
    whole_cnt = torch.zeros(rows, dtype=torch.int32, device=DEV)
    whole_theta = torch.empty(rows, device=DEV)
    binding.spark_stat_topk(x, k, theta=whole_theta, count=whole_cnt)
    torch.cuda.synchronize()
    for r in range(rows):
        tag = f"n={n} row {r}"
        assert abs(out["theta"][r] - ref.theta[r]) <= 1e-5 * ref.std[r] + 1e-6 * abs(ref.theta[r]), tag
        assert abs(out["std"][r] - ref.std[r]) <= 1e-5 * ref.std[r], tag
        assert abs(out["theta"][r] - whole_theta[r].item()) <= 1e-5 * ref.std[r] + 1e-6 * abs(ref.theta[r]), tag
        got = np.concatenate([out["lists"][s][r, :out["counts"][s][r]] + b0 for s, b0 in enumerate(bounds[:-1])])
        assert np.all(np.diff(got) > 0), tag
        assert_active_set(got, xs[r], ref.theta[r], ref.std[r], tag)
        for s in range(len(bounds) - 1):
            c = out["counts"][s][r]
            assert np.all(out["lists"][s][r, c:] == -1), tag
        keep = np.zeros(n, bool)
        keep[got] = True
        theta_gpu = np.float64(out["theta"][r])
        expect = np.where(keep, xs[r] - theta_gpu, 0.0)
        tol = 1e-6 * (np.abs(xs[r]) + abs(theta_gpu)) if dtype == torch.float32 else 2.0 ** -8 * np.abs(expect) + 1e-30
        assert np.all(np.abs(out["y"][r] - expect) <= tol), tag
    assert abs(int(whole_cnt.sum().item()) - sum(int(c.sum()) for c in out["counts"])) <= 2 * rows


def test_fill_in_place_and_one_entry_shards():
    """-inf fill, y aliasing x, and a shard of a single column (its centred sum of squares is 0)."""
    rows, n, k = 5, 520, 40
    bounds = [0, 8, 512, 520]
    x = synth.topk_rows(rows, n, seed=6200, dtype=torch.float32, device=torch.device(DEV))
    keep = x.clone()
    out = _global_on_gpu(x, k, bounds, fill=binding.FILL_NEG_INF)
    ref = oracle.stat_topk_sharded(synth.to_oracle(keep.cpu()), k, bounds, fill=oracle.FILL_NEG_INF)
    assert np.array_equal(np.isneginf(out["y"]), np.isneginf(ref.y))
    one = torch.empty(rows, 2, device=DEV)
    binding.spark_stat_topk_shard_stats(x[:, 16:17], one)      # pitch 520 floats, one column
    torch.cuda.synchronize()
    assert torch.equal(one[:, 0], x[:, 16]) and torch.all(one[:, 1] == 0)
    theta = torch.from_numpy(ref.theta.astype(np.float32)).to(DEV)
    binding.spark_stat_topk_apply(x[:, 8:512], theta, binding.FILL_ZERO, x[:, 8:512])       # in place
    torch.cuda.synchronize()
    expect = np.where(keep[:, 8:512].cpu().numpy() > theta.cpu().numpy()[:, None],
                      keep[:, 8:512].cpu().numpy() - theta.cpu().numpy()[:, None], 0.0)
    assert np.allclose(x[:, 8:512].cpu().numpy(), expect, rtol=1e-6, atol=1e-6)
    assert torch.equal(x[:, :8], keep[:, :8]) and torch.equal(x[:, 512:], keep[:, 512:])


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_local_variant_is_the_plain_call_on_every_shard(dtype):
    rows, n, k, m = 11, 8192, 656, 4
    bounds = [i * n // m for i in range(m + 1)]
    x = synth.topk_rows(rows, n, seed=6300, dtype=dtype, device=torch.device(DEV))
    xs = synth.to_oracle(x.cpu())
    ref = oracle.stat_topk_sharded(xs, k, bounds, local=True)
    total = np.zeros(rows, np.int64)
    for b0, b1 in zip(bounds, bounds[1:]):
        cnt = torch.zeros(rows, dtype=torch.int32, device=DEV)
        idx = torch.full((rows, b1 - b0), -1, dtype=torch.int32, device=DEV)
        theta = torch.empty(rows, device=DEV)
        binding.spark_stat_topk(x[:, b0:b1], k // m, theta=theta, count=cnt, idx=idx)
        torch.cuda.synchronize()
        part = oracle.stat_topk_rows(xs[:, b0:b1], k // m)
        for r in range(rows):
            assert abs(theta[r].item() - part.theta[r]) <= 1e-5 * part.std[r] + 1e-6 * abs(part.theta[r])
            assert_active_set(idx[r, :cnt[r]].cpu().numpy(), xs[r, b0:b1], part.theta[r], part.std[r], f"shard {b0} row {r}")
        total += cnt.cpu().numpy()
    assert np.all(np.abs(total - ref.count) <= 8)
