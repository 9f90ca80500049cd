"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
import synth
from paper_2506_06644_amd import binding

from parity_util import (TOL_BF16, TOL_BF16_TIGHT, TOL_F32, assert_active_set, check_ffn_against_oracle,
                         rel_l2, run_gpu_ffn)

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


# ------------------------------------------------------------------------------- stat top-k
def _topk_case(rows, n, k, dtype, fill=binding.FILL_ZERO, seed=4242, ld=None, with_idx=True):
    x = synth.topk_rows(rows, n, seed=seed, dtype=dtype)
    ld = ld or (n + 7) // 8 * 8
    xd = torch.zeros(rows, ld, dtype=dtype, device=DEV)
    xd[:, :n] = x.to(DEV)
    xv = xd[:, :n]
    y = torch.full((rows, ld), 7.0, dtype=dtype, device=DEV)[:, :n]
    theta = torch.zeros(rows, dtype=torch.float32, device=DEV)
    count = torch.zeros(rows, dtype=torch.int32, device=DEV)
    idx = torch.full((rows, n), -1, dtype=torch.int32, device=DEV) if with_idx else None
    binding.spark_stat_topk(xv, k, fill, y, theta, count, idx)
    torch.cuda.synchronize()
    ref = oracle.stat_topk_rows(synth.to_oracle(x).astype(np.float64), k, fill)
    yg = y.float().cpu().numpy().astype(np.float64)
    tg, cg = theta.cpu().numpy(), count.cpu().numpy()
    xs = synth.to_oracle(x).astype(np.float64)
    ulp = 2.0 ** -8 if dtype == torch.bfloat16 else 2.0 ** -22
    for r in range(rows):
        assert abs(tg[r] - ref.theta[r]) <= 2e-6 * (ref.std[r] + abs(ref.theta[r])), f"row {r} theta"
        act_g = xs[r] > tg[r]          # what the GPU decided, re-derived from its own theta
        if with_idx:
            gi = idx[r].cpu().numpy()
            m = int(cg[r])
            assert np.all(np.diff(gi[:m]) > 0) and np.all(gi[m:] == -1)
            ndiff = assert_active_set(gi[:m], xs[r], ref.theta[r], ref.std[r], f"row {r}")
            act_g = np.zeros(n, bool)
            act_g[gi[:m]] = True
        else:
            ndiff = int((act_g != (xs[r] > ref.theta[r])).sum())
        assert abs(int(cg[r]) - int(ref.count[r])) <= ndiff
        both = act_g & (xs[r] > ref.theta[r])
        # survivors: x - theta (rounded once to the storage type)
        assert np.all(np.abs(yg[r][both] - ref.y[r][both]) <= ulp * np.abs(ref.y[r][both])
                      + 4e-6 * (ref.std[r] + abs(ref.theta[r]))), f"row {r} values"
        dropped = ~act_g
        if fill == binding.FILL_ZERO:
            assert np.all(yg[r][dropped] == 0.0)
        else:
            assert np.all(np.isneginf(yg[r][dropped]))
    return ref


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("rows,n,k", [(5, 1024, 82), (33, 9216, 737), (7, 1000, 77), (3, 14336, 1147),
                                      (4, 13824, 1106), (2, 40000, 900), (2, 70000, 5000), (3, 8, 2),
                                      (2, 2, 1)])
def test_stat_topk_matches_oracle(rows, n, k, dtype):
    _topk_case(rows, n, k, dtype)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("n", [256, 260, 516, 1280, 1288, 2304, 2312, 4608, 4616, 10240, 10248])
def test_stat_topk_row_lengths_around_the_kernel_tiers(n, dtype):
    """Row lengths at and just past the sizes where the kernel changes its shape (one wavefront per
    row with 1, 2, 5 or 9 vectors per lane; 256 threads with 5, 9 or 14), with and without a ragged
    last vector."""
    _topk_case(6, n, max(1, n // 12), dtype)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_stat_topk_ragged_pitch_neg_inf_and_optional_outputs(dtype):
    _topk_case(6, 1003, 80, dtype, fill=binding.FILL_NEG_INF, ld=1016)
    _topk_case(6, 9216, 737, dtype, with_idx=False)
    # stats only, idx capped
    x = synth.topk_rows(4, 2048, seed=9, dtype=dtype).to(DEV)
    count = torch.zeros(4, dtype=torch.int32, device=DEV)
    idx = torch.full((4, 16), -1, dtype=torch.int32, device=DEV)
    binding.spark_stat_topk(x, 200, count=count, idx=idx)
    torch.cuda.synchronize()
    ref = oracle.stat_topk_rows(synth.to_oracle(x).astype(np.float64), 200)
    assert np.all(np.abs(count.cpu().numpy() - ref.count) <= 2)
    for r in range(4):
        assert np.array_equal(idx[r].cpu().numpy(), ref.idx[r, :16])


def test_stat_topk_in_place_and_degenerate_rows():
    x = synth.topk_rows(9, 4096, seed=3, dtype=torch.float32)
    x[4] = 2.5                                  # constant row: std = 0, nothing survives
    xd = x.to(DEV)
    theta = torch.zeros(9, device=DEV)
    count = torch.zeros(9, dtype=torch.int32, device=DEV)
    binding.spark_stat_topk(xd, 300, y=xd, theta=theta, count=count)
    torch.cuda.synchronize()
    ref = oracle.stat_topk_rows(x.numpy().astype(np.float64), 300)
    assert count[4].item() == 0 and theta[4].item() == 2.5 and not xd[4].any()
    assert rel_l2(xd.cpu().numpy(), ref.y) < 1e-5


def _row_masks(idx, count, n):
    """Boolean [rows, n] membership mask of index lists idx[rows, cap] with `count` valid entries each."""
    rows, cap = idx.shape
    valid = np.arange(cap)[None, :] < count[:, None]
    mask = np.zeros((rows, n), bool)
    rr = np.broadcast_to(np.arange(rows)[:, None], idx.shape)
    mask[rr[valid], idx[valid]] = True
    return mask


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_stat_topk_full_prefill_shape_every_row(dtype):
    """8192 x 9216 (the prefill / training shape) as the benchmark launches it: theta, count and the
    active set of EVERY row against the oracle, the kept values of every row, and the comparison with
    exact sort-based top-k on the same rows: a threshold set is the exact top-|I| set, so it either
    contains or is contained in the exact top-k set (precision or recall is 1)."""
    rows, n, k, cap = 8192, 9216, 737, 2048
    x = synth.topk_rows(rows, n, seed=4242, dtype=dtype, device=DEV)
    y = torch.empty_like(x)
    theta = torch.zeros(rows, device=DEV)
    count = torch.zeros(rows, dtype=torch.int32, device=DEV)
    idx = torch.full((rows, cap), -1, dtype=torch.int32, device=DEV)
    binding.spark_stat_topk(x, k, y=y, theta=theta, count=count, idx=idx)
    torch.cuda.synchronize()
    assert torch.equal((y > 0).sum(1).to(torch.int32), count) and (y >= 0).all()
    tg, cg = theta.cpu().numpy().astype(np.float64), count.cpu().numpy().astype(np.int64)
    assert cg.max() <= cap
    ulp = 2.0 ** -8 if dtype == torch.bfloat16 else 2.0 ** -22
    flips = 0
    precision, recall = [], []
    for lo in range(0, rows, 1024):
        hi = lo + 1024
        xs = synth.to_oracle(x[lo:hi]).astype(np.float64)
        ref = oracle.stat_topk_rows(xs, k, want_idx=False)
        scale = ref.std + np.abs(ref.theta)
        assert np.all(np.abs(tg[lo:hi] - ref.theta) <= 2e-6 * scale), f"theta, rows {lo}..{hi}"
        gmask = _row_masks(idx[lo:hi].cpu().numpy(), cg[lo:hi], n)
        rmask = xs > ref.theta[:, None]
        diff = gmask ^ rmask
        assert np.all(np.abs(xs - ref.theta[:, None])[diff] < 1e-3 * np.broadcast_to(ref.std[:, None], xs.shape)[diff]), (
            f"active sets differ outside the band, rows {lo}..{hi}")
        flips += int(diff.sum())
        assert np.all(np.abs(cg[lo:hi] - ref.count) <= diff.sum(1))
        # kept values: x - theta rounded once to the storage type; everything else exactly 0
        yg = y[lo:hi].float().cpu().numpy().astype(np.float64)
        both = gmask & rmask
        tol = ulp * np.abs(ref.y) + 4e-6 * scale[:, None]
        assert np.all((np.abs(yg - ref.y) <= tol)[both]), f"values, rows {lo}..{hi}"
        assert np.all(yg[~gmask] == 0.0)
        assert np.array_equal(yg > 0, gmask)
        # exact sort-based top-k of the same rows
        tk = _row_masks(oracle.exact_topk_rows(xs, k), np.full(hi - lo, k), n)
        inter = (gmask & tk).sum(1)
        assert np.array_equal(inter, np.minimum(cg[lo:hi], k)), f"nesting with exact top-k, rows {lo}..{hi}"
        precision.append(inter / np.maximum(cg[lo:hi], 1))
        recall.append(inter / k)
    precision, recall = np.concatenate(precision), np.concatenate(recall)
    print(f"{dtype}: count mean {cg.mean():.1f} min {cg.min()} max {cg.max()}, {flips} entries flipped inside the band, "
          f"precision mean {precision.mean():.4f}, recall mean {recall.mean():.4f}", flush=True)
    # a sample of rows: the active set IS the exact top-|I| set
    for r in range(0, rows, 257):
        m = int(cg[r])
        top_m = oracle.exact_topk(synth.to_oracle(x[r]).astype(np.float64), m)
        assert np.array_equal(idx[r, :m].cpu().numpy(), top_m), f"row {r}: not the exact top-{m} set"


# ------------------------------------------------------------------------------- Spark-FFN decode
def _ffn_case(shape, wdtype, qdtype, batch, n_layers=1, gelu=binding.GELU_ERF, via_layers=False, seed=1234,
              force_general=False, tuning=None):
    weights = synth.ffn_stack(shape, n_layers, base_seed=seed, dtype=wdtype)
    q = synth.tokens(shape, batch, seed + 4444, dtype=qdtype)
    out = run_gpu_ffn(shape, weights, q, gelu=gelu, via_layers=via_layers, force_general=force_general, tuning=tuning)
    tol = TOL_F32 if wdtype == torch.float32 else TOL_BF16
    worst = check_ffn_against_oracle(shape, weights, q, out, tol, gelu=gelu,
                                     what=f"{shape.name} {wdtype} B={batch}")
    if wdtype == torch.bfloat16:
        assert worst <= TOL_BF16_TIGHT
    return out


@pytest.mark.parametrize("batch", [1, 3, 16])
@pytest.mark.parametrize("wdtype,qdtype", [(torch.float32, torch.float32), (torch.bfloat16, torch.bfloat16),
                                           (torch.bfloat16, torch.float32), (torch.float32, torch.bfloat16)])
def test_tiny_layer(wdtype, qdtype, batch):
    _ffn_case(synth.TINY, wdtype, qdtype, batch)


@pytest.mark.parametrize("wdtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("batch", [1, 5, 64])
def test_ragged_shape(wdtype, batch):
    _ffn_case(synth.RAGGED, wdtype, wdtype, batch)


def test_tanh_gelu_variant():
    _ffn_case(synth.TINY, torch.float32, torch.float32, 2, gelu=binding.GELU_TANH)
    _ffn_case(synth.TINY, torch.float32, torch.float32, 1, gelu=binding.GELU_TANH)


# batch 1 has two implementations (phase by phase over the layers of a call, separate kernels per
# layer): both are held to the oracle
@pytest.mark.parametrize("force_general", [0, 1])
@pytest.mark.parametrize("shape,wdtype,qdtype", [
    (synth.TINY, torch.float32, torch.float32), (synth.TINY, torch.bfloat16, torch.bfloat16),
    (synth.TINY, torch.bfloat16, torch.float32), (synth.RAGGED, torch.bfloat16, torch.bfloat16),
    (synth.RAGGED, torch.float32, torch.float32), (synth.GEMMA2_2B, torch.bfloat16, torch.bfloat16)])
def test_batch1_both_paths(shape, wdtype, qdtype, force_general):
    _ffn_case(shape, wdtype, qdtype, 1, n_layers=3, via_layers=True, force_general=force_general, seed=31)


@pytest.mark.parametrize("n_layers", [1, 2, 9, 70])
def test_layer_counts(n_layers):
    """Short stacks, and one longer than a set of launches holds."""
    _ffn_case(synth.TINY, torch.bfloat16, torch.bfloat16, 1, n_layers=n_layers, via_layers=True, seed=500)


def test_batch1_is_reproducible():
    sh = synth.GEMMA2_2B
    weights = synth.ffn_stack(sh, 4, base_seed=1000, dtype=torch.bfloat16)
    q = synth.tokens(sh, 1, 2001, torch.bfloat16)
    a = run_gpu_ffn(sh, weights, q, via_layers=True)
    for _ in range(3):
        b = run_gpu_ffn(sh, weights, q, via_layers=True)
        assert np.array_equal(a["y"], b["y"]) and np.array_equal(a["idx"], b["idx"])


@pytest.mark.parametrize("rpb,npb", [(16, 64), (48, 192), (256, 1024), (64, 128)])
def test_block_sizes_of_the_phased_path(rpb, npb):
    """Every split of the neurons into predictor / gather blocks gives the oracle's layer (ragged tails included)."""
    tuning = binding.Tuning(rows_per_predict_block=rpb, neurons_per_gather_block=npb)
    _ffn_case(synth.RAGGED, torch.bfloat16, torch.bfloat16, 1, n_layers=3, via_layers=True, seed=77, tuning=tuning)
    _ffn_case(synth.TINY, torch.float32, torch.float32, 1, n_layers=2, via_layers=True, seed=78, tuning=tuning)


def test_paper_layer_shape_and_9b_shape():
    _ffn_case(synth.PAPER_2B, torch.bfloat16, torch.bfloat16, 1, n_layers=2, via_layers=True, seed=9)
    _ffn_case(synth.GEMMA2_9B, torch.bfloat16, torch.bfloat16, 1, n_layers=2, via_layers=True, seed=10)
    _ffn_case(synth.GEMMA2_9B, torch.bfloat16, torch.bfloat16, 8, n_layers=1, seed=11)


@pytest.mark.parametrize("batch", [1, 4, 16, 64])
def test_gemma2_2b_layer(batch):
    out = _ffn_case(synth.GEMMA2_2B, torch.bfloat16, torch.bfloat16, batch, seed=1000)
    assert np.all(np.abs(out["count"] - 737) < 6 * 26)


def test_gemma2_2b_fp32_weights():
    _ffn_case(synth.GEMMA2_2B, torch.float32, torch.float32, 1, seed=1001)


def test_layers_entry_point_matches_single_calls():
    sh = synth.TINY
    weights = synth.ffn_stack(sh, 5, base_seed=1000, dtype=torch.bfloat16)
    for batch in (1, 4):
        q = synth.tokens(sh, batch, 2000 + batch, torch.bfloat16)
        a = run_gpu_ffn(sh, weights, q, via_layers=True)
        b = run_gpu_ffn(sh, weights, q, via_layers=False)
        check_ffn_against_oracle(sh, weights, q, a, TOL_BF16_TIGHT, what="layers")
        assert np.array_equal(a["idx"], b["idx"]) and np.array_equal(a["uidx"], b["uidx"])
        assert rel_l2(a["y"], b["y"]) < 1e-6


def test_dense_evaluation_gives_the_same_layer():
    sh = synth.TINY
    weights = synth.ffn_stack(sh, 1, base_seed=77, dtype=torch.bfloat16)
    q = synth.tokens(sh, 3, 78, torch.bfloat16)
    dense = run_gpu_ffn(sh, weights, q, dense=True)
    check_ffn_against_oracle(sh, weights, q, dense, TOL_BF16_TIGHT, dense=True, what="dense")
    sparse = run_gpu_ffn(sh, weights, q)
    assert rel_l2(dense["y"], sparse["y"]) < 1e-6


def test_dense_layers_entry_point():
    """Dense evaluation of a stack, phase by phase (batch 1) and layer by layer (batch 3)."""
    for sh, batch, n_layers in ((synth.TINY, 1, 5), (synth.RAGGED, 1, 3), (synth.TINY, 3, 2), (synth.GEMMA2_2B, 1, 2)):
        weights = synth.ffn_stack(sh, n_layers, base_seed=91, dtype=torch.bfloat16)
        q = synth.tokens(sh, batch, 92, torch.bfloat16)
        dense = run_gpu_ffn(sh, weights, q, dense=True, via_layers=True)
        check_ffn_against_oracle(sh, weights, q, dense, TOL_BF16_TIGHT, dense=True, what="dense layers")


def test_batch_members_do_not_influence_each_other():
    sh = synth.TINY
    weights = synth.ffn_stack(sh, 1, base_seed=5, dtype=torch.bfloat16)
    q = synth.tokens(sh, 16, 2016, torch.bfloat16)
    full = run_gpu_ffn(sh, weights, q)
    for b in (0, 9, 15):
        solo = run_gpu_ffn(sh, weights, q[b:b + 1])
        assert np.array_equal(solo["idx"][0, 0], full["idx"][0, b])
        assert rel_l2(solo["y"][0, 0], full["y"][0, b]) < 1e-6


@pytest.mark.parametrize("batch", [1, 4, 64])
@pytest.mark.parametrize("path", [0, 1])
def test_degenerate_layers(batch, path):
    """Constant scores (zero predictor weights): std = 0, theta = mean, nothing is strictly greater, so the
    active sets and the union are empty and y = 0.  And k = d_ff - 1: theta drops so far that almost every
    neuron is active (the gather degenerates to the dense layer)."""
    sh = synth.TINY
    weights = synth.ffn_stack(sh, 2, base_seed=321, dtype=torch.bfloat16)
    q = synth.tokens(sh, batch, 322, torch.bfloat16)
    zeroed = [(torch.zeros_like(w[0]), w[1], w[2]) for w in weights]
    out = run_gpu_ffn(sh, zeroed, q, via_layers=True, force_general=path)
    assert np.all(out["y"] == 0.0) and np.all(out["count"] == 0) and np.all(out["ucount"] == 0)
    assert np.all(out["theta"] == 0.0) and np.all(out["idx"] == -1)
    import dataclasses
    wide = dataclasses.replace(sh, k=sh.d_ff - 1)
    out = run_gpu_ffn(wide, weights, q, via_layers=True, force_general=path)
    check_ffn_against_oracle(wide, weights, q, out, TOL_BF16_TIGHT, what=f"k=d_ff-1 B={batch}")
    assert np.all(out["count"] > 0.99 * sh.d_ff)


def test_batch_sizes_around_the_token_blocks():
    """Batches that do not fill the 16-token blocks of the matrix-core path, and the largest batch."""
    sh = synth.TINY
    weights = synth.ffn_stack(sh, 2, base_seed=55, dtype=torch.bfloat16)
    for batch in (2, 15, 17, 33, 48, 63, 64):
        q = synth.tokens(sh, batch, 56 + batch, torch.bfloat16)
        out = run_gpu_ffn(sh, weights, q, via_layers=True)
        check_ffn_against_oracle(sh, weights, q, out, TOL_BF16_TIGHT, what=f"B={batch}")


@pytest.mark.parametrize("batch", [2, 16, 40])
def test_matrix_core_path_with_a_ragged_number_of_neurons(batch):
    """d_ff that is neither a multiple of the 16-row tiles nor of the 64-bit mask words, on the batched
    matrix-core path (rows of 32-element multiples, so that path is the one that runs)."""
    sh = synth.FFNShape("ragged-dff", 256, 1000, 128, 77)
    weights = synth.ffn_stack(sh, 3, base_seed=611, dtype=torch.bfloat16)
    q = synth.tokens(sh, batch, 612 + batch, torch.bfloat16)
    out = run_gpu_ffn(sh, weights, q, via_layers=True)
    check_ffn_against_oracle(sh, weights, q, out, TOL_BF16_TIGHT, what=f"ragged d_ff B={batch}")


@pytest.mark.parametrize("d_ff", [16384, 16400])
@pytest.mark.parametrize("batch", [1, 5, 33])
def test_most_neurons_the_matrix_core_path_takes_and_one_tile_more(d_ff, batch):
    """The batched matrix-core path keeps the union mask of a layer in 256 words of 64 bits: 16384
    neurons are the most it takes, and a layer with one 16-row tile more goes through the general kernels.
    Batch 1 runs the phase-by-phase kernels at both sizes."""
    sh = synth.FFNShape("wide", 256, d_ff, 128, round(0.08 * d_ff))
    weights = synth.ffn_stack(sh, 2, base_seed=911, dtype=torch.bfloat16)
    q = synth.tokens(sh, batch, 912 + batch, torch.bfloat16)
    out = run_gpu_ffn(sh, weights, q, via_layers=True)
    check_ffn_against_oracle(sh, weights, q, out, TOL_BF16_TIGHT, what=f"d_ff={d_ff} B={batch}")


@pytest.mark.parametrize("d_model,d_ff,r,k", [(1280, 1000, 512, 77), (2304, 600, 1024, 48), (3072, 200, 1536, 20),
                                              (1536, 2085, 768, 160)])
@pytest.mark.parametrize("batch", [17, 32, 40, 64])
def test_staged_kernels_of_several_token_blocks(d_model, d_ff, r, k, batch):
    """More than 16 tokens, rows of whole 512-byte multiples: tiles of 16 rows are brought into LDS
    by whole-row loads and multiplied from there.  Every compiled row length (512 .. 1536), two,
    three and four token blocks (three run as four), ragged numbers of neurons and of union tiles,
    short and long workgroups; against the oracle and against the k-split kernels."""
    sh = synth.FFNShape("staged", d_model, d_ff, r, k)
    for n_layers, block in ((1, 0), (3, 32), (2, 256)):
        weights = synth.ffn_stack(sh, n_layers, base_seed=740 + n_layers, dtype=torch.bfloat16)
        q = synth.tokens(sh, batch, 750 + batch, torch.bfloat16)
        tune = binding.Tuning(rows_per_predict_block=block, neurons_per_gather_block=block)
        out = run_gpu_ffn(sh, weights, q, via_layers=True, tuning=tune)
        check_ffn_against_oracle(sh, weights, q, out, TOL_BF16_TIGHT, what=f"staged B={batch} L={n_layers}")
        other = run_gpu_ffn(sh, weights, q, via_layers=True, tuning=binding.Tuning(variant=100))
        assert np.max(np.abs(out["ucount"].astype(np.int64) - other["ucount"])) <= 2
        assert rel_l2(out["y"], other["y"]) < 1e-3


@pytest.mark.parametrize("d_model,d_ff,r,k", [(1280, 1000, 512, 77), (2304, 600, 1024, 48), (3584, 200, 1536, 20),
                                              (4096, 2085, 2048, 160)])
@pytest.mark.parametrize("batch", [3, 16, 17, 32])
def test_staged_kernels_with_four_and_eight_parts_per_row(d_model, d_ff, r, k, batch):
    """One and two token blocks on the LDS-staged kernels: the rows are split into 4 or 8 parts among
    the compute waves of a token block (2 or 4 with two blocks), which is what lets rows of 2048
    elements in; forced through the tuning switch at 16 tokens and below."""
    sh = synth.FFNShape("staged-parts", d_model, d_ff, r, k)
    for n_layers, block in ((1, 0), (3, 64)):
        weights = synth.ffn_stack(sh, n_layers, base_seed=760 + n_layers, dtype=torch.bfloat16)
        q = synth.tokens(sh, batch, 770 + batch, torch.bfloat16)
        tune = binding.Tuning(rows_per_predict_block=block, neurons_per_gather_block=block, variant=500)
        out = run_gpu_ffn(sh, weights, q, via_layers=True, tuning=tune)
        check_ffn_against_oracle(sh, weights, q, out, TOL_BF16_TIGHT, what=f"staged parts B={batch} L={n_layers}")


@pytest.mark.parametrize("d_model,d_ff,r,k", [(1024, 1000, 512, 77), (2304, 600, 1024, 48), (3584, 40, 1536, 5),
                                              (1024, 2085, 512, 160)])
@pytest.mark.parametrize("batch", [2, 5, 9, 16])
def test_whole_row_kernels_of_one_token_block(d_model, d_ff, r, k, batch):
    """At most 16 tokens, rows of whole 256-byte multiples: a wave reads four consecutive rows whole
    and multiplies on the 4x4x4 matrix instruction.  Every compiled row length (512 .. 2048), one
    to four groups of four tokens, ragged numbers of neurons and of union rows, one and several
    layers, short (64 rows) and long (256 rows) workgroups; against the oracle and against the
    k-split kernels, which read MFMA-shaped pieces."""
    sh = synth.FFNShape("rows4", d_model, d_ff, r, k)
    for n_layers, block in ((1, 0), (3, 256), (2, 64)):
        weights = synth.ffn_stack(sh, n_layers, base_seed=720 + n_layers, dtype=torch.bfloat16)
        q = synth.tokens(sh, batch, 730 + batch, torch.bfloat16)
        tune = binding.Tuning(rows_per_predict_block=block, neurons_per_gather_block=block, variant=400)
        out = run_gpu_ffn(sh, weights, q, via_layers=True, tuning=tune)
        check_ffn_against_oracle(sh, weights, q, out, TOL_BF16_TIGHT, what=f"whole rows B={batch} L={n_layers}")
        other = run_gpu_ffn(sh, weights, q, via_layers=True, tuning=binding.Tuning(variant=100))
        # (a score within rounding of the threshold may fall on either side of it)
        assert np.max(np.abs(out["ucount"].astype(np.int64) - other["ucount"])) <= 2
        assert rel_l2(out["y"], other["y"]) < 1e-3


@pytest.mark.parametrize("batch", [2, 3, 4])
@pytest.mark.parametrize("shape", [synth.GEMMA2_2B, synth.FFNShape("few", 1024, 1000, 520, 77)])
def test_few_tokens(shape, batch):
    """Two to four tokens: the 2B shape (whole-row kernels) and a shape whose rows are not multiples of 32
    elements (general kernels) against the oracle; the 2B shape also against the k-split kernels."""
    weights = synth.ffn_stack(shape, 2, base_seed=800, dtype=torch.bfloat16)
    q = synth.tokens(shape, batch, 810 + batch, torch.bfloat16)
    out = run_gpu_ffn(shape, weights, q, via_layers=True)
    check_ffn_against_oracle(shape, weights, q, out, TOL_BF16_TIGHT, what=f"few tokens B={batch}")
    other = run_gpu_ffn(shape, weights, q, via_layers=True, tuning=binding.Tuning(variant=100))
    assert np.array_equal(out["count"], other["count"]) and np.array_equal(out["idx"], other["idx"])
    assert rel_l2(out["y"], other["y"]) < 1e-6


@pytest.mark.parametrize("shape,batch", [(synth.TINY, 1), (synth.TINY, 4), (synth.TINY, 16),
                                         (synth.FFNShape("graph", 1280, 1000, 512, 77), 4),
                                         (synth.FFNShape("graph", 1280, 1000, 512, 77), 16),
                                         (synth.FFNShape("graph", 1280, 1000, 512, 77), 40)])
def test_calls_can_be_captured_in_a_graph_and_replayed(shape, batch):
    """The library allocates nothing and clears nothing with memset nodes, so a call can sit in a HIP
    graph: three replays, with eager calls on other inputs in between, each give the eager result.
    (The second shape takes the whole-row kernels at 4 and 16 tokens and the LDS-staged ones at 40.)"""
    sh = shape
    dev = torch.device(DEV)
    weights = synth.ffn_stack(sh, 3, base_seed=900, dtype=torch.bfloat16, device=dev)
    layers = [binding.make_layer(w[0], w[1], w[2], sh.k) for w in weights]
    ws = binding.make_workspace(sh.d_model, sh.d_ff, batch, dev)
    q = synth.tokens(sh, batch, 901, torch.bfloat16, dev)
    q_static = q.clone()
    y_graph = torch.zeros(3, batch, sh.d_model, device=dev)
    y_eager = torch.zeros_like(y_graph)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        binding.spark_ffn_decode_layers(layers, q_static, y_graph, ws)      # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        binding.spark_ffn_decode_layers(layers, q_static, y_graph, ws)
    for rep in range(3):
        qr = synth.tokens(sh, batch, 910 + rep, torch.bfloat16, dev)
        q_static.copy_(qr)
        y_graph.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        # eager work on the same workspace between the replays, on other tokens and then on these
        binding.spark_ffn_decode_layers(layers, q, y_eager, ws)
        binding.spark_ffn_decode_layers(layers, qr, y_eager, ws)
        torch.cuda.synchronize()
        assert torch.equal(y_graph, y_eager), rep
