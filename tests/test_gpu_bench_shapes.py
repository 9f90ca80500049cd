"""GPU parity at the launch configurations the benchmark times.

Block sizes, tiles per workgroup, row slices and the choice between kernel variants all depend on
the number of layers in a call and on the batch, so every (shape, layers, batch) that `bench.py`
reports is run here at exactly that size and held to the oracle: every layer's threshold and every
token's active set against the oracle's predictor scores and statistical top-k, the union list of
every layer, and y of the first, a middle and the last layer element by element.
Weights are drawn on the device (as the benchmark does) and copied to the host for the oracle, so
both sides see the same bytes.
"""
import numpy as np
import pytest
import torch

import oracle
import synth
from paper_2506_06644_amd import binding

from parity_util import (BAND, TOL_BF16_TIGHT, assert_active_set, check_ffn_against_oracle, check_union,
                         run_gpu_ffn)

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def check_stack(shape, weights_dev, q, out, what):
    """Every layer / token: theta and the active set against the oracle's statistical top-k of the
    oracle-side predictor scores (float64 GEMM of the same stored weights), and the union list."""
    L, B = len(weights_dev), q.shape[0]
    q1 = synth.to_oracle(q)[:, :shape.r].astype(np.float64)
    for l in range(L):
        k1n = synth.to_oracle(weights_dev[l][0]).astype(np.float64)
        S = q1 @ k1n.T                                              # [B, d_ff]
        ref = oracle.stat_topk_rows(S, shape.k, want_y=False)
        sets, ref_sets, in_band = [], [], np.zeros(shape.d_ff, bool)
        for b in range(B):
            tag = f"{what} layer {l} token {b}"
            assert abs(out["theta"][l, b] - ref.theta[b]) <= 1e-5 * ref.std[b] + 1e-6 * abs(ref.theta[b]), tag
            m = int(out["count"][l, b])
            gidx = out["idx"][l, b, :m]
            assert np.all(np.diff(gidx) > 0) and np.all(out["idx"][l, b, m:] == -1), tag
            assert_active_set(gidx, S[b], ref.theta[b], ref.std[b], tag)
            sets.append(gidx)
            ref_sets.append(ref.idx[b, :int(ref.count[b])])
            in_band |= np.abs(S[b] - ref.theta[b]) < BAND * ref.std[b]
        mu = int(out["ucount"][l])
        assert np.all(out["uidx"][l, mu:] == -1)
        check_union(out["uidx"][l, :mu], sets, ref_sets, in_band, f"{what} layer {l}")


def check_picked_layers(shape, weights_dev, q, out, pick, what):
    L = len(weights_dev)
    sub = {k: (v[pick] if v.shape[0] == L else v) for k, v in out.items()}
    host = [tuple(t.cpu() for t in weights_dev[i]) for i in pick]
    worst = check_ffn_against_oracle(shape, host, q, sub, TOL_BF16_TIGHT, what=what)
    print(f"{what}: worst y rel L2 over layers {pick}: {worst:.2e}", flush=True)


@pytest.fixture(scope="module")
def stack_2b():
    return synth.ffn_stack(synth.GEMMA2_2B, 26, base_seed=1000, dtype=torch.bfloat16, device=DEV)


@pytest.mark.parametrize("batch", [1, 4, 16, 64])
def test_gemma2_2b_stack_of_26_layers(stack_2b, batch):
    sh = synth.GEMMA2_2B
    q = synth.tokens(sh, batch, 2000 + batch, torch.bfloat16)
    out = run_gpu_ffn(sh, stack_2b, q, via_layers=True)
    check_stack(sh, stack_2b, q, out, f"2B x 26 B={batch}")
    check_picked_layers(sh, stack_2b, q, out, [0, 13, 25], f"2B x 26 B={batch}")


def test_gemma2_9b_stack_of_42_layers():
    sh = synth.GEMMA2_9B
    weights = synth.ffn_stack(sh, 42, base_seed=1000, dtype=torch.bfloat16, device=DEV)
    for batch in (1, 8):
        q = synth.tokens(sh, batch, 2000 + batch, torch.bfloat16)
        out = run_gpu_ffn(sh, weights, q, via_layers=True)
        check_stack(sh, weights, q, out, f"9B x 42 B={batch}")
        check_picked_layers(sh, weights, q, out, [0, 20, 41], f"9B x 42 B={batch}")
    del weights
    torch.cuda.empty_cache()


def test_paper_layer_stack_of_26_layers():
    """The layer the paper itself trains (d_ff 13824, k 1106, r 1024), 26 of them in one call, as the
    benchmark's unscored extra shape."""
    sh = synth.PAPER_2B
    weights = synth.ffn_stack(sh, 26, base_seed=1000, dtype=torch.bfloat16, device=DEV)
    q = synth.tokens(sh, 1, 2001, torch.bfloat16)
    out = run_gpu_ffn(sh, weights, q, via_layers=True)
    check_stack(sh, weights, q, out, "paper layer x 26")
    check_picked_layers(sh, weights, q, out, [0, 12, 25], "paper layer x 26")
    del weights
    torch.cuda.empty_cache()
