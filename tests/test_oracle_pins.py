"""Pins for the CPU oracle: what the paper and the mathematics fix, checked without a GPU.

Each pin compares the oracle (plain C loops in double) with something that is not the
oracle: printed / textbook values, closed forms, invariants, library routines for the
special case a step reduces to, brute force on tiny inputs, or 50-digit arithmetic.
"""
import math
import os
import statistics

import numpy as np
import pytest
import scipy.special
import scipy.stats
import torch

import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# --------------------------------------------------------------------------- quantile Q
def test_quantile_textbook_values(oracle):
    rows = [l.split() for l in open(os.path.join(GOLDEN, "normal_quantile.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) >= 10
    for p, q in rows:
        assert oracle.normal_quantile(float(p)) == pytest.approx(float(q), abs=2e-12)


def test_quantile_against_two_library_routines(oracle):
    nd = statistics.NormalDist()
    ps = np.concatenate([np.linspace(1e-6, 1 - 1e-6, 401), [737 / 9216, 1 - 737 / 9216,
                                                             1 - 82 / 1024, 1 - 1147 / 14336,
                                                             1 - 1106 / 13824, 1e-12, 1 - 1e-9]])
    for p in ps:
        got = oracle.normal_quantile(float(p))
        assert got == pytest.approx(float(scipy.special.ndtri(p)), rel=1e-11, abs=1e-12)
        if 1e-9 < p < 1 - 1e-9:
            assert got == pytest.approx(nd.inv_cdf(float(p)), rel=1e-10, abs=1e-11)


def test_quantile_round_trip_symmetry_edges(oracle):
    for p in [1e-10, 0.01, 0.08, 0.3, 0.5, 0.7, 0.92, 0.99, 1 - 1e-10]:
        z = oracle.normal_quantile(p)
        assert scipy.stats.norm.cdf(z) == pytest.approx(p, rel=1e-12)
        if 1e-3 < p < 1 - 1e-3:      # 1 - p is itself rounded, which dominates in the far tail
            assert oracle.normal_quantile(1 - p) == pytest.approx(-z, rel=1e-12, abs=1e-13)
    assert oracle.normal_quantile(0.5) == 0.0
    assert oracle.normal_quantile(0.0) == -math.inf
    assert oracle.normal_quantile(1.0) == math.inf
    assert math.isnan(oracle.normal_quantile(1.5))
    # monotone
    zs = [oracle.normal_quantile(p) for p in np.linspace(0.001, 0.999, 200)]
    assert all(b > a for a, b in zip(zs, zs[1:]))


def test_quantile_values_used_by_the_configs(oracle):
    # z_k for the benchmark shapes, recomputed by an independent routine
    for d, k in [(1024, 82), (9216, 737), (14336, 1147), (13824, 1106)]:
        assert oracle.normal_quantile(1 - k / d) == pytest.approx(
            statistics.NormalDist().inv_cdf(1 - k / d), abs=1e-11)
    assert oracle.normal_quantile(1 - 737 / 9216) == pytest.approx(1.405275953, abs=1e-8)


# --------------------------------------------------------------------------- GELU
def test_gelu_against_library(oracle):
    xs = np.linspace(-6, 6, 241)
    ref_erf = torch.nn.functional.gelu(torch.tensor(xs, dtype=torch.float64)).numpy()
    ref_tanh = torch.nn.functional.gelu(torch.tensor(xs, dtype=torch.float64),
                                        approximate="tanh").numpy()
    for x, a, b in zip(xs, ref_erf, ref_tanh):
        assert oracle.gelu(float(x), oracle.GELU_ERF) == pytest.approx(a, rel=1e-12, abs=1e-15)
        assert oracle.gelu(float(x), oracle.GELU_TANH) == pytest.approx(b, rel=1e-12, abs=1e-15)
    assert oracle.gelu(0.0) == 0.0
    # x * Phi(x) with Phi from a statistics library
    assert oracle.gelu(1.3) == pytest.approx(1.3 * scipy.stats.norm.cdf(1.3), rel=1e-13)


# --------------------------------------------------------------------------- mean / std / theta
def test_threshold_is_mean_plus_std_times_quantile_with_bessel(oracle):
    rng = np.random.default_rng(11)
    for d, k in [(7, 3), (64, 5), (1000, 77), (9216, 737)]:
        x = rng.standard_normal(d) * 3.0 + 1.5
        out = oracle.stat_topk(x, k)
        assert out.mean == pytest.approx(np.mean(x), rel=1e-13, abs=1e-14)
        assert out.std == pytest.approx(np.std(x, ddof=1), rel=1e-13)
        assert out.std == pytest.approx(statistics.stdev(x.tolist()), rel=1e-12)
        z = scipy.special.ndtri(1 - k / d)
        assert out.z == pytest.approx(z, rel=1e-11)
        assert out.theta == pytest.approx(np.mean(x) + np.std(x, ddof=1) * z, rel=1e-11)
        # a 1/d variance would move theta by about std*z/(2d): make sure that is resolved
        wrong = np.mean(x) + np.std(x, ddof=0) * z
        assert abs(out.theta - wrong) > 1e3 * abs(out.theta - (np.mean(x) + np.std(x, ddof=1) * z))


def test_closed_form_single_spike(oracle):
    # x = (c, 0, ..., 0): mean = c/d, std = c/sqrt(d) exactly, so
    # theta = c/d + c z/sqrt(d) and only the spike survives, shifted by theta.
    for d, k, c in [(16, 2, 5.0), (1024, 82, 3.0), (9216, 737, 0.25)]:
        x = np.zeros(d)
        x[d // 3] = c
        out = oracle.stat_topk(x, k)
        z = scipy.special.ndtri(1 - k / d)
        theta = c / d + c * z / math.sqrt(d)
        assert out.theta == pytest.approx(theta, rel=1e-12)
        assert out.count == 1 and out.idx.tolist() == [d // 3]
        assert out.y[d // 3] == pytest.approx(c - theta, rel=1e-12)
        assert np.count_nonzero(out.y) == 1


def test_zero_and_shift_structure(oracle):
    rng = np.random.default_rng(5)
    for d, k in [(33, 4), (1024, 82), (9216, 737)]:
        x = rng.standard_normal(d) * rng.uniform(0.5, 2) + rng.uniform(-1, 1)
        o = oracle.stat_topk(x, k)
        act = x > o.theta
        assert np.array_equal(np.flatnonzero(act), o.idx)
        assert o.count == int(act.sum())
        assert np.all(o.y[~act] == 0.0)
        assert np.all(o.y[act] > 0.0)
        assert np.array_equal(o.y[act], x[act] - o.theta)
        assert o.y.max() == pytest.approx(x.max() - o.theta, rel=1e-14)
        assert o.y.sum() == pytest.approx(x[act].sum() - o.count * o.theta, rel=1e-12)
        assert np.all(np.diff(o.idx) > 0)
        # Soft-Threshold(x, theta) = max(x - theta, 0), the textbook shrinkage operator
        assert np.array_equal(o.y, np.maximum(x - o.theta, 0.0))


def test_neg_inf_fill_variant(oracle):
    rng = np.random.default_rng(6)
    x = rng.standard_normal(257)
    a = oracle.stat_topk(x, 20, oracle.FILL_ZERO)
    b = oracle.stat_topk(x, 20, oracle.FILL_NEG_INF)
    assert a.theta == b.theta and np.array_equal(a.idx, b.idx)
    act = x > a.theta
    assert np.array_equal(b.y[act], a.y[act])
    assert np.all(np.isneginf(b.y[~act]))
    # what the variant is for: softmax puts exactly zero mass on the dropped entries
    w = scipy.special.softmax(b.y)
    assert np.all(w[~act] == 0.0) and w.sum() == pytest.approx(1.0)


def test_tie_at_threshold_is_inactive(oracle):
    # x = (-1, 0, 1) with k chosen so that z = 0 is impossible (k = d/2 needs even d):
    # use d = 4, k = 2 -> Q(1/2) = 0 -> theta = mean; entries equal to the mean stay out.
    x = np.array([-2.0, 0.0, 0.0, 2.0])
    o = oracle.stat_topk(x, 2)
    assert o.z == 0.0 and o.theta == 0.0
    assert o.idx.tolist() == [3] and o.y.tolist() == [0.0, 0.0, 0.0, 2.0]


def test_degenerate_constant_row(oracle):
    o = oracle.stat_topk(np.full(50, 3.25), 7)
    assert o.std == 0.0 and o.theta == 3.25 and o.count == 0 and not o.y.any()


def test_argument_errors(oracle):
    with pytest.raises(ValueError):
        oracle.stat_topk(np.zeros(1), 1)
    for k in (0, 10, -1):
        with pytest.raises(ValueError):
            oracle.stat_topk(np.arange(10.0), k)


# --------------------------------------------------------------------------- P4 nesting, brute force
def test_active_set_is_the_sorted_top_m_set(oracle):
    rng = np.random.default_rng(2)
    for d in (2, 3, 5, 8, 17, 40, 64):
        x = rng.standard_normal(d)
        order = np.argsort(-x, kind="stable")
        for k in range(1, d):
            o = oracle.stat_topk(x, k)
            m = o.count
            assert set(o.idx.tolist()) == set(order[:m].tolist())
            tk = set(oracle.exact_topk(x, k).tolist())
            assert tk == set(order[:k].tolist())
            got = set(o.idx.tolist())
            assert got <= tk if m <= k else tk <= got


def test_exact_topk_matches_library_sort(oracle):
    rng = np.random.default_rng(3)
    x = rng.standard_normal((5, 300))
    idx = oracle.exact_topk_rows(x, 31)
    for r in range(5):
        want = np.sort(torch.topk(torch.tensor(x[r]), 31).indices.numpy())
        assert np.array_equal(idx[r], want)
    # ties go to the lower index
    assert oracle.exact_topk(np.array([1.0, 2.0, 2.0, 2.0, 0.0]), 2).tolist() == [1, 2]


# --------------------------------------------------------------------------- P2 / P3 count ~ k
@pytest.mark.parametrize("d,k,rows", [(1024, 82, 2000), (9216, 737, 1000), (14336, 1147, 600)])
def test_gaussian_rows_keep_about_k_entries(oracle, d, k, rows):
    rng = np.random.default_rng(d)
    x = rng.standard_normal((rows, d)) * 1.7 - 0.3
    out = oracle.stat_topk_rows(x, k, want_y=False, want_idx=False)
    cnt = out.count.astype(np.float64)
    assert abs(cnt.mean() - k) < max(0.005 * k, 4 * math.sqrt(k * (1 - k / d) / rows))
    assert np.all(np.abs(cnt - k) <= 6 * math.sqrt(k * (1 - k / d)))
    # Theorem 1 with delta = 0.01 (never violated; far looser than the above)
    delta = 0.01
    bound = 4 * math.sqrt(math.log(6 / delta) / d) * (1 + math.sqrt(-2 * math.log(min(k / d, 1 - k / d))))
    assert np.all(np.abs(cnt - k) / d <= bound)


def test_predictor_scores_at_random_init_keep_about_k(oracle):
    # weights N(0, 1/d_model), q ~ N(0,1): the "random initialisation" case of Section 4
    sh = synth.TINY
    counts = []
    for seed in range(40):
        k1n, k2n, vn = synth.ffn_layer(sh, 100 + seed, torch.float32)
        q = synth.tokens(sh, 1, 900 + seed, torch.float32)[0]
        o = oracle.spark_ffn(synth.to_oracle(k1n), synth.to_oracle(k2n), synth.to_oracle(vn),
                             synth.to_oracle(q), sh.k, skip_inactive=True)
        counts.append(o.count)
    assert abs(np.mean(counts) - sh.k) < 3.0
    assert 0.06 < np.mean(counts) / sh.d_ff < 0.10       # "about 8% nonzeros" (Fig.3)


# --------------------------------------------------------------------------- P6 equivariance
def test_affine_and_permutation_equivariance(oracle):
    rng = np.random.default_rng(8)
    x = rng.standard_normal(777)
    base = oracle.stat_topk(x, 60)
    for a, b in [(2.0, 0.0), (0.125, 3.0), (7.0, -11.0)]:
        o = oracle.stat_topk(a * x + b, 60)
        assert np.array_equal(o.idx, base.idx)
        assert np.allclose(o.y, a * base.y, rtol=1e-11, atol=1e-12)
        assert o.theta == pytest.approx(a * base.theta + b, rel=1e-11)
    perm = rng.permutation(777)
    o = oracle.stat_topk(x[perm], 60)
    assert o.theta == pytest.approx(base.theta, rel=1e-12)
    assert np.allclose(o.y, base.y[perm], rtol=0, atol=1e-12)
    assert set(perm[o.idx].tolist()) == set(base.idx.tolist())


# --------------------------------------------------------------------------- P7 variational form
def test_soft_threshold_minimises_the_l1_objective(oracle):
    rng = np.random.default_rng(9)
    x = rng.standard_normal(40) + 0.2
    o = oracle.stat_topk(x, 6)
    assert o.theta >= 0

    def obj(zv):
        return o.theta * np.abs(zv).sum() + 0.5 * np.sum((x - zv) ** 2)

    best = obj(o.y)
    for _ in range(300):
        zv = np.maximum(o.y + rng.standard_normal(40) * rng.choice([1e-3, 1e-1, 1.0]), 0.0)
        assert obj(zv) >= best - 1e-12
    # against a generic bounded minimiser
    from scipy.optimize import minimize
    res = minimize(obj, np.ones(40), bounds=[(0, None)] * 40, method="L-BFGS-B",
                   options={"ftol": 1e-15, "gtol": 1e-10, "maxiter": 5000})
    assert np.allclose(res.x, o.y, atol=1e-5)


# --------------------------------------------------------------------------- P8 steps of Eq.2
def _layer(shape, seed, dtype=torch.float32):
    k1n, k2n, vn = synth.ffn_layer(shape, seed, dtype)
    q = synth.tokens(shape, 3, seed + 7, dtype)
    return [synth.to_oracle(t) for t in (k1n, k2n, vn, q)]


@pytest.mark.parametrize("shape", [synth.TINY, synth.RAGGED])
def test_each_step_reduces_to_a_library_routine(oracle, shape):
    k1n, k2n, vn, q = _layer(shape, 1234)
    q = q[0]
    o = oracle.spark_ffn(k1n, k2n, vn, q, shape.k)
    K1 = k1n.astype(np.float64)
    K2 = k2n.astype(np.float64)
    V = vn.astype(np.float64)
    qd = q.astype(np.float64)
    r = shape.r
    # predictor = GEMV with the first r input dims only
    assert np.allclose(o.s, K1 @ qd[:r], rtol=1e-13, atol=1e-15)
    # top-k is the vector routine applied to s
    st = oracle.stat_topk(o.s, shape.k)
    assert np.array_equal(st.y, o.a) and np.array_equal(st.idx, o.idx)
    # u = GELU(a) * (K2^T q[r:]) with a library GELU and a library GEMV
    g = K2 @ qd[r:]
    gel = torch.nn.functional.gelu(torch.tensor(o.a, dtype=torch.float64)).numpy()
    assert np.allclose(o.u, gel * g, rtol=1e-12, atol=1e-18)
    assert np.all(o.u[np.setdiff1d(np.arange(shape.d_ff), o.idx)] == 0.0)
    # y = weighted sum of the active rows of Vn
    assert np.allclose(o.y, V[o.idx].T @ o.u[o.idx], rtol=1e-12, atol=1e-16)
    assert np.allclose(o.y, V.T @ o.u, rtol=1e-12, atol=1e-16)
    # the split is at r: moving mass between the halves of q must matter in the right place
    q2 = q.copy()
    q2[r:] = 0
    o2 = oracle.spark_ffn(k1n, k2n, vn, q2, shape.k)
    assert np.array_equal(o2.s, o.s) and not o2.y.any()
    q3 = q.copy()
    q3[:r] *= 2.0
    o3 = oracle.spark_ffn(k1n, k2n, vn, q3, shape.k)
    assert np.array_equal(o3.idx, o.idx) and np.allclose(o3.a, 2 * o.a, rtol=1e-12)


def test_one_active_neuron_closed_form(oracle):
    # K1n has a single non-zero row -> s is a spike -> exactly one active neuron j and
    # y = GELU(c - theta) * (K2n[j] . q[r:]) * Vn[j]  with theta = c/d + c z / sqrt(d).
    d_model, d_ff, r, k = 12, 30, 5, 3
    rng = np.random.default_rng(4)
    k1n = np.zeros((d_ff, r), np.float32)
    j = 17
    k1n[j] = rng.integers(1, 4, r)
    k2n = rng.integers(-3, 4, (d_ff, d_model - r)).astype(np.float32)
    vn = rng.integers(-3, 4, (d_ff, d_model)).astype(np.float32)
    q = rng.integers(1, 3, d_model).astype(np.float32)
    o = oracle.spark_ffn(k1n, k2n, vn, q, k)
    c = float(k1n[j] @ q[:r])
    theta = c / d_ff + c * scipy.special.ndtri(1 - k / d_ff) / math.sqrt(d_ff)
    assert o.idx.tolist() == [j]
    a = c - theta
    gel = a * scipy.stats.norm.cdf(a)
    want = gel * float(k2n[j] @ q[r:]) * vn[j].astype(np.float64)
    assert np.allclose(o.y, want, rtol=1e-12)


def test_linearity_in_v_and_k2(oracle):
    k1n, k2n, vn, q = _layer(synth.TINY, 77)
    q = q[1]
    o = oracle.spark_ffn(k1n, k2n, vn, q, 82)
    o_v = oracle.spark_ffn(k1n, k2n, 4 * vn, q, 82)
    o_k = oracle.spark_ffn(k1n, -2 * k2n, vn, q, 82)
    assert np.allclose(o_v.y, 4 * o.y, rtol=1e-13)
    assert np.allclose(o_k.y, -2 * o.y, rtol=1e-13)
    assert np.array_equal(o_v.idx, o.idx) and np.array_equal(o_k.idx, o.idx)


def test_against_fifty_digit_arithmetic(oracle):
    import mpmath as mp

    mp.mp.dps = 50
    sh = synth.FFNShape("mp", 24, 40, 10, 6)
    k1n, k2n, vn, q = _layer(sh, 31)
    q = q[2]
    o = oracle.spark_ffn(k1n, k2n, vn, q, sh.k)
    d, r = sh.d_ff, sh.r
    s = [mp.fsum(mp.mpf(float(k1n[j, i])) * mp.mpf(float(q[i])) for i in range(r)) for j in range(d)]
    mean = mp.fsum(s) / d
    std = mp.sqrt(mp.fsum((v - mean) ** 2 for v in s) / (d - 1))
    z = mp.sqrt(2) * mp.erfinv(2 * (1 - mp.mpf(sh.k) / d) - 1)
    theta = mean + std * z
    y = [mp.mpf(0)] * sh.d_model
    active = []
    for j in range(d):
        if s[j] > theta:
            active.append(j)
            a = s[j] - theta
            g = mp.fsum(mp.mpf(float(k2n[j, i])) * mp.mpf(float(q[r + i])) for i in range(sh.r2))
            u = a * mp.ncdf(a) * g
            y = [y[c] + u * mp.mpf(float(vn[j, c])) for c in range(sh.d_model)]
    assert o.idx.tolist() == active
    assert o.theta == pytest.approx(float(theta), rel=1e-13)
    scale = max(abs(float(v)) for v in y)
    for c in range(sh.d_model):
        assert abs(o.y[c] - float(y[c])) <= 1e-13 * scale


# --------------------------------------------------------------------------- P9 sparse == dense, FLOPs
@pytest.mark.parametrize("shape", [synth.TINY, synth.RAGGED])
def test_skipping_inactive_neurons_changes_nothing(oracle, shape):
    k1n, k2n, vn, q = _layer(shape, 4321, torch.bfloat16)
    for b in range(q.shape[0]):
        dense = oracle.spark_ffn(k1n, k2n, vn, q[b], shape.k, skip_inactive=False)
        sparse = oracle.spark_ffn(k1n, k2n, vn, q[b], shape.k, skip_inactive=True)
        assert np.array_equal(dense.y, sparse.y)
        assert np.array_equal(dense.u, sparse.u)
        assert np.array_equal(dense.idx, sparse.idx)
        m, d, r, dff = sparse.count, shape.d_model, shape.r, shape.d_ff
        # Eq.3: the dense form costs 4 d_model d_ff FLOPs
        assert 2 * sum(dense.macs) == 4 * d * dff
        # Eq.4 (with the realised count m in place of k), both of its forms
        assert sparse.macs == (dff * r, m * (d - r), m * d)
        assert 2 * sum(sparse.macs) == 2 * r * dff + 2 * (d - r) * m + 2 * d * m
        assert 2 * sum(sparse.macs) == 2 * (dff - m) * r + 4 * d * m
        # same result for any thread count
        one = oracle.spark_ffn(k1n, k2n, vn, q[b], shape.k, skip_inactive=True, threads=1)
        assert np.array_equal(one.y, sparse.y)


def test_flop_table_of_the_paper():
    # Appendix table: FFN 4 d d_ff -> d d_ff + 3 d k at r = d/2; 3.2x at 8% non-zeros
    d, dff = 2304, 13824
    k = round(0.08 * dff)
    assert k == 1106
    r = d // 2
    sparse = 2 * r * dff + 2 * (d - r) * k + 2 * d * k
    assert sparse == d * dff + 3 * d * k
    assert round(4 * d * dff / sparse, 1) == 3.2
    assert round(1 - sparse / (4 * d * dff), 2) == 0.69   # r = d/2
    r = 1024                                                # the paper's r
    sparse = 2 * r * dff + 2 * (d - r) * k + 2 * d * k
    assert round(1 - sparse / (4 * d * dff), 2) == 0.72   # "-72% FFN FLOPs"


# --------------------------------------------------------------------------- P10 batching
def test_batch_is_token_by_token_and_union_size(oracle):
    sh = synth.TINY
    k1n, k2n, vn, _ = _layer(sh, 55)
    q = synth.to_oracle(synth.tokens(sh, 16, 2016, torch.float32))
    outs, union = oracle.spark_ffn_batch(k1n, k2n, vn, q, sh.k)
    for b in (0, 7, 15):
        solo = oracle.spark_ffn(k1n, k2n, vn, q[b], sh.k, skip_inactive=True)
        assert np.array_equal(solo.y, outs[b].y) and np.array_equal(solo.idx, outs[b].idx)
    assert np.array_equal(union, np.unique(np.concatenate([o.idx for o in outs])))
    expect = sh.d_ff * (1 - (1 - sh.k / sh.d_ff) ** 16)
    assert abs(len(union) - expect) < 0.08 * expect


# --------------------------------------------------------------------------- rows
def test_rows_entry_equals_vector_entry(oracle):
    x = synth.topk_rows(64, 500, seed=1, dtype=torch.float32).numpy().astype(np.float64)
    out = oracle.stat_topk_rows(x, 40)
    for r in (0, 13, 63):
        one = oracle.stat_topk(x[r], 40)
        assert out.theta[r] == one.theta and out.count[r] == one.count
        assert np.array_equal(out.y[r], one.y)
        assert np.array_equal(out.idx[r, : one.count], one.idx)
        assert np.all(out.idx[r, one.count:] == -1)
    one_thread = oracle.stat_topk_rows(x, 40, threads=1)
    assert np.array_equal(one_thread.y, out.y)


# --------------------------------------------------------------------------- Spark attention (Eq.7)
def _attn_case(seed, n_ctx, d_attn, r, scale=0.125):
    rng = np.random.default_rng(seed)
    k1c = (rng.standard_normal((n_ctx, r)) * scale).astype(np.float32)
    k2c = (rng.standard_normal((n_ctx, d_attn - r)) * scale).astype(np.float32)
    vc = rng.standard_normal((n_ctx, d_attn)).astype(np.float32)
    q = rng.standard_normal(d_attn).astype(np.float32)
    return k1c, k2c, vc, q


def test_softplus_values(oracle):
    assert oracle.softplus(0.0) == pytest.approx(math.log(2.0), rel=1e-15)
    for x in (-745.0, -40.0, -3.0, -1e-9, 1e-9, 0.5, 3.0, 40.0, 700.0, 1e6):
        assert oracle.softplus(x) == pytest.approx(float(np.logaddexp(0.0, x)), rel=1e-14, abs=1e-300)
    assert oracle.softplus(800.0) == 800.0 and oracle.softplus(-800.0) == 0.0


def test_attention_with_every_key_kept_is_the_gated_softmax_lookup(oracle):
    """n_ctx <= k: Top_k keeps everything, and Eq.7 is V (softmax(K1^T q1) * softplus(K2^T q2)), here
    with library softmax / logaddexp / matmul in float64."""
    for n_ctx, k in ((40, 40), (17, 256), (1, 5)):
        k1c, k2c, vc, q = _attn_case(n_ctx, n_ctx, 32, 16)
        o = oracle.spark_attention(k1c, k2c, vc, q, k)
        s = k1c.astype(np.float64) @ q[:16].astype(np.float64)
        p = scipy.special.softmax(s)
        g = np.logaddexp(0.0, k2c.astype(np.float64) @ q[16:].astype(np.float64))
        assert o.count == n_ctx and o.theta == -math.inf
        np.testing.assert_allclose(o.p, p, rtol=1e-12, atol=0)
        np.testing.assert_allclose(o.y, vc.astype(np.float64).T @ (p * g), rtol=1e-11, atol=1e-14)


def test_attention_keeps_the_exact_top_m_and_renormalises_over_it(oracle):
    """n_ctx > k: the kept keys are the sort-based top-m (m = count), weights are the softmax over those
    keys only, everything else has weight exactly 0."""
    for seed, n_ctx, k in ((1, 300, 30), (2, 1000, 256), (3, 64, 1), (4, 64, 63)):
        k1c, k2c, vc, q = _attn_case(seed, n_ctx, 48, 24)
        o = oracle.spark_attention(k1c, k2c, vc, q, k)
        s = k1c.astype(np.float64) @ q[:24].astype(np.float64)
        theta = s.mean() + s.std(ddof=1) * float(scipy.special.ndtri(1.0 - k / n_ctx))
        assert o.theta == pytest.approx(theta, rel=1e-11)
        top = np.sort(np.argsort(-s, kind="stable")[:o.count])
        assert np.array_equal(o.idx, top)
        p = np.zeros(n_ctx)
        p[top] = scipy.special.softmax(s[top])
        np.testing.assert_allclose(o.p, p, rtol=1e-12, atol=0)
        assert np.all(o.p[np.setdiff1d(np.arange(n_ctx), top)] == 0.0)
        g = np.logaddexp(0.0, k2c.astype(np.float64) @ q[24:].astype(np.float64))
        np.testing.assert_allclose(o.y, vc.astype(np.float64).T @ (p * g), rtol=1e-11, atol=1e-14)
        sk = oracle.spark_attention(k1c, k2c, vc, q, k, skip_inactive=True)
        assert np.array_equal(sk.y, o.y)          # the skipped terms are exact zeros


def test_attention_closed_forms(oracle):
    k1c, k2c, vc, q = _attn_case(7, 500, 32, 16)
    # (1) zero gate keys: softplus(0) = ln 2; identical values: the convex combination is that value
    v = np.linspace(-1.0, 2.0, 32).astype(np.float32)
    o = oracle.spark_attention(k1c, np.zeros_like(k2c), np.tile(v, (500, 1)), q, 40)
    np.testing.assert_allclose(o.y, math.log(2.0) * v.astype(np.float64), rtol=1e-13)
    # (2) values = identity: y_i = p_i g_i on the kept keys, exactly 0 elsewhere, and sum y_i / g_i = 1
    k1c, k2c, _, q = _attn_case(8, 32, 32, 16)
    o = oracle.spark_attention(k1c, k2c, np.eye(32, dtype=np.float32), q, 6)
    assert 1 <= o.count < 32
    np.testing.assert_allclose(o.y, o.p * o.g, rtol=1e-14)
    off = np.setdiff1d(np.arange(32), o.idx)
    assert np.all(o.y[off] == 0.0)
    assert float(np.sum(o.y[o.idx] / o.g[o.idx])) == pytest.approx(1.0, rel=1e-13)
    # (3) constant scores: nothing exceeds theta = mean, the lookup returns 0
    k1c, k2c, vc, q = _attn_case(9, 100, 32, 16)
    o = oracle.spark_attention(np.zeros_like(k1c), k2c, vc, q, 10)
    assert o.count == 0 and np.all(o.y == 0.0) and o.theta == 0.0


def test_attention_on_a_given_kept_set(oracle):
    """Eq.7 with the kept set handed in: on the oracle's own set it is the oracle's y; on any other set it
    is the library softmax over exactly those keys, gated and applied to the values; an empty set gives 0."""
    for seed, n_ctx, k in ((21, 300, 30), (22, 1000, 256), (23, 17, 40)):
        k1c, k2c, vc, q = _attn_case(seed, n_ctx, 48, 24)
        o = oracle.spark_attention(k1c, k2c, vc, q, k)
        np.testing.assert_allclose(oracle.spark_attention_on_set(k1c, k2c, vc, q, o.idx), o.y, rtol=1e-11, atol=1e-14)
        rng = np.random.default_rng(seed)
        for m in (1, 2, min(n_ctx, 50)):
            kept = np.sort(rng.choice(n_ctx, size=m, replace=False)).astype(np.int32)
            s = k1c[kept].astype(np.float64) @ q[:24].astype(np.float64)
            g = np.logaddexp(0.0, k2c[kept].astype(np.float64) @ q[24:].astype(np.float64))
            want = vc[kept].astype(np.float64).T @ (scipy.special.softmax(s) * g)
            np.testing.assert_allclose(oracle.spark_attention_on_set(k1c, k2c, vc, q, kept), want, rtol=1e-11, atol=1e-14)
        # dropping the weakest kept key changes y by about that key's softmax mass, and is not the same y
        if o.count > 2:
            weakest = o.idx[np.argmin(o.s[o.idx])]
            y2 = oracle.spark_attention_on_set(k1c, k2c, vc, q, o.idx[o.idx != weakest])
            assert not np.array_equal(y2, o.y)
        assert np.all(oracle.spark_attention_on_set(k1c, k2c, vc, q, np.zeros(0, np.int32)) == 0.0)
    with pytest.raises(ValueError):
        oracle.spark_attention_on_set(k1c, k2c, vc, q, np.array([n_ctx], np.int32))


def test_attention_invariances(oracle):
    k1c, k2c, vc, q = _attn_case(11, 400, 32, 16)
    base = oracle.spark_attention(k1c, k2c, vc, q, 50)
    # adding a constant to every score (an extra key feature 1, query entry c) shifts theta and nothing else
    c = 3.25
    k1x = np.concatenate([k1c, np.ones((400, 1), np.float32)], axis=1)
    qx = np.concatenate([q[:16], [np.float32(c)], q[16:]])
    sh = oracle.spark_attention(k1x, k2c, np.concatenate([vc, vc[:, :1]], axis=1), qx, 50)
    assert sh.theta == pytest.approx(base.theta + c, rel=1e-12)
    assert np.array_equal(sh.idx, base.idx)
    np.testing.assert_allclose(sh.y[:32], base.y, rtol=1e-10, atol=1e-13)
    # permuting the keys (rows of all three caches) permutes the kept set and leaves y alone
    perm = np.random.default_rng(12).permutation(400)
    pm = oracle.spark_attention(k1c[perm], k2c[perm], vc[perm], q, 50)
    assert np.array_equal(np.sort(perm[pm.idx]), base.idx)
    np.testing.assert_allclose(pm.y, base.y, rtol=1e-11, atol=1e-14)
    # kept count ~ k on Gaussian scores (Theorem 1), at the paper's attention setting
    counts = []
    for seed in range(20):
        a, b, v, qq = _attn_case(100 + seed, 8192, 32, 16)
        counts.append(oracle.spark_attention(a, b, v, qq, 256).count)
    assert abs(np.mean(counts) - 256) < 12 and min(counts) > 180 and max(counts) < 340


# --------------------------------------------------------------------------- Huber statistical top-k (Eq.13, Eq.14) and its gradient
def test_huber_is_the_library_huber(oracle):
    for delta in (0.05, 0.7, 3.0):
        for x in np.linspace(-5, 5, 41):
            assert oracle.huber(x, delta) == pytest.approx(float(scipy.special.huber(delta, x)), rel=1e-14, abs=1e-300)


def test_huber_stat_topk_piecewise_form_and_limits(oracle):
    """The three cases listed in the proof of Theorem 2 (divided by delta), with the constant of the
    first case taken from the Huber definition (delta^2 / 2: the value that makes the cases meet at
    theta + delta); delta = 0 is StatTop_k itself; 0 <= StatTop_k(x) - y <= delta / 2."""
    rng = np.random.default_rng(21)
    x = rng.standard_normal(500)
    base = oracle.stat_topk(x, 60)
    y0, th0 = oracle.huber_stat_topk(x, 60, 0.0)
    assert np.array_equal(y0, base.y) and th0[0] == base.theta
    for delta in (1e-3, 0.2, 0.9, 50.0):
        y, th = oracle.huber_stat_topk(x, 60, delta)
        assert th[0] == base.theta
        a = x - base.theta
        want = np.where(a > delta, (delta * x - delta * base.theta - 0.5 * delta * delta) / delta,
                        np.where(a >= 0, 0.5 * a * a / delta, 0.0))
        assert np.allclose(y, want, rtol=1e-13, atol=1e-15)
        assert np.all(base.y - y >= -1e-15) and np.all(base.y - y <= delta / 2 + 1e-15)
        assert np.array_equal(y > 0, base.y > 0)
    # the two branches meet at theta + delta, value and slope
    d = 0.37
    assert oracle.huber(d, d) / d == pytest.approx(d / 2, rel=1e-15)
    eps = 1e-7
    assert (oracle.huber(d + eps, d) - oracle.huber(d - eps, d)) / (2 * eps) / d == pytest.approx(1.0, abs=1e-6)


def _fd_jacobian(f, x, h=1e-6):
    J = np.empty((x.size, x.size))
    for j in range(x.size):
        e = np.zeros_like(x)
        e[j] = h
        J[:, j] = (f(x + e) - f(x - e)) / (2 * h)
    return J


@pytest.mark.parametrize("delta", [0.0, 0.05, 0.4, 5.0])
def test_vjp_against_finite_differences_of_the_forward(oracle, delta):
    """The whole Jacobian of the forward operator by central differences (the forward shares no code
    with the gradient's formula), including the path through theta."""
    rng = np.random.default_rng(5)
    d, k = 14, 4
    for trial in range(6):
        x = rng.standard_normal(d) * (0.5 + trial)
        if delta == 0.0:      # stay away from the kinks of plain soft thresholding
            th = oracle.stat_topk(x, k).theta
            if np.min(np.abs(x - th)) < 1e-3:
                continue
        J = _fd_jacobian(lambda v: oracle.huber_stat_topk(v, k, delta)[0], x)
        for _ in range(3):
            gy = rng.standard_normal(d)
            got = oracle.huber_stat_topk_vjp(x, gy, k, delta)
            assert np.allclose(got, gy @ J, rtol=2e-6, atol=2e-7)


@pytest.mark.parametrize("delta", [0.0, 0.3])
def test_vjp_against_automatic_differentiation(oracle, delta):
    """The same operator written with library tensor ops (mean, unbiased std, clamp, where) and
    differentiated by autograd in float64."""
    g = torch.Generator().manual_seed(77)
    rows, d, k = 5, 300, 31
    x = torch.randn(rows, d, generator=g, dtype=torch.float64, requires_grad=True)
    gy = torch.randn(rows, d, generator=g, dtype=torch.float64)
    z = float(scipy.stats.norm.ppf(1 - k / d))
    theta = x.mean(dim=1, keepdim=True) + x.std(dim=1, unbiased=True, keepdim=True) * z
    a = torch.clamp(x - theta, min=0)
    y = a if delta == 0 else torch.where(a < delta, 0.5 * a * a, delta * (a - 0.5 * delta)) / delta
    y.backward(gy)
    got = oracle.huber_stat_topk_vjp(x.detach().numpy(), gy.numpy(), k, delta)
    assert np.allclose(got, x.grad.numpy(), rtol=1e-10, atol=1e-12)
    yo, _ = oracle.huber_stat_topk(x.detach().numpy(), k, delta)
    assert np.allclose(yo, y.detach().numpy(), rtol=1e-12, atol=1e-14)


def test_vjp_invariants(oracle):
    """y does not change when a constant is added to x, so every row of gx sums to zero; plain
    StatTop_k is positively homogeneous of degree one, so gx . x = gy . y (Euler); a constant row
    keeps nothing and gets a zero gradient."""
    rng = np.random.default_rng(31)
    x = rng.standard_normal((7, 200)) * 3 + 1
    gy = rng.standard_normal((7, 200))
    for delta in (0.0, 0.25):
        gx = oracle.huber_stat_topk_vjp(x, gy, 20, delta)
        assert np.allclose(gx.sum(axis=1), 0, atol=1e-12)
    gx = oracle.huber_stat_topk_vjp(x, gy, 20, 0.0)
    y, _ = oracle.huber_stat_topk(x, 20, 0.0)
    assert np.allclose((gx * x).sum(axis=1), (gy * y).sum(axis=1), rtol=1e-11)
    const = np.full(50, 2.5)
    assert np.array_equal(oracle.huber_stat_topk_vjp(const, np.ones(50), 5, 0.1), np.zeros(50))
    assert np.array_equal(oracle.huber_stat_topk(const, 5, 0.1)[0], np.zeros(50))


def test_gradient_is_continuous_with_huber_and_jumps_without(oracle):
    """Theorem 2: move one entry across the threshold; with delta > 0 the gradient changes by an
    amount proportional to the step, with delta = 0 it jumps."""
    rng = np.random.default_rng(41)
    x = rng.standard_normal(120)
    gy = np.ones(120)
    k = 12
    i = int(np.argmin(np.abs(x - oracle.stat_topk(x, k).theta)))

    def active(t):
        v = x.copy()
        v[i] += t
        return v[i] > oracle.stat_topk(v, k).theta

    lo, hi = -1.0, 1.0
    assert not active(lo) and active(hi)
    for _ in range(60):
        mid = 0.5 * (lo + hi)
        lo, hi = (lo, mid) if active(mid) else (mid, hi)
    for delta, smooth in ((0.2, True), (0.0, False)):
        step = []
        for gap in (1e-3, 1e-5):
            a, b = x.copy(), x.copy()
            a[i] += lo - gap
            b[i] += hi + gap
            step.append(np.max(np.abs(oracle.huber_stat_topk_vjp(a, gy, k, delta) -
                                      oracle.huber_stat_topk_vjp(b, gy, k, delta))))
        if smooth:
            assert step[0] < 0.05 and step[1] < step[0] / 50
        else:
            assert step[1] > 0.5


def test_huber_argument_errors(oracle):
    x = np.arange(10.0)
    for bad in (-0.1, float("nan")):
        with pytest.raises(Exception):
            oracle.huber_stat_topk(x, 3, bad)
        with pytest.raises(Exception):
            oracle.huber_stat_topk_vjp(x, x, 3, bad)
    with pytest.raises(Exception):
        oracle.huber_stat_topk_vjp(x, x, 10, 0.1)


# --------------------------------------------------------------------------- 8-bit weight codes (OCP E4M3)
def test_fp8_code_values_against_the_library_type_and_the_format_definition(oracle):
    """All 256 codes against torch's float8_e4m3fn, plus the points the format fixes: bias 7, three
    mantissa bits, subnormals down to 2^-9, largest finite value 448, no infinities, two NaN codes."""
    lib = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float32).numpy()
    for code in range(256):
        v = oracle.fp8_e4m3_value(code)
        if code in (0x7F, 0xFF):
            assert math.isnan(v) and math.isnan(lib[code])
        else:
            assert v == float(lib[code]), code
    assert oracle.fp8_e4m3_value(0x00) == 0.0 and oracle.fp8_e4m3_value(0x38) == 1.0
    assert oracle.fp8_e4m3_value(0x01) == 2.0 ** -9 and oracle.fp8_e4m3_value(0x08) == 2.0 ** -6
    assert oracle.fp8_e4m3_value(0x7E) == 448.0 and oracle.fp8_e4m3_value(0xFE) == -448.0
    assert oracle.fp8_e4m3_value(0x3C) == 1.5 and oracle.fp8_e4m3_value(0xB8) == -1.0


def test_fp8_rows_dequantise_exactly(oracle):
    """The synthetic quantiser keeps scales to 8 significant bits, so scale * value(code) is exact in
    float32: the oracle's weights are the stored weights, and re-quantising them returns the codes."""
    w = synth.ffn_layer(synth.TINY, 3, torch.float32)[0]
    codes, scales = synth.quantize_rows_fp8(w)
    deq = oracle.fp8_dequantize_rows(codes.numpy(), scales.numpy())
    exact = scales.numpy().astype(np.float64)[:, None] * np.vectorize(oracle.fp8_e4m3_value)(codes.numpy())
    assert np.array_equal(deq.astype(np.float64), exact)
    assert np.max(np.abs(deq - w.numpy()) / np.abs(w.numpy()).max(axis=1, keepdims=True)) <= 2.0 ** -4 * 1.01
    again = (torch.from_numpy(deq) / scales[:, None]).to(torch.float8_e4m3fn).view(torch.uint8)
    assert torch.equal(again, codes)


def test_int8_rows_dequantise_exactly(oracle):
    """Signed 8-bit codes: scale * code against numpy's int8 view, exact in float32 with 8-bit scales,
    and the quantiser's round trip."""
    w = synth.ffn_layer(synth.TINY, 4, torch.float32)[2]
    codes, scales = synth.quantize_rows_int8(w)
    deq = oracle.int8_dequantize_rows(codes.numpy(), scales.numpy())
    exact = scales.numpy().astype(np.float64)[:, None] * codes.numpy().view(np.int8).astype(np.float64)
    assert np.array_equal(deq.astype(np.float64), exact)
    assert codes.numpy().view(np.int8).min() >= -127
    assert np.max(np.abs(deq - w.numpy()) / np.abs(w.numpy()).max(axis=1, keepdims=True)) <= 0.5 / 127 * 1.02
    again = torch.round(torch.from_numpy(deq) / scales[:, None]).to(torch.int8).view(torch.uint8)
    assert torch.equal(again, codes)


# ------------------------------------------------ sharded statistical top-k (Appendix D.2)
SHARDINGS = [[0, 2304, 4608, 6912, 9216], [0, 1000, 6000, 9216], [0, 9215, 9216], [0, 9216]]


@pytest.mark.parametrize("bounds", SHARDINGS)
def test_combined_shard_statistics_are_the_statistics_of_the_whole_row(oracle, bounds):
    """Means and variances of the shards, combined as every device would after the exchange, against
    numpy's mean and sample standard deviation of the unsharded rows (shards of very different means)."""
    rng = np.random.default_rng(17)
    x = rng.standard_normal((9, 9216)) * rng.uniform(0.1, 30.0, (9, 1)) + rng.uniform(-50.0, 50.0, (9, 1))
    x[:, :bounds[1]] += 40.0
    ns = [b1 - b0 for b0, b1 in zip(bounds, bounds[1:])]
    stats = [oracle.shard_stats(x[:, b0:b1]) for b0, b1 in zip(bounds, bounds[1:])]
    mean, std = oracle.combine_shard_stats(ns, [s[0] for s in stats], [s[1] for s in stats])
    assert np.allclose(mean, x.mean(axis=1), rtol=1e-13, atol=1e-12)
    assert np.allclose(std, x.std(axis=1, ddof=1), rtol=1e-12)
    for m_, v_ in stats[:1]:
        assert np.allclose(m_, [statistics.fmean(r) for r in x[:, :bounds[1]]], rtol=1e-13, atol=1e-12)


@pytest.mark.parametrize("bounds", SHARDINGS)
@pytest.mark.parametrize("fill", [0, 1])
def test_global_sharded_top_k_is_the_unsharded_operator(oracle, bounds, fill):
    """Appendix D.2: with the exchanged statistics the output is exactly that of the unsharded operator
    (the C oracle on whole rows): thresholds to rounding, identical sets and values."""
    rng = np.random.default_rng(18)
    x = rng.standard_normal((6, 9216)) * 3.0 + 1.5
    x[:, :bounds[1]] -= 2.0
    whole = oracle.stat_topk_rows(x, 737, fill)
    sharded = oracle.stat_topk_sharded(x, 737, bounds, fill)
    assert np.allclose(sharded.theta, whole.theta, rtol=1e-13, atol=1e-13)
    assert np.allclose(sharded.std, whole.std, rtol=1e-12)
    assert np.array_equal(sharded.count, whole.count) and np.array_equal(sharded.idx, whole.idx)
    both = np.isfinite(whole.y)
    assert np.array_equal(both, np.isfinite(sharded.y))
    assert np.allclose(sharded.y[both], whole.y[both], rtol=0, atol=1e-12)


def test_local_sharded_top_k_keeps_its_share_on_every_shard(oracle):
    """Appendix D.2's local variant (k' = k / m on every shard, no exchange): every shard keeps about
    k / m entries whatever its level, while the global variant keeps almost nothing of a shard that lies
    three standard deviations below the others; on identically distributed shards the two keep about the
    same number.  The expected counts come from the normal tail, not from the oracle."""
    rng = np.random.default_rng(19)
    n, m, k = 8192, 4, 656
    bounds = [i * n // m for i in range(m + 1)]
    x = rng.standard_normal((40, n))
    loc = oracle.stat_topk_sharded(x, k, bounds, local=True)
    glo = oracle.stat_topk_sharded(x, k, bounds)
    assert abs(loc.count.mean() - k) < 0.04 * k and abs(glo.count.mean() - k) < 0.04 * k
    for r in range(3):   # per shard, the local variant is the plain operator with k / m
        c0 = 0
        for b0, b1 in zip(bounds, bounds[1:]):
            part = oracle.stat_topk_rows(x[r:r + 1, b0:b1], k // m)
            c = int(part.count[0])
            assert np.array_equal(loc.idx[r, c0:c0 + c], part.idx[0, :c] + b0)
            assert np.allclose(loc.y[r, b0:b1], part.y[0])
            c0 += c
        assert c0 == loc.count[r]
    shifted = x.copy()
    shifted[:, :n // m] -= 3.0
    loc = oracle.stat_topk_sharded(shifted, k, bounds, local=True)
    glo = oracle.stat_topk_sharded(shifted, k, bounds)
    in_first = lambda res: np.mean([(res.idx[r, :res.count[r]] < n // m).sum() for r in range(40)])
    assert abs(in_first(loc) - k / m) < 0.1 * k / m
    # global: the mixture has mean -0.75 and variance 1 + 27/16; a first-shard entry passes the threshold
    # with the normal tail probability of (theta + 3), which is tiny
    z = scipy.special.ndtri(1 - k / n)
    theta = -0.75 + math.sqrt(1 + 27 / 16) * z
    expect = n / m * scipy.stats.norm.sf(theta + 3.0)
    assert in_first(glo) < max(3.0 * expect, 1.0) and expect < 0.5


def test_sharded_top_k_argument_errors(oracle):
    x = np.zeros((2, 64))
    for bad in ([1, 64], [0, 32, 32, 64], [0, 63]):
        with pytest.raises(ValueError):
            oracle.stat_topk_sharded(x, 5, bad)
    with pytest.raises(ValueError):
        oracle.stat_topk_sharded(x, 64, [0, 64])
    with pytest.raises(ValueError):
        oracle.combine_shard_stats([1], [[0.0]], [[0.0]])
