#!/usr/bin/env python3
"""Benchmark of the Spark-FFN sparse decode path on one MI355X.

A "step" is one pass of the whole hot path (predictor, statistical top-k, compaction,
gathered K2 / V products) over every layer of a stack of Gemma-2-2B-shaped layers that is
resident in HBM (26 layers x 84.9 MB = 2.2 GB of weights, 627 MB of them touched per step, so
the weights cannot stay in the 256 MB Infinity Cache), for one batch-1 token vector.  Inputs are
synthetic (weights N(0, 1/d_model) in bf16, token N(0, 1) in bf16) and are on the device before
the timed region starts.

Prints ONE JSON line.  `value` is layers per second; the `roofline` object prices the
dominant kernel (the predictor sweep) against MI355X's 8 TB/s HBM peak on its algorithmic
bytes, with the whole call and the other kernels beside it; `cpu_baseline` is the CPU oracle
timed on the host cores on a bounded sample.

HBM traffic (`roofline.traffic`) is measured in the same run: before this process touches the
GPU it starts `rocprofv3 --pmc FETCH_SIZE` and `rocprofv3 --pmc WRITE_SIZE` over
`python3 bench.py --traffic-probe` (the same workload, a few calls) and scales each counter by
what it reads for the library's plain copy kernel of known size.  If the profiler is missing or a
run fails, `traffic` is null and `traffic_note` says why.
"""
from __future__ import annotations

import argparse
import csv
import glob
import json
import os
import shutil
import signal
import subprocess
import sys
import tempfile
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
CAL_COPY_BYTES = 256 << 20   # size of the calibration copy in the traffic probe


# ------------------------------------------------------------------------------- HBM traffic
def traffic_probe(args):
    """Child of `measure_traffic` (runs under rocprofv3 --pmc): a few calls of the main workload, of
    the row-wise top-k kernels and of the plain copy kernel.  Prints nothing that is parsed."""
    import torch

    import synth
    from paper_2506_06644_amd import binding

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    src = torch.full((CAL_COPY_BYTES,), 7, dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    for _ in range(3):
        binding.spark_copy_bytes(dst, src)
    torch.cuda.synchronize()
    del src, dst
    shape = synth.SHAPES[args.shape]
    L, B = args.layers, args.batch
    weights = synth.ffn_stack(shape, L, base_seed=1000, dtype=torch.bfloat16, device=dev)
    q = synth.tokens(shape, B, 2000 + B, dtype=torch.bfloat16, device=dev)
    layers = [binding.make_layer(w[0], w[1], w[2], shape.k) for w in weights]
    ws = binding.make_workspace(shape.d_model, shape.d_ff, B, dev)
    y = torch.empty(L, B, shape.d_model, device=dev)
    for _ in range(4):
        binding.spark_ffn_decode_layers(layers, q, y, ws)
    torch.cuda.synchronize()
    del weights, layers, ws, y
    if not args.no_stat_topk:
        rows, n, k = 8192, 9216, 737
        for dt in (torch.bfloat16, torch.float32):
            x = synth.topk_rows(rows, n, seed=4242, dtype=dt, device=dev)
            out = torch.empty_like(x)
            gy = synth.grad_rows(rows, n, seed=4243, dtype=dt, device=dev)
            theta = torch.empty(rows, device=dev)
            count = torch.empty(rows, dtype=torch.int32, device=dev)
            for _ in range(2):
                binding.spark_stat_topk(x, k, y=out, theta=theta, count=count)
                binding.spark_stat_topk_huber_backward(x, gy, k, 0.25, out)
            torch.cuda.synchronize()
            del x, out, gy
    print("traffic probe done", flush=True)


def _counter_rows(out_dir, counter):
    """[(kernel name, value)] of one rocprofv3 --pmc run written as csv."""
    rows = []
    for path in glob.glob(os.path.join(out_dir, "**", "*counter_collection.csv"), recursive=True):
        with open(path, newline="") as f:
            for rec in csv.DictReader(f):
                if rec.get("Counter_Name") == counter:
                    rows.append((rec.get("Kernel_Name", ""), float(rec.get("Counter_Value", "nan"))))
    return rows


def measure_traffic(args):
    """HBM bytes per dispatch of every kernel of the workload: FETCH_SIZE and WRITE_SIZE (KiB per
    dispatch, one counter per profiler run) of `bench.py --traffic-probe`, each scaled by the factor
    that makes the counter of the plain copy kernel equal to the bytes it is known to move.
    Returns ({kernel name: {"fetch_bytes", "write_bytes", "dispatches"}}, note)."""
    rocprof = shutil.which("rocprofv3") or "/opt/rocm/bin/rocprofv3"
    if not os.path.exists(rocprof):
        return None, "rocprofv3 not found"
    per_counter, notes = {}, []
    for counter in ("FETCH_SIZE", "WRITE_SIZE"):
        out_dir = tempfile.mkdtemp(prefix="spark_traffic_", dir="/tmp")
        cmd = [rocprof, "--pmc", counter, "-d", out_dir, "-o", "t", "-f", "csv", "--", sys.executable,
               os.path.join(ROOT, "bench.py"), "--traffic-probe", "--shape", args.shape, "--layers", str(args.layers),
               "--batch", str(args.batch)] + (["--no-stat-topk"] if args.no_stat_topk else [])
        env = dict(os.environ, TMPDIR="/tmp")
        try:
            proc = subprocess.Popen(cmd, cwd="/tmp", env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT,
                                    start_new_session=True, text=True)
            try:
                log, _ = proc.communicate(timeout=args.traffic_timeout)
            except subprocess.TimeoutExpired:
                os.killpg(proc.pid, signal.SIGKILL)
                proc.communicate()
                return None, f"rocprofv3 --pmc {counter} did not finish within {args.traffic_timeout} s"
            if proc.returncode != 0 or "traffic probe done" not in log:
                return None, f"rocprofv3 --pmc {counter} failed (exit {proc.returncode}): {log[-300:]!r}"
            rows = _counter_rows(out_dir, counter)
        except OSError as e:
            return None, f"could not run rocprofv3: {e}"
        finally:
            shutil.rmtree(out_dir, ignore_errors=True)
        if not rows:
            return None, f"rocprofv3 --pmc {counter} wrote no counter rows"
        per_kernel = {}
        for name, val in rows:
            per_kernel.setdefault(name, []).append(val)
        cal = [v for name, vals in per_kernel.items() if "copy_bytes_kernel" in name for v in vals]
        if not cal or not sum(cal) > 0:
            return None, f"the calibration copy does not appear in the {counter} run"
        scale = CAL_COPY_BYTES / (sum(cal) / len(cal))      # bytes per counter unit
        notes.append(f"{counter} x {scale / 1024:.3f} KiB")
        per_counter[counter] = {name: (sum(v) / len(v) * scale, len(v)) for name, v in per_kernel.items()}
    out = {}
    for name, (fb, n) in per_counter["FETCH_SIZE"].items():
        wb = per_counter["WRITE_SIZE"].get(name, (0.0, 0))[0]
        out[name] = {"fetch_bytes": fb, "write_bytes": wb, "dispatches": n}
    return out, ("two rocprofv3 --pmc runs of `bench.py --traffic-probe` in this run; counter units from the "
                 f"{CAL_COPY_BYTES >> 20} MiB copy kernel: " + ", ".join(notes))


def traffic_of(traffic, *needles):
    """fetch + write bytes per dispatch of the one kernel whose name contains every needle (None if
    traffic was not measured or the kernel did not run in the probe)."""
    if not traffic:
        return None
    hits = [v for name, v in traffic.items() if all(n in name for n in needles)]
    if len(hits) != 1:
        return None
    return hits[0]["fetch_bytes"] + hits[0]["write_bytes"]


def algorithmic_bytes(shape, counts, wbytes):
    """Weights the method must touch for one token in one layer: K1n fully, K2n and Vn at the
    active rows only.  `counts` = measured active count per layer."""
    per_layer = [wbytes * (shape.d_ff * shape.r + m * shape.r2 + m * shape.d_model) for m in counts]
    return per_layer


def time_region(fn, steps, warmup, torch):
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(steps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    return e0.elapsed_time(e1) * 1e-3, wall


def back_to_back_time(fn, n, torch):
    """Average duration of `n` back-to-back calls of `fn` between one event pair on the stream
    the library launches on (torch's current stream): for a call that is a single kernel launch
    this is the kernel's duration (consecutive launches on one stream do not overlap)."""
    a = torch.cuda.Event(enable_timing=True)
    b = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    a.record()
    for _ in range(n):
        fn()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) * 1e-3 / n


def sampled_launch_time(fn, samples, torch):
    """Average duration of single launches of `fn`, each bracketed by its own event pair on
    the stream the library launches on (torch's current stream)."""
    evs = []
    for _ in range(samples):
        a = torch.cuda.Event(enable_timing=True)
        b = torch.cuda.Event(enable_timing=True)
        a.record()
        fn()
        b.record()
        evs.append((a, b))
    torch.cuda.synchronize()
    ts = sorted(a.elapsed_time(b) * 1e-3 for a, b in evs)
    return sum(ts) / len(ts), ts[len(ts) // 2]


def cpu_baseline(shape, weights_cpu, q_cpu, budget_s=12.0):
    """The CPU oracle as it stands (skip-inactive form, OpenMP over neurons) on one layer of
    the same workload, repeated for about `budget_s` seconds."""
    import oracle

    k1n, k2n, vn = weights_cpu
    oracle.spark_ffn(k1n, k2n, vn, q_cpu, shape.k, skip_inactive=True)  # warm
    n, t0 = 0, time.perf_counter()
    while True:
        oracle.spark_ffn(k1n, k2n, vn, q_cpu, shape.k, skip_inactive=True)
        n += 1
        dt = time.perf_counter() - t0
        if dt >= budget_s or n >= 200000:
            break
    return {"value": n / dt, "unit": "layers/s", "cores": oracle.max_threads(), "kind": "oracle",
            "sample": f"{n} evaluations of layer 0 of the same stack (batch 1), {dt:.1f} s"}


def stat_topk_bench(torch, binding, synth, dev, with_cpu, traffic, np):
    """Row-wise statistical top-k on the 8192 x 9216 activation matrix (k = 737), bf16 and fp32:
    one read and one write of the tensor are the algorithmic bytes.  With the oracle at hand, the
    active sets of a row sample are compared with exact sort-based top-k on the same rows (Section 3's
    cost argument: 2d flops for the statistics against a sort), and both are timed on the host."""
    rows, n, k = 8192, 9216, 737
    out = {"workload": f"rows={rows} n={n} k={k}, rows N(mu_i, sigma_i^2) with 1% Student-t3 outliers"}
    for name, dt, w, tname in (("bf16", torch.bfloat16, 2, "spark::bf16_t"), ("f32", torch.float32, 4, "float")):
        x = synth.topk_rows(rows, n, seed=4242, dtype=dt, device=dev)
        y = torch.empty_like(x)
        theta = torch.empty(rows, device=dev)
        count = torch.empty(rows, dtype=torch.int32, device=dev)

        def step():
            binding.spark_stat_topk(x, k, y=y, theta=theta, count=count)

        gpu_s, _ = time_region(step, 50, 5, torch)
        avg_s, _ = sampled_launch_time(step, 20, torch)
        nbytes = 2.0 * rows * n * w + 8.0 * rows
        cnt = count.cpu().numpy()
        # the launch duration is the average over the 50 launches between one pair of events: the
        # kernel writes as much as it reads, and an event pair of its own around every launch adds the
        # markers' own 4 - 5 us to a 50 us kernel (reported beside it); rocprofv3's kernel average
        # (profiles/stat_topk_8192x9216.md) agrees with the former
        per_s = gpu_s / 50
        out[name] = {"rows_per_s": rows / per_s, "us_per_call": per_s * 1e6,
                     "roofline": {"bound": "hbm", "achieved": nbytes / per_s / 1e9, "peak": HBM_PEAK_GBS,
                                  "unit": "GB/s", "frac": nbytes / per_s / 1e9 / HBM_PEAK_GBS,
                                  "traffic": traffic_of(traffic, "stat_topk_cached_kernel<" + tname),
                                  "kernel": "stat_topk_cached_kernel", "bytes_per_launch": nbytes,
                                  "launch_us": per_s * 1e6, "launch_us_between_own_events": avg_s * 1e6},
                     "count_mean": float(cnt.mean()), "count_std": float(cnt.std()), "count_min": int(cnt.min()),
                     "count_max": int(cnt.max())}
        # backward pass of the Huber-smoothed operator (gradient through theta): x and gy read
        # once, gx written once
        gy = synth.grad_rows(rows, n, seed=4243, dtype=dt, device=dev)

        def back():
            binding.spark_stat_topk_huber_backward(x, gy, k, 0.25, y)

        bavg_s, _ = sampled_launch_time(back, 20, torch)
        bgpu_s, _ = time_region(back, 50, 5, torch)
        bper_s = bgpu_s / 50
        bbytes = 3.0 * rows * n * w
        out[name]["backward"] = {"us_per_call": bper_s * 1e6, "rows_per_s": rows / bper_s, "delta": 0.25,
                                 "roofline": {"bound": "hbm", "achieved": bbytes / bper_s / 1e9, "peak": HBM_PEAK_GBS,
                                              "unit": "GB/s", "frac": bbytes / bper_s / 1e9 / HBM_PEAK_GBS,
                                              "traffic": traffic_of(traffic, "stat_topk_vjp_cached_kernel<" + tname),
                                              "kernel": "stat_topk_vjp_cached_kernel",
                                              "bytes_per_launch": bbytes, "launch_us": bper_s * 1e6,
                                              "launch_us_between_own_events": bavg_s * 1e6}}
        del gy
        # one device's share of the same rows sharded four ways by columns (Appendix D.2, global variant):
        # statistics of its shard, the combination of the four shards' statistics, thresholding of its
        # shard; the shard is read twice and written once
        m_sh = 4
        ns = n // m_sh
        stats = torch.zeros(m_sh, rows, 2, device=dev)
        for s_ in range(m_sh):
            binding.spark_stat_topk_shard_stats(x[:, s_ * ns:(s_ + 1) * ns], stats[s_])
        th = torch.empty(rows, device=dev)

        def shard_share():
            binding.spark_stat_topk_shard_stats(x[:, :ns], stats[0])
            binding.spark_stat_topk_combine_stats(stats, [ns] * m_sh, k, th)
            binding.spark_stat_topk_apply(x[:, :ns], th, binding.FILL_ZERO, y[:, :ns], count)

        sh_s, _ = time_region(shard_share, 20, 3, torch)
        sbytes = 3.0 * rows * ns * w
        out[name]["sharded_global"] = {"shards": m_sh, "us_per_device_share": sh_s / 20 * 1e6,
                                       "algorithmic_bytes": sbytes, "achieved_gbs": sbytes / (sh_s / 20) / 1e9,
                                       "hbm_frac": sbytes / (sh_s / 20) / 1e9 / HBM_PEAK_GBS,
                                       "note": "three launches per share (statistics, combination, thresholding); "
                                               "the exchange of 8 bytes per row and shard is not part of it"}
        del stats, th
        if with_cpu:
            import oracle
            # the GPU's active sets of the first `sample` rows against exact sort-based top-k of the
            # same rows (oracle): precision |I n T_k| / |I|, recall |I n T_k| / k, and nesting (a
            # threshold set is the exact top-|I| set, so it contains T_k or is contained in it)
            sample, cap = 1024, 2048
            idx = torch.full((sample, cap), -1, dtype=torch.int32, device=dev)
            binding.spark_stat_topk(x[:sample], k, count=count[:sample], idx=idx)
            torch.cuda.synchronize()
            xs = synth.to_oracle(x[:sample]).astype(np.float64)
            gi, gc = idx.cpu().numpy(), count[:sample].cpu().numpy().astype(np.int64)
            t0 = time.perf_counter()
            tk = oracle.exact_topk_rows(xs, k)
            t_exact = time.perf_counter() - t0
            t0 = time.perf_counter()
            ref = oracle.stat_topk_rows(xs, k, want_y=True, want_idx=True)
            t_stat = time.perf_counter() - t0
            in_tk = np.zeros((sample, n), bool)
            in_tk[np.arange(sample)[:, None], tk] = True
            valid = np.arange(cap)[None, :] < gc[:, None]
            hit = np.zeros((sample, cap), bool)
            hit[valid] = in_tk[np.broadcast_to(np.arange(sample)[:, None], gi.shape)[valid], gi[valid]]
            inter = hit.sum(1)
            out[name]["vs_exact_topk"] = {
                "rows": sample, "precision_mean": float((inter / np.maximum(gc, 1)).mean()),
                "recall_mean": float((inter / k).mean()), "recall_min": float((inter / k).min()),
                "nested_rows": int((inter == np.minimum(gc, k)).sum()),
                "count_equals_oracle_rows": int((gc == ref.count).sum()),
                "oracle_exact_topk_rows_per_s": sample / t_exact, "oracle_stat_topk_rows_per_s": sample / t_stat,
                "cores": oracle.max_threads()}
            del idx
        if with_cpu and name == "f32":
            import oracle
            sample = 512
            xs = synth.to_oracle(x[:sample])
            t0 = time.perf_counter()
            reps = 0
            while time.perf_counter() - t0 < 3.0:
                oracle.stat_topk_rows(xs, k)
                reps += 1
            dt_s = time.perf_counter() - t0
            t0, ereps = time.perf_counter(), 0
            while time.perf_counter() - t0 < 3.0:
                oracle.exact_topk_rows(xs, k)
                ereps += 1
            et_s = time.perf_counter() - t0
            out["cpu_baseline"] = {"value": sample * reps / dt_s, "unit": "rows/s", "cores": oracle.max_threads(),
                                   "kind": "oracle", "sample": f"{reps} passes over the first {sample} rows (fp32), {dt_s:.1f} s",
                                   "exact_sort_topk_rows_per_s": sample * ereps / et_s,
                                   "exact_sort_topk_sample": f"{ereps} passes of the sort-based exact top-k over the same rows, {et_s:.1f} s"}
        del x, y
    return out


def time_config(torch, binding, shape, layers, q, dev, steps=20):
    """One stack / batch: us per layer and fraction of 8 TB/s on the algorithmic bytes (all of K1n,
    plus the K2n and Vn rows of the union of the tokens' active sets)."""
    L, B = len(layers), q.shape[0]
    ws = binding.make_workspace(shape.d_model, shape.d_ff, B, dev)
    y = torch.empty(L, B, shape.d_model, device=dev)
    ucnt = torch.zeros(L, dtype=torch.int32, device=dev)
    binding.spark_ffn_decode_layers(layers, q, y, ws, union_count=ucnt)
    torch.cuda.synchronize()
    union = ucnt.cpu().numpy()
    nbytes = float(sum(algorithmic_bytes(shape, [int(m) for m in union], 2)))
    gpu_s, _ = time_region(lambda: binding.spark_ffn_decode_layers(layers, q, y, ws), steps, 3, torch)
    per_call = gpu_s / steps
    del ws, y
    return {"shape": shape.name, "layers": L, "batch": B, "us_per_layer": per_call / L * 1e6,
            "layers_per_s": L / per_call, "tokens_per_s": B / per_call, "union_size_mean": float(union.mean()),
            "algorithmic_bytes_per_layer": nbytes / L, "achieved_gbs": nbytes / per_call / 1e9,
            "hbm_frac": nbytes / per_call / 1e9 / HBM_PEAK_GBS}


def other_configs(torch, binding, synth, dev, main_shape, L, weights, layers):
    """The batched decode configurations on the same stack, the Gemma-2-9B-shaped stack at batch 1
    and 8 (42 layers, 8.6 GB of weights), and 26 layers of the paper's own layer shape at batch 1."""
    res = []
    shape = synth.SHAPES[main_shape]
    for B in (4, 16, 64):
        q = synth.tokens(shape, B, 2000 + B, dtype=torch.bfloat16, device=dev)
        res.append(time_config(torch, binding, shape, layers, q, dev))
    if main_shape == "gemma2-2b":
        shape9 = synth.SHAPES["gemma2-9b"]
        w9 = synth.ffn_stack(shape9, 42, base_seed=1000, dtype=torch.bfloat16, device=dev)
        l9 = [binding.make_layer(w[0], w[1], w[2], shape9.k) for w in w9]
        for B in (1, 8):
            q = synth.tokens(shape9, B, 2000 + B, dtype=torch.bfloat16, device=dev)
            res.append(time_config(torch, binding, shape9, l9, q, dev))
        del w9, l9
        torch.cuda.empty_cache()
        # the layer the paper itself trains (Section 4.1: d_ff 13824, k 1106, r 1024), 26 of them
        shp = synth.SHAPES["spark-paper-2b"]
        wp = synth.ffn_stack(shp, 26, base_seed=1000, dtype=torch.bfloat16, device=dev)
        lp = [binding.make_layer(w[0], w[1], w[2], shp.k) for w in wp]
        res.append(time_config(torch, binding, shp, lp, synth.tokens(shp, 1, 2001, dtype=torch.bfloat16, device=dev), dev))
        del wp, lp
        torch.cuda.empty_cache()
    return res


def attention_bench(torch, binding, synth, dev, with_cpu):
    """One decode step of Spark attention at the paper's Gemma-2-2B setting: 26 layers x 4 key / value
    heads (104 caches of 8192 keys, token-major, bf16), 2 query heads per cache, d_attn 256, r 128, at
    most 256 attended keys.  Algorithmic bytes: all of the k1c caches, plus the k2c and vc rows of the
    kept keys of every query head."""
    H, group, n_ctx, d_attn, r, k = 104, 2, 8192, 256, 128, 256
    caches = [synth.attn_caches(n_ctx, d_attn, r, 3000 + h, torch.bfloat16, dev) for h in range(H)]
    q = synth.attn_queries(H, group, d_attn, 3999, torch.bfloat16, dev)
    heads = [binding.make_attn_head(c[0], c[1], c[2], k, group) for c in caches]
    ws = torch.empty(binding.attn_workspace_bytes(H, group, n_ctx), dtype=torch.uint8, device=dev)
    y = torch.empty(H, group, d_attn, device=dev)
    cnt = torch.zeros(H, group, dtype=torch.int32, device=dev)
    binding.spark_attn_decode(heads, q, y, ws, kept_count=cnt)
    torch.cuda.synchronize()
    kept = cnt.cpu().numpy().astype(float)

    def step():
        binding.spark_attn_decode(heads, q, y, ws)

    gpu_s, _ = time_region(step, 100, 10, torch)
    per = gpu_s / 100
    nbytes = 2.0 * (H * n_ctx * r + kept.sum() * ((d_attn - r) + d_attn))
    dense_bytes = 2.0 * H * n_ctx * 2 * d_attn
    out = {"workload": f"{H} caches x {n_ctx} keys, {group} query heads per cache, d_attn={d_attn} r={r} k={k}, bf16",
           "us_per_step": per * 1e6, "query_heads_per_s": H * group / per, "kept_mean": float(kept.mean()),
           "kept_min": int(kept.min()), "kept_max": int(kept.max()), "algorithmic_bytes": nbytes,
           "achieved_gbs": nbytes / per / 1e9, "hbm_frac": nbytes / per / 1e9 / HBM_PEAK_GBS,
           "dense_attention_bytes": dense_bytes}
    if with_cpu:
        import oracle
        k1c, k2c, vc = (synth.to_oracle(t) for t in caches[0])
        q0 = synth.to_oracle(q[0, 0])
        t0, n = time.perf_counter(), 0
        while time.perf_counter() - t0 < 4.0:
            oracle.spark_attention(k1c, k2c, vc, q0, k, skip_inactive=True)
            n += 1
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": n / dt, "unit": "query heads/s", "cores": 1, "kind": "oracle",
                               "sample": f"{n} evaluations of query head 0 of the same step, {dt:.1f} s"}
    return out


def prefill_bench(torch, binding, synth, dev, np):
    """A 4096-token prompt through one Gemma-2-2B-shaped Spark-FFN layer in chunks of 8, 16, 32 and 64
    tokens (the paper's prefill set-up uses 64: Section 4.3; Appendix C.3 places the point where the
    batched path turns from memory-bound to FLOP-bound near 64).  Tokens are independent N(0,1) rows, so
    a chunk's union grows from 49 % of the neurons at 8 tokens to nearly all of them at 64.  All chunks
    read the same layer's 85 MB of weights, which stay in the Infinity Cache: the rate is reported as
    tokens/s and as matrix-core throughput, on the flops the individual masks ask for (2*d_ff*r +
    2*m_t*(2*d_model - r) per token) and on the flops the tiles execute (every union row for every token
    of the chunk, the V product on three bf16 planes of the activations)."""
    sh, T = synth.GEMMA2_2B, 4096
    w = synth.ffn_layer(sh, 1000, torch.bfloat16, dev)
    q = synth.tokens(sh, T, 7000, torch.bfloat16, dev)
    layer = binding.make_layer(w[0], w[1], w[2], sh.k)
    y = torch.empty(T, sh.d_model, device=dev)
    cnt = torch.zeros(T, dtype=torch.int32, device=dev)
    r2 = sh.d_model - sh.r
    out = {"workload": f"{T} tokens through one gemma2-2b-shaped layer, bf16, by chunk size", "by_chunk": []}
    for chunk in (8, 16, 32, 64):
        ws = binding.make_prefill_workspace(sh.d_model, sh.d_ff, chunk, dev)
        ucnt = torch.zeros(T // chunk, dtype=torch.int32, device=dev)
        binding.spark_ffn_prefill(layer, q, chunk, y, ws, active_count=cnt, union_count=ucnt)
        torch.cuda.synchronize()
        m = cnt.cpu().numpy().astype(np.float64)
        u = ucnt.cpu().numpy().astype(np.float64)

        def step():
            binding.spark_ffn_prefill(layer, q, chunk, y, ws)

        gpu_s, _ = time_region(step, 10, 2, torch)
        per = gpu_s / 10
        flops_masks = float(np.sum(2.0 * sh.d_ff * sh.r + 2.0 * m * (r2 + sh.d_model)))
        flops_tiles = float(np.sum(chunk * (2.0 * sh.d_ff * sh.r + 2.0 * u * (r2 + 3 * sh.d_model))))
        weight_bytes = float(np.sum(2.0 * (sh.d_ff * sh.r + u * (r2 + sh.d_model))))
        out["by_chunk"].append({
            "chunk": chunk, "us_per_call": per * 1e6, "us_per_chunk": per * 1e6 / (T // chunk), "tokens_per_s": T / per,
            "union_size_mean": float(u.mean()), "tflops_on_individual_masks": flops_masks / per / 1e12,
            "tflops_executed_by_tiles": flops_tiles / per / 1e12, "mfma_frac_executed": flops_tiles / per / 1e12 / 2500.0,
            "weight_bytes_fetched_per_call": weight_bytes, "weight_fetch_gbs": weight_bytes / per / 1e9})
        del ws
    # comparison point, library GEMMs (not this library's code): the same 4096 tokens through the same
    # layer evaluated densely as three bf16 matrix products (scores and gate products for every neuron,
    # then all of V) - what a matrix-core GPU does with a long prompt when it ignores the sparsity
    k1t, k2t, vt = w[0].t().contiguous(), w[1].t().contiguous(), w[2]

    def dense_gemms():
        s_ = q[:, :sh.r] @ k1t
        g_ = q[:, sh.r:] @ k2t
        return (torch.nn.functional.gelu(s_.float()).to(torch.bfloat16) * g_) @ vt

    d_s, _ = time_region(dense_gemms, 10, 3, torch)
    out["dense_library_gemms"] = {"us_per_call": d_s / 10 * 1e6, "tokens_per_s": T / (d_s / 10),
                                  "tflops": 2.0 * T * sh.d_ff * 2 * sh.d_model / (d_s / 10) / 1e12,
                                  "note": "torch matmuls on bf16, dense layer without the top-k: a reference for what the "
                                          "matrix cores deliver on a long prompt, not a result of this library"}
    last = out["by_chunk"][-1]
    out.update({k: last[k] for k in ("us_per_chunk", "tokens_per_s", "mfma_frac_executed")})
    out["active_count_mean"] = float(m.mean())
    out["note"] = ("weights come from cache (all chunks read one layer), so the weight fetch rate may exceed the HBM "
                   "peak; the top-level figures are those of chunk 64")
    return out


def fp8_bench(torch, binding, synth, dev, np, kind="fp8"):
    """Batch-1 decode with 8-bit weight rows (OCP E4M3 or signed 8-bit integer codes + one fp32 scale per row; Appendix D.4's
    quantisation synergy): the Gemma-2-2B-shaped layers of the main benchmark quantised row by row, 52
    of them so that a step still touches more than the 256 MB Infinity Cache (26 would touch 314 MB).
    Algorithmic bytes per layer: d_ff (r + 4) for the predictor, m (2 d_model - r + 8) for the m
    active neurons' rows and scales."""
    sh, L = synth.GEMMA2_2B, 52
    packed = []
    for l in range(L):
        w = synth.ffn_layer(sh, 1000 + l, torch.float32, dev)
        layer_arrays = []
        for t in w:
            quantize = synth.quantize_rows_fp8 if kind == "fp8" else synth.quantize_rows_int8
            codes, scales = quantize(t)
            if l == 0 and t is w[0]:      # the device's conversion agrees with the host's
                c2, s2 = quantize(t.cpu())
                assert torch.equal(codes.cpu(), c2) and torch.equal(scales.cpu(), s2)
            layer_arrays.append(binding.pack_fp8_rows(codes, scales))
        packed.append(layer_arrays)
        del w
    code = binding.FP8_E4M3 if kind == "fp8" else binding.INT8
    layers = [binding.make_layer_fp8(p[0], p[1], p[2], sh.d_model, sh.d_ff, sh.r, sh.k, code_dtype=code) for p in packed]
    q = synth.tokens(sh, 1, 2001, torch.bfloat16, dev)
    ws = binding.make_workspace(sh.d_model, sh.d_ff, 1, dev)
    y = torch.empty(L, 1, sh.d_model, device=dev)
    cnt = torch.zeros(L, 1, dtype=torch.int32, device=dev)
    binding.spark_ffn_decode_layers(layers, q, y, ws, active_count=cnt)
    torch.cuda.synchronize()
    m = cnt.cpu().numpy().astype(np.float64)[:, 0]

    def step():
        binding.spark_ffn_decode_layers(layers, q, y, ws)

    gpu_s, _ = time_region(step, 200, 20, torch)
    per = gpu_s / 200
    nbytes = float(np.sum(sh.d_ff * (sh.r + 4) + m * (2 * sh.d_model - sh.r + 8)))
    out = {"workload": f"gemma2-2b-shape, {L} layers, batch 1, {'E4M3' if kind == 'fp8' else 'signed 8-bit integer'} "
                       "weight codes with per-row fp32 scales",
           "us_per_layer": per / L * 1e6, "layers_per_s": L / per, "active_count_mean": float(m.mean()),
           "algorithmic_bytes_per_layer": nbytes / L, "achieved_gbs": nbytes / per / 1e9,
           "hbm_frac": nbytes / per / 1e9 / HBM_PEAK_GBS, "batches": []}
    # the same stack with 4, 16 and 64 tokens per call (the batched matrix-core kernels on widened codes);
    # algorithmic bytes: the predictor rows and, for the union U of the tokens' active sets, the K2n and Vn rows
    for B in (4, 16, 64):
        qb = synth.tokens(sh, B, 2001 + B, torch.bfloat16, dev)
        wsb = binding.make_workspace(sh.d_model, sh.d_ff, B, dev)
        yb = torch.empty(L, B, sh.d_model, device=dev)
        ucnt = torch.zeros(L, dtype=torch.int32, device=dev)
        binding.spark_ffn_decode_layers(layers, qb, yb, wsb, union_count=ucnt)
        torch.cuda.synchronize()
        u = ucnt.cpu().numpy().astype(np.float64)
        gpu_b, _ = time_region(lambda: binding.spark_ffn_decode_layers(layers, qb, yb, wsb), 50, 5, torch)
        perb = gpu_b / 50
        nb = float(np.sum(sh.d_ff * (sh.r + 4) + u * (2 * sh.d_model - sh.r + 8)))
        out["batches"].append({"batch": B, "us_per_layer": perb / L * 1e6, "tokens_per_s": B / perb,
                               "union_size_mean": float(u.mean()), "algorithmic_bytes_per_layer": nb / L,
                               "achieved_gbs": nb / perb / 1e9, "hbm_frac": nb / perb / 1e9 / HBM_PEAK_GBS})
    return out


def master_weight_error(torch, binding, synth, dev, shape, q, y0, cnt0, idx0):
    """Reported, not gated: layer 0 of the stack as the kernels evaluate it (bf16-rounded weights) against
    the oracle on the unrounded fp32 master weights of the same seed (what rounding the weights costs)."""
    import numpy as np

    import oracle

    master = synth.ffn_layer(shape, 1000, torch.float32, dev)      # the stack's layer 0 before rounding
    o = oracle.spark_ffn(*(synth.to_oracle(t) for t in master), synth.to_oracle(q)[0], shape.k, skip_inactive=True)
    yg = y0.cpu().numpy().astype(np.float64)
    gset = set(int(i) for i in idx0[:int(cnt0)].cpu().numpy())
    oset = set(int(i) for i in o.idx)
    return {"rel_l2_y_vs_oracle_on_fp32_master_weights": float(np.linalg.norm(yg - o.y) / np.linalg.norm(o.y)),
            "active_set_symmetric_difference": len(gset ^ oset), "active_count_oracle_master": int(o.count),
            "layer": 0}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--layers", type=int, default=26)
    ap.add_argument("--shape", default="gemma2-2b")
    ap.add_argument("--batch", type=int, default=1)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dense", action="store_true")
    ap.add_argument("--no-stat-topk", action="store_true")
    ap.add_argument("--no-attention", action="store_true")
    ap.add_argument("--no-extra", action="store_true",
                    help="skip the single-layer-call timing and the batched / 9B-shaped / paper-shaped configurations")
    ap.add_argument("--no-traffic", action="store_true",
                    help="do not start the two rocprofv3 --pmc child runs that measure HBM traffic")
    ap.add_argument("--traffic-timeout", type=int, default=240, help="seconds allowed per counter run")
    ap.add_argument("--traffic-probe", action="store_true", help=argparse.SUPPRESS)
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1")
    if args.traffic_probe:
        return traffic_probe(args)

    # HBM traffic first: the counter runs are child processes, started before this process
    # initialises the GPU
    if args.no_traffic:
        traffic, traffic_note = None, "not measured (--no-traffic)"
    elif args.batch != 1:
        traffic, traffic_note = None, "measured for the batch-1 workload only"
    else:
        traffic, traffic_note = measure_traffic(args)

    import numpy as np
    import torch

    import synth
    from paper_2506_06644_amd import binding

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    shape = synth.SHAPES[args.shape]
    L, B = args.layers, args.batch

    weights = synth.ffn_stack(shape, L, base_seed=1000, dtype=torch.bfloat16, device=dev)
    q = synth.tokens(shape, B, 2000 + B, dtype=torch.bfloat16, device=dev)
    layers = [binding.make_layer(w[0], w[1], w[2], shape.k) for w in weights]
    ws = binding.make_workspace(shape.d_model, shape.d_ff, B, dev)
    y = torch.empty(L, B, shape.d_model, device=dev)
    cnt = torch.zeros(L, B, dtype=torch.int32, device=dev)
    ucnt = torch.zeros(L, dtype=torch.int32, device=dev)
    idx0 = torch.full((1, B, shape.d_ff), -1, dtype=torch.int32, device=dev)

    def step():
        # the product call of a decoder: y only (the index lists and counts are optional outputs)
        binding.spark_ffn_decode_layers(layers, q, y, ws)

    # untimed calls that also return the active counts (for the byte accounting) and layer 0's set
    binding.spark_ffn_decode_layers(layers, q, y, ws, active_count=cnt, union_count=ucnt)
    binding.spark_ffn_decode_layers(layers[:1], q, y[:1], ws, active_idx=idx0)
    step()
    torch.cuda.synchronize()
    counts = cnt.cpu().numpy()
    union = ucnt.cpu().numpy()
    assert np.isfinite(y.cpu().numpy()).all()

    gpu_s, wall_s = time_region(step, args.steps, args.warmup, torch)
    ms_per_step = gpu_s * 1e3 / args.steps
    layers_per_s = L * args.steps / gpu_s

    fetch_rows = union if B > 1 else counts[:, 0]
    per_layer = algorithmic_bytes(shape, [int(m) for m in fetch_rows], 2)
    bytes_step = float(sum(per_layer))
    call_avg_s, call_med_s = sampled_launch_time(step, 50, torch)
    if B == 1:
        # Each kernel of the call launched alone (the other launches switched off for that call; their
        # outputs of the full call above are still in the workspace).  `launch_us` is the average over
        # single launches, each between its own pair of events on the launch stream; the average of
        # 200 back-to-back launches between one pair of events is given beside it (consecutive
        # launches overlap their ramp and tail, so it is a little shorter).
        k1_bytes = 2.0 * shape.d_ff * shape.r * L
        kernels = {}
        for name, mask, nbytes in (("predict_layers_kernel", 1, k1_bytes),
                                   ("gather_layers_kernel", 2, bytes_step - k1_bytes),
                                   ("gather+reduce", 6, None)):
            tune = binding.Tuning(phases=mask)

            def one():
                binding.spark_ffn_decode_layers_tuned(layers, q, y, ws, tune)

            for _ in range(5):
                one()
            avg_s, med_s = sampled_launch_time(one, 100, torch)
            b2b = sorted(back_to_back_time(one, 200, torch) for _ in range(3))[1]
            kernels[name] = {"launch_us": avg_s * 1e6, "launch_us_median": med_s * 1e6,
                             "launch_us_back_to_back": b2b * 1e6}
            if nbytes:
                kernels[name].update(bytes_per_launch=nbytes, achieved=nbytes / avg_s / 1e9,
                                     frac=nbytes / avg_s / 1e9 / HBM_PEAK_GBS)
        # the reduce kernel alone is shorter than the host's launch interval: back-to-back launches
        # of it would time the host, so it is timed behind the gather and the gather subtracted
        both = kernels.pop("gather+reduce")
        kernels["reduce_layers_kernel"] = {
            k: both[k] - kernels["gather_layers_kernel"][k] for k in ("launch_us", "launch_us_median", "launch_us_back_to_back")}
        kernels["reduce_layers_kernel"]["timed_as"] = "gather + reduce launches minus gather alone"
        step()
        torch.cuda.synchronize()
        dom = kernels["predict_layers_kernel"]
        roofline = {"bound": "hbm", "achieved": dom["achieved"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": dom["frac"], "traffic": traffic_of(traffic, "predict_layers_kernel"),
                    "traffic_note": traffic_note,
                    "kernel": "predict_layers_kernel (the predictor sweep over all K1n of the call: the dominant "
                              "kernel, %d layers per launch)" % L,
                    "bytes_per_launch": dom["bytes_per_launch"], "launch_us": dom["launch_us"],
                    "launch_us_median": dom["launch_us_median"],
                    "launch_us_back_to_back": dom["launch_us_back_to_back"],
                    "other_kernels": {k: dict(v, traffic=traffic_of(traffic, k)) for k, v in kernels.items()
                                      if k != "predict_layers_kernel"},
                    "whole_call": {"bytes": bytes_step, "call_us": call_avg_s * 1e6,
                                   "call_us_median": call_med_s * 1e6, "achieved": bytes_step / call_avg_s / 1e9,
                                   "frac": bytes_step / call_avg_s / 1e9 / HBM_PEAK_GBS,
                                   "traffic": (None if traffic is None else sum(
                                       traffic_of(traffic, k) or 0.0 for k in
                                       ("predict_layers_kernel", "gather_layers_kernel", "reduce_layers_kernel")))}}
    else:
        achieved = bytes_step / call_avg_s / 1e9
        roofline = {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": achieved / HBM_PEAK_GBS, "traffic": None, "traffic_note": traffic_note,
                    "kernel": "whole spark_ffn_decode_layers call (several kernels per layer)",
                    "bytes_per_launch": bytes_step, "launch_us": call_avg_s * 1e6,
                    "launch_us_median": call_med_s * 1e6}

    out = {
        "metric": "Spark-FFN decode layers/s + achieved HBM GB/s vs peak (Gemma-2-2B shape, b=1)",
        "value": layers_per_s, "unit": "layers/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 weights and token, fp32 accumulate", "data": "synthetic",
        "config": {"workload": f"{shape.name}-shape Spark-FFN decode, {L} layers resident in HBM run back to "
                               f"back, batch {B}, d_model={shape.d_model} d_ff={shape.d_ff} r={shape.r} "
                               f"k={shape.k}", "layers": L, "batch": B},
        "tokens_per_s": layers_per_s / L * B,
        "us_per_layer": gpu_s / args.steps / L * 1e6,
        "achieved_gbs_whole_step": bytes_step * args.steps / gpu_s / 1e9,
        "hbm_frac_whole_step": bytes_step * args.steps / gpu_s / 1e9 / HBM_PEAK_GBS,
        "active_count_mean": float(counts.mean()), "active_count_min": int(counts.min()),
        "active_count_max": int(counts.max()), "union_size_mean": float(union.mean()),
        "host_wall_s": wall_s,
        "roofline": roofline,
        "paper_context": "paper reports whole-model decode speed-ups only: up to 1.79x on a 16-core CPU VM "
                         "(gemma.cpp) and 1.40x on an NVIDIA T4 (llama.cpp), batch 1; no per-layer figure",
    }

    if not args.no_dense:
        yd = torch.empty(L, B, shape.d_model, device=dev)

        def dense_step():
            binding.spark_ffn_dense_decode_layers(layers, q, yd, ws)

        dsteps = max(10, args.steps // 10)
        d_s, _ = time_region(dense_step, dsteps, 3, torch)
        dense_bytes = 2.0 * shape.d_ff * 2 * shape.d_model
        out["dense"] = {"layers_per_s": L * dsteps / d_s, "us_per_layer": d_s / dsteps / L * 1e6,
                        "bytes_per_layer": dense_bytes,
                        "achieved_gbs": dense_bytes * L * dsteps / d_s / 1e9,
                        "hbm_frac": dense_bytes * L * dsteps / d_s / 1e9 / HBM_PEAK_GBS,
                        "speedup_sparse_over_dense": (layers_per_s) / (L * dsteps / d_s)}
        err = (yd - y).norm() / y.norm()
        out["dense"]["rel_l2_vs_sparse"] = float(err)
        del yd

    if B == 1 and not args.no_extra:
        # the same stack called one layer at a time (what a decoder whose layers feed each other
        # would do): every call is a predictor sweep, a gather and a reduction of one layer
        def chain_step():
            for l in range(L):
                binding.spark_ffn_decode(layers[l], q, y[l], ws)

        csteps = max(5, args.steps // 20)
        c_s, _ = time_region(chain_step, csteps, 2, torch)
        out["single_layer_calls"] = {"us_per_layer": c_s / csteps / L * 1e6,
                                     "hbm_frac": bytes_step / L / (c_s / csteps / L) / 1e9 / HBM_PEAK_GBS}
        step()
        torch.cuda.synchronize()

    if B == 1 and not args.no_cpu_baseline and args.shape in ("gemma2-2b", "gemma2-9b", "spark-paper-2b", "tiny"):
        out["master_weights"] = master_weight_error(torch, binding, synth, dev, shape, q, y[0, 0], cnt[0, 0], idx0[0, 0])

    if not args.no_extra:
        out["other_configs"] = other_configs(torch, binding, synth, dev, args.shape, L, weights, layers)

    if not args.no_stat_topk:
        out["stat_topk"] = stat_topk_bench(torch, binding, synth, dev, not args.no_cpu_baseline, traffic, np)

    if not args.no_extra:
        out["prefill"] = prefill_bench(torch, binding, synth, dev, np)
        out["fp8_weights"] = fp8_bench(torch, binding, synth, dev, np)
        out["int8_weights"] = fp8_bench(torch, binding, synth, dev, np, kind="int8")
    if not args.no_attention:
        out["attention"] = attention_bench(torch, binding, synth, dev, not args.no_cpu_baseline)

    if not args.no_cpu_baseline:
        wcpu = tuple(synth.to_oracle(t) for t in weights[0])
        out["cpu_baseline"] = cpu_baseline(shape, wcpu, synth.to_oracle(q)[0])
    else:
        out["cpu_baseline"] = None
    print(json.dumps(out))


if __name__ == "__main__":
    main()
