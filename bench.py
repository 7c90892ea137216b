#!/usr/bin/env python3
"""Benchmark of the Superposed Decoding timestep on one MI355X.

One "step" is one spd_step: superposition weights, superposed embedding, the batch-1
transformer forward over the KV cache, LM head, vocabulary top-k, k x k expansion, n-gram
probes, interpolation, prune and state update -- the whole hot path.  Inputs (weights, KV
cache, n-gram store) are resident in HBM before the timed region starts.

Prints ONE JSON line (see the keys below).  `value` is draft-tokens/s = k * steps / time.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X published HBM3E peak


def algorithmic_bytes(shape, ctx_positions: float) -> dict:
    """Bytes one timestep must move: every streamed weight once plus the cached keys and
    values of `ctx_positions` positions (not the embedding table: only k rows are read)."""
    es = 2 if shape.dtype == "bf16" else 4
    dh = shape.d_head
    qkv = (shape.n_heads + 2 * shape.n_kv_heads) * dh * shape.d_model * es
    o = shape.d_model * shape.n_heads * dh * es
    gateup = 2 * shape.d_ffn * shape.d_model * es
    down = shape.d_model * shape.d_ffn * es
    head = shape.vocab * shape.d_model * es
    kv_pos = 2 * shape.n_layers * shape.n_kv_heads * dh * es
    return {"gemv_qkv": qkv, "gemv_o": o, "gemv_gateup": gateup, "gemv_down": down, "gemv_head": head,
            "kv_per_position": kv_pos,
            "step": shape.n_layers * (qkv + o + gateup + down) + head + kv_pos * ctx_positions}


def recorded_traffic(workload: str, k: int, prefix: int):
    """HBM bytes per launch of the fused forward kernel as counted by rocprofv3 (FETCH_SIZE +
    WRITE_SIZE, scaled by a plain copy): taken from the committed counter summary of this
    workload, since counters cannot be read from inside the benchmark.  Returns (bytes, the
    file it came from), or (None, None) if there is no summary for this workload."""
    names = [f"spd_step_{workload}_prefix{prefix}_k{k}_hbm_counters.txt", f"spd_step_{workload}_k{k}_hbm_counters.txt"]
    defaults = {"7b": 64, "13b": 256, "70b": 512, "tiny": 16}
    if prefix != defaults.get(workload):
        names = names[:1]
    for name in names:
        try:
            for line in open(os.path.join(ROOT, "profiles", name)):
                if line.startswith("traffic_bytes_per_launch"):
                    return float(line.split("=")[1]), "profiles/" + name
        except OSError:
            pass
    return None, None


def cpu_baseline(shape, weights, tables, lambdas, prefix, k, alpha, tau, delta):
    """The CPU oracle, as it stands, timed on this host, in two legs.
    All cores: the whole model at full depth on the workload's real prefix -- the prefix pass
    (untimed), the first timestep, then 2 timed SPD timesteps (each a few seconds at the 7B
    shape).  Models too large for that (more than 40 GB of weights) are timed on 1- and 3-layer
    truncations and extrapolated per layer, and the sample says so.
    One thread: the same timestep on 1- and 3-layer truncations with every numerical library
    limited to one thread, extrapolated per layer (per-layer = (t3 - t1) / 2, rest = t1 -
    per-layer, step = rest + n_layers * per-layer)."""
    import synth
    from oracle import spd_oracle as O
    from threadpoolctl import threadpool_info, threadpool_limits

    def host(name):
        return synth.host_view(weights[name]) if not isinstance(weights[name], np.ndarray) else weights[name]

    otabs = O.NgramTables(tables)
    cfg = O.DecodeCfg(k, alpha, tau, delta, tuple(lambdas))
    full_prefix = list(map(int, prefix))

    def timed_steps(n_layers, pre, n_steps):
        names = [n for n, _, _ in synth.weight_names(shape.truncated(n_layers))]
        w = {n: host(n) for n in names}
        lm = O.OracleLM(w, n_layers, shape.n_heads, shape.n_kv_heads, shape.rms_eps, shape.rope_theta)
        lm.reset()
        logits = lm.forward(lm.embedding_rows(pre))
        state, _ = O.first_step(logits, pre, cfg, keep_logits=False)
        t0 = time.perf_counter()
        for _ in range(n_steps):
            gamma = O.superposition_weights(state.logscores)
            x = O.superposed_embedding(lm.embedding_rows([d[-1] for d in state.drafts]), gamma.astype(np.float32))
            logits = lm.forward(x[None, :])
            state, _ = O.expand_and_prune(state, logits, otabs, cfg, keep_logits=False)
        return (time.perf_counter() - t0) / n_steps

    def extrapolated(pre, n_steps):
        if shape.n_layers <= 3:
            t = timed_steps(shape.n_layers, pre, n_steps)
            return t, 0.0, t
        t1, t3 = timed_steps(1, pre, n_steps), timed_steps(3, pre, n_steps)
        per_layer = max((t3 - t1) / 2, 0.0)
        rest = max(t1 - per_layer, 0.0)
        return rest + shape.n_layers * per_layer, per_layer, rest

    cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    weight_gb = shape.streamed_params() * (2 if shape.dtype == "bf16" else 4) / 1e9
    if weight_gb <= 40.0:
        step_s = timed_steps(shape.n_layers, full_prefix, 2)
        sample = (f"2 timed oracle timesteps of the whole {shape.name} model ({shape.n_layers} layers) after its "
                  f"{len(full_prefix)}-token prefix pass and first timestep, same tensors and n-gram tables as the GPU run, "
                  f"all {cores} threads")
    else:
        step_s, per_layer, rest = extrapolated(full_prefix[:8], 2)
        sample = (f"{weight_gb:.0f} GB of weights: 2 timed oracle timesteps each on 1- and 3-layer truncations of the "
                  f"{shape.name} model (8-token prefix), all {cores} threads; per-layer {per_layer * 1e3:.1f} ms, rest "
                  f"{rest * 1e3:.1f} ms, extrapolated to {shape.n_layers} layers")
    with threadpool_limits(limits=1):
        single_s, per_layer1, rest1 = extrapolated(full_prefix[:8], 1)
    return {"value": k / step_s, "unit": "draft-tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": sample, "ms_per_step": step_s * 1e3,
            "single_thread_ms_per_step": single_s * 1e3,
            "single_thread_value": k / single_s,
            "single_thread_sample": f"1 timed oracle timestep each on 1- and 3-layer truncations (8-token prefix), one thread; "
                                    f"per-layer {per_layer1 * 1e3:.0f} ms, rest {rest1 * 1e3:.0f} ms, extrapolated to "
                                    f"{shape.n_layers} layers"}


def probe_sweep(pkg, shape, weights, tables, lambdas, prefix, tau, delta, args):
    """Cost of the n-gram stage against the number of orders interpolated (the storage-saving
    variant keeps n = 2..4 only) and against k: average duration of the expand_prune kernel
    (k^2 options x orders probes of the hash tables, interpolation, prune) and of the whole step."""
    import torch
    n_steps = min(args.steps, 24)
    sess = pkg.Session(shape, weights, max_ctx=len(prefix) + args.warmup + n_steps + 4, k_max=16, kv_dtype=args.kv_dtype)
    rows = []
    for orders in (None, (2, 3), (2, 3, 4), (2, 3, 4, 5, 6)):
        alpha = 0.0
        if orders is not None:
            sub = {n: tables[n] for n in orders}
            sess.spd_load_ngrams(sub, lambdas)
            alpha = 0.55 if orders == (2, 3, 4) else 0.54
        for k in (1, 3, 5, 10):
            dc = pkg.SpdDecodeCfg(k, alpha, tau, delta)
            sess.spd_prefill(prefix)
            for _ in range(1 + args.warmup):
                sess.spd_step(dc, fetch=False)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(n_steps):
                sess.spd_step(dc, fetch=False)
            torch.cuda.synchronize()
            step_ms = (time.perf_counter() - t0) * 1e3 / n_steps
            sess.spd_prefill(prefix)
            for _ in range(1 + args.warmup):
                sess.spd_step(dc, fetch=False)
            sess.spd_set_kernel_timing(True)
            for _ in range(n_steps):
                sess.spd_step(dc, fetch=False)
            timing = sess.spd_get_kernel_timing()
            sess.spd_set_kernel_timing(False)
            ms, n = timing["expand_prune"]
            rows.append({"orders": list(orders) if orders else [], "entries": sum(len(tables[n][1]) for n in (orders or ())),
                         "alpha": alpha, "k": k, "expand_prune_us": ms * 1e3 / n, "ms_per_step": step_ms})
    sess.close()
    print(json.dumps({"probe_sweep": rows, "workload": shape.name, "prefix": len(prefix), "steps": n_steps}))


def phase_clocks(pkg, shape, weights, prefix, k, args):
    """Where the fused forward kernel spends a layer: every block stamps a clock when it has
    finished a phase (its outputs are stored: "arrival" at the synchronisation point behind the
    phase) and when it has the input of the next one ("release").  Per synchronisation point,
    averaged over the layers and over `steps` timesteps, in microseconds: how long the phase
    before it took for the last block, how far apart the blocks finish, how long after the last
    arrival the first / median / last block is released, and the period from one last arrival to
    the next (these add up to the layer time).  Prints a table, not JSON."""
    import torch
    n_steps = min(args.steps, 16)
    sess = pkg.Session(shape, weights, max_ctx=len(prefix) + args.warmup + n_steps + 8, k_max=max(k, 8), kv_dtype=args.kv_dtype)
    dc = pkg.SpdDecodeCfg(k, 0.0, 1.0, 0.1)
    sess.spd_prefill(prefix)
    for _ in range(1 + args.warmup):
        sess.spd_step(dc, fetch=False)
    sess.spd_set_kernel_timing(True)
    L = shape.n_layers
    names = ["qkv -> attention", "attention -> o_proj", "o_proj -> gate/up", "gate/up -> down", "down -> next qkv"]
    agg = {}
    for _ in range(n_steps):
        sess.spd_step(dc, fetch=False)
        st = sess.spd_get_phase_clock().astype(np.float64) / 100.0   # [blocks, stamps], microseconds
        arr, rel = st[:, 0::2], st[:, 1::2]
        nb = rel.shape[1]
        last_arr = arr[:, :nb].max(0)
        d = {"spread": last_arr - arr[:, :nb].min(0), "med_to_last": last_arr - np.median(arr[:, :nb], 0),
             "rel_first": rel.min(0) - last_arr, "rel_med": np.median(rel, 0) - last_arr, "rel_last": rel.max(0) - last_arr,
             "phase": np.concatenate([[0], last_arr[1:] - rel.max(0)[:-1]]),
             "period": np.concatenate([[0], last_arr[1:] - last_arr[:-1]]),
             "span": np.array([arr.max() - arr[:, 0].min()])}
        for key, v in d.items():
            agg[key] = agg.get(key, 0) + v / n_steps
    t = sess.spd_get_kernel_timing()
    sess.close()
    ctx0 = len(prefix) + 2 + args.warmup
    print(f"# {shape.name}, k = {k}, context {ctx0}..{ctx0 + n_steps - 1}, {n_steps} timesteps; microseconds, averaged over the {L} layers")
    print(f"# kernel span by the blocks' clocks: {agg['span'][0]:.1f}; fused_forward by HIP events: "
          f"{t['fused_forward'][0] * 1e3 / t['fused_forward'][1]:.1f} per launch")
    print(f"{'synchronisation point':<22} {'phase before it':>16} {'arrival spread':>15} {'median->last':>13} "
          f"{'release first':>14} {'median':>8} {'last':>8} {'period':>8}")
    tot = 0.0
    for j, nm in enumerate(names):
        idx = 1 + 5 * np.arange(L) + j
        row = [agg[key][idx].mean() for key in ("phase", "spread", "med_to_last", "rel_first", "rel_med", "rel_last", "period")]
        tot += row[-1]
        print(f"{nm:<22} {row[0]:16.2f} {row[1]:15.2f} {row[2]:13.2f} {row[3]:14.2f} {row[4]:8.2f} {row[5]:8.2f} {row[6]:8.2f}")
    ab = algorithmic_bytes(shape, 0)
    layer_bytes = ab["gemv_qkv"] + ab["gemv_o"] + ab["gemv_gateup"] + ab["gemv_down"]
    print(f"# per layer: {tot:.2f}; streaming a layer's {layer_bytes / 1e6:.1f} MB of weights at the 8 TB/s peak: "
          f"{layer_bytes / 8e12 * 1e6:.2f}")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=64)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--workload", default="7b", choices=["7b", "tiny", "13b", "70b"])
    ap.add_argument("--prefix", type=int, default=None)
    ap.add_argument("--k", type=int, default=3)
    ap.add_argument("--kv-dtype", default=None, choices=["fp16", "fp32"],
                    help="element type of the key/value cache (default: fp16 for the bf16 workloads, whose algorithmic "
                         "bytes count a cached element at 2 bytes; fp32 for the fp32 one)")
    ap.add_argument("--ngram-entries", type=int, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-timing", action="store_true")
    ap.add_argument("--no-graph", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device-to-device copy (a known traffic for scaling HBM counters)")
    ap.add_argument("--probe-sweep", action="store_true",
                    help="instead of the benchmark: time the n-gram stage (expand_prune kernel) against the "
                         "orders loaded (none, 2..3, 2..4, 2..6) and k = 1, 3, 5, 10; prints one JSON line")
    ap.add_argument("--phase-clocks", action="store_true",
                    help="instead of the benchmark: per-phase clock stamps of the fused forward kernel (a table)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (the SPD step is a single-GPU, batch-1 path); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)
    if args.kv_dtype is None:
        args.kv_dtype = "fp32" if args.workload == "tiny" else "fp16"

    import torch

    import paper_2405_18400_amd as pkg
    import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    shape = {"7b": synth.LLAMA7B, "tiny": synth.TINY, "13b": synth.LLAMA13B, "70b": synth.LLAMA70B}[args.workload]
    m = args.prefix or {"7b": 64, "tiny": 16, "13b": 256, "70b": 512}[args.workload]
    entries = args.ngram_entries or {"7b": 10_000_000, "tiny": 100_000, "13b": 50_000_000, "70b": 10_000_000}[args.workload]
    k, alpha, tau, delta = args.k, 0.54, 1.0, 0.1
    lambdas = synth.PAPER_LAMBDAS
    K, W = args.steps, args.warmup
    max_ctx = m + max(W + K, 32) + 2

    t_setup = time.time()
    if shape.dtype == "bf16":
        weights = synth.make_weights_device(shape, seed=0)
    else:
        weights = synth.make_weights(shape, seed=0)
    prefix = synth.make_prefix_uniform(shape.vocab, m, seed=0) if args.workload == "tiny" else synth.make_prefix_zipf(shape.vocab, m, seed=0)
    if args.phase_clocks:
        return phase_clocks(pkg, shape, weights, prefix, k, args)
    if args.workload == "tiny":
        tables = synth.make_ngram_tables_uniform(shape.vocab, {2: entries // 2, 3: entries // 2}, seed=0)
    else:
        tables = synth.make_ngram_tables_zipf(shape.vocab, entries, seed=0)
    if args.probe_sweep:
        return probe_sweep(pkg, shape, weights, tables, lambdas, prefix, tau, delta, args)
    sess = pkg.Session(shape, weights, max_ctx=max_ctx, k_max=max(k, 8), kv_dtype=args.kv_dtype)
    sess.spd_load_ngrams(tables, lambdas)
    if args.no_graph:
        sess.spd_set_graph(False)
    dc = pkg.SpdDecodeCfg(k, alpha, tau, delta)
    t_setup = time.time() - t_setup

    def run(n_steps):
        for _ in range(n_steps):
            sess.spd_step(dc, fetch=False)

    # prefill + first timestep + warm-up (captures the step graph), untimed
    sess.spd_prefill(prefix)
    sess.spd_step(dc, fetch=False)
    run(W)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    with torch.cuda.stream(sess.stream):
        ev0.record(sess.stream)
        run(K)
        ev1.record(sess.stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    gpu_ms = ev0.elapsed_time(ev1)
    ms_per_step = wall * 1e3 / K
    tok, par, sc = sess.spd_step(dc)          # one fetched step: the run produced finite drafts
    assert np.all(np.isfinite(sc)) and len(set(zip(par.tolist(), tok.tolist()))) == k

    ctx_mean = m + W + 1 + (K - 1) / 2.0  # cached positions read by the average timed step
    ab = algorithmic_bytes(shape, ctx_mean)
    step_gbs = ab["step"] / (ms_per_step * 1e-3) / 1e9

    # per-kernel durations with HIP events on the library's stream (plain launches, same steps)
    roofline = {"bound": "hbm", "kernel": "spd_step (all kernels)", "achieved": step_gbs, "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": step_gbs / HBM_PEAK_GBS, "traffic": None}
    kernels = {}
    if not args.no_kernel_timing:
        sess.spd_prefill(prefix)
        sess.spd_step(dc, fetch=False)
        run(W)
        sess.spd_set_kernel_timing(True)
        run(min(K, 32))
        timing = sess.spd_get_kernel_timing()
        sess.spd_set_kernel_timing(False)
        for name, (ms, n) in timing.items():
            if n:
                kernels[name] = {"avg_us": ms * 1e3 / n, "launches_per_step": n / min(K, 32)}
                if name in ab:
                    kernels[name]["GBps"] = ab[name] / (ms * 1e-3 / n) / 1e9
        # dominant kernel: the fused forward (the whole model in one launch) where it runs,
        # else the largest matrix-vector product
        fwd_bytes = ab["step"]
        traffic, traffic_source = None, None
        if "fused_forward" in kernels:
            dom, dom_bytes = "fused_forward", fwd_bytes
            traffic, traffic_source = recorded_traffic(args.workload, k, m)
        else:
            dom, dom_bytes = "gemv_gateup", ab["gemv_gateup"]
        if dom in kernels:
            gbs = dom_bytes / (kernels[dom]["avg_us"] * 1e-6) / 1e9
            kernels[dom]["GBps"] = gbs
            roofline = {"bound": "hbm", "kernel": dom, "achieved": gbs, "peak": HBM_PEAK_GBS,
                        "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS, "traffic": traffic,
                        "traffic_source": (traffic_source + " (rocprofv3 counters of an earlier run of this command, not of this run)")
                        if traffic_source else None,
                        "bytes_per_launch": dom_bytes, "avg_launch_us": kernels[dom]["avg_us"],
                        "step_achieved": step_gbs, "step_frac": step_gbs / HBM_PEAK_GBS,
                        "step_bytes": ab["step"]}

    # k independent batch-1 passes on the same GPU (k = 1 SPD = greedy): k x the step time of k = 1
    dc1 = pkg.SpdDecodeCfg(1, 0.0, tau, delta)
    sess.spd_prefill(prefix)
    sess.spd_step(dc1, fetch=False)
    run1 = lambda n: [sess.spd_step(dc1, fetch=False) for _ in range(n)]
    run1(W)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    run1(K)
    torch.cuda.synchronize()
    greedy_ms = (time.perf_counter() - t1) * 1e3 / K

    # the paper's own comparison (Section 4.3): k independent passes of nucleus sampling, here
    # top-p 0.9 (BASELINE config 3), each step = the same forward + the sampler; seeded draws
    sc = pkg.SpdSampleCfg(0.9, tau)
    us = np.random.default_rng(0).random(max(W + K + 1, 8)).astype(np.float32)
    sess.spd_prefill(prefix)
    sess.spd_nucleus_step(sc, float(us[0]), fetch=False)
    for i in range(W):
        sess.spd_nucleus_step(sc, float(us[1 + i]), fetch=False)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for i in range(K):
        sess.spd_nucleus_step(sc, float(us[1 + W + i]), fetch=False)
    torch.cuda.synchronize()
    nucleus_ms = (time.perf_counter() - t1) * 1e3 / K
    ntok, nlp = sess.spd_nucleus_step(sc, 0.5)
    assert 0 <= ntok < shape.vocab and np.isfinite(nlp)

    # the prefix pass alone (the first-timestep forward over M), dense on the matrix cores where
    # the model allows it: tokens/s, and the two rooflines by ALGORITHMIC work -- model flops
    # (2 x parameters of the layers x tokens) against the dense bf16 MFMA peak, and one pass over
    # the weights against the HBM peak (short chunks are bound by the latter).  The kernels feed
    # every activation as a hi + lo bf16 pair, i.e. issue twice the model's products: that is
    # their own overhead and is not counted.
    sess.spd_prefill(prefix)
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    sess.spd_prefill(prefix)
    torch.cuda.synchronize()
    prefill_ms = (time.perf_counter() - t2) * 1e3
    layer_params = shape.streamed_params() - shape.vocab * shape.d_model
    es = 2 if shape.dtype == "bf16" else 4
    prefill = {"tokens": m, "ms": prefill_ms, "tokens_per_s": m / prefill_ms * 1e3,
               "dense": bool(sess.spd_get_dense_prefill()),
               "model_tflops": 2.0 * layer_params * m / (prefill_ms * 1e-3) / 1e12,
               "weight_pass_GBps": shape.streamed_params() * es / (prefill_ms * 1e-3) / 1e9}
    prefill["frac_of_bf16_mfma_peak"] = prefill["model_tflops"] / 2500.0
    prefill["frac_of_hbm_peak"] = prefill["weight_pass_GBps"] / HBM_PEAK_GBS

    # end-to-end generation as the paper times it: prefix pass + 10 tokens
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    drafts, scores = sess.spd_generate(prefix, dc, 10)
    e2e_ms = (time.perf_counter() - t2) * 1e3

    # resets (Section 5.3): one of the k drafts is committed every s = 8 timesteps and its 8
    # tokens are passed again as ordinary prefix tokens; splice (Section 4.5): a one-draft nucleus
    # opening is committed, which passes only its newest token again
    def timed(f):
        torch.cuda.synchronize()
        t = time.perf_counter()
        r = f()
        torch.cuda.synchronize()
        return (time.perf_counter() - t) * 1e3, r
    s_reset = 8
    sess.spd_prefill(prefix)
    for _ in range(s_reset):
        sess.spd_step(dc, fetch=False)
    sess.spd_commit(0.5)                                    # untimed: first use of this chunk size
    for _ in range(s_reset):
        sess.spd_step(dc, fetch=False)
    commit_ms, _ = timed(lambda: sess.spd_commit(0.5))
    seg_ms, _ = timed(lambda: [sess.spd_step(dc, fetch=False) for _ in range(s_reset)])
    sess.spd_prefill(prefix)
    for i in range(4):
        sess.spd_nucleus_step(sc, float(us[i]), fetch=False)
    splice_ms, (ci, ctoks) = timed(lambda: sess.spd_commit(0.5))
    assert ci == 0 and len(ctoks) == 4
    resets = {"s": s_reset, "commit_ms": commit_ms, "segment_ms": seg_ms,
              "overhead_frac": commit_ms / (commit_ms + seg_ms), "splice_commit_ms": splice_ms}

    out = {
        "metric": "draft-tokens/sec at k=3 (7B-shape bf16, batch 1); % of peak HBM GB/s",
        "value": k * K / wall, "unit": "draft-tokens/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": shape.dtype, "data": "synthetic",
        "config": {"workload": f"{shape.name}, random-init N(0,0.02), prefix {m} Zipf tokens, k={k}, "
                               f"alpha={alpha}, tau={tau}, delta={delta}, n-gram tables n=2..6 with "
                               f"{sum(len(v[1]) for v in tables.values())} entries; {K} consecutive timesteps "
                               f"(context {m + 1 + W}..{m + W + K})",
                   "k": k, "prefix": m, "graph": not args.no_graph, "fused_forward": sess.spd_get_fused(),
                   "kv_cache": args.kv_dtype},
        "pct_peak_hbm": 100.0 * step_gbs / HBM_PEAK_GBS,
        "gpu_ms_per_step_events": gpu_ms / K,
        "roofline": roofline,
        "kernels": kernels,
        "k_independent_passes": {"ms_per_pass_step": nucleus_ms, "ms_for_k_drafts": k * nucleus_ms,
                                 "speedup_of_spd": k * nucleus_ms / ms_per_step,
                                 "kind": "k nucleus-sampling passes (top-p 0.9), one token per pass per step",
                                 "greedy_ms_per_pass_step": greedy_ms,
                                 "speedup_of_spd_over_k_greedy": k * greedy_ms / ms_per_step},
        "prefill": prefill,
        "resets": resets,
        "generate_10_tokens_ms": e2e_ms,
        "setup_s": t_setup,
    }
    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        out["copy_calibration_bytes"] = 1 << 30
        del src, dst
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(shape, weights, tables, lambdas, prefix, k, alpha, tau, delta)
    sess.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
