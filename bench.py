#!/usr/bin/env python3
"""Benchmark of the fused MoE-layer forward (moe_layer_forward through the C-ABI) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config C4] [--no-cpu-baseline]

A step is one pass of the whole hot path (route -> dispatch -> grouped gate/up + SwiGLU -> grouped down ->
combine) over one synthetic batch that is already resident in HBM. Prints ONE JSON line:
  value           tokens/s of the whole layer (T / mean step time over exactly K steps, wall clock between two
                  device synchronisations)
  roofline        the dominant kernel (grouped gate/up + SwiGLU): algorithmic flops (prefill configs) or bytes
                  (decode config) per launch divided by its mean duration, measured with HIP events recorded on
                  the launch stream around that stage in a second pass of K steps
  roofline_down   the same for the grouped down projection
  roofline_layer  the whole layer against the roofline the task's target names for this workload
  cpu_baseline    the CPU oracle timed once on the same inputs on this machine's host cores
  stages_us       mean HIP-event time of every stage (second pass)
  step_event_us   median and minimum over the K steps of the second pass of a step's summed stage event times
  also            the other four layer workloads (C1, C2, C3 and the decode config C5, the HBM-bound half of the
                  headline metric) measured the same way, when the main workload is C4; the affinity-aware token
                  compressor (the producer of the retained-token index list) on its 8064-token workload; the
                  predictor features; the expert cache
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0          # MI355X HBM3E
PREWARM_S = 0.1                # untimed spin-up before the warm-up steps (clock ramp of an idle GPU)


def load_traffic(workload, kernel):
    """Measured HBM bytes per launch from the committed rocprofv3 --pmc summaries, if any, and the commit of the
    tree they were taken on (a figure from an older tree than the one running is visible as such)."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    try:
        with open(path) as f:
            j = json.load(f)
        return j.get(workload, {}).get(kernel), j.get("_meta", {}).get("commit")
    except (OSError, ValueError):
        return None, None


def kernel_roofline(workload, kernel, hbm_bound, flops, nbytes, seconds):
    """Roofline entry of one kernel: algorithmic flops or bytes per launch over its mean event time."""
    if hbm_bound:
        roof = {"bound": "hbm", "achieved": nbytes / seconds / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s"}
    else:
        roof = {"bound": "mfma", "achieved": flops / seconds / 1e12, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s"}
    roof["frac"] = roof["achieved"] / roof["peak"]
    roof["kernel"] = kernel
    roof["kernel_us"] = seconds * 1e6
    tr, commit = load_traffic(workload, kernel)
    # HBM bytes per launch of that kernel (rocprofv3 FETCH_SIZE + WRITE_SIZE, scaled by a 1 GiB copy's readings)
    roof["traffic"] = (tr["fetch_bytes"] + tr["write_bytes"]) if tr else None
    if tr:
        roof["traffic_detail"] = tr
        roof["traffic_commit"] = commit
    roof["algorithmic_bytes"] = nbytes
    roof["algorithmic_flops"] = flops
    return roof


def measure(name, steps, warmup, with_cpu_baseline, weight_sets=None):
    import numpy as np
    import torch
    from paper_2605_05899_amd import harness, moe, synth

    inp = synth.make_config(name)
    d = harness.DeviceLayer(inp, torch, moe)
    args = d.layer_args()
    # The weight-streaming configs (C3, C5) rotate over distinct device copies of the layer's weights, one copy per
    # step in turn, so that no step can find the weights of the step before it in the 256 MB last-level cache.
    if weight_sets is None:
        weight_sets = 2 if name in ("C3", "C5") else 1
    clone = lambda t: None if t is None else t.clone()
    arg_sets = [args] + [args[:5] + tuple(clone(t) for t in args[5:12]) + args[12:] for _ in range(weight_sets - 1)]
    step_no = [0]

    def step():
        moe.moe_layer_forward(*arg_sets[step_no[0] % weight_sets])
        step_no[0] += 1

    # Spin-up, not measurement: an idle MI355X needs about 25 ms of continuous work before its clocks settle (the
    # first 30 steps of this layer run up to 30 % slower), so the layer runs untimed for PREWARM_S seconds first;
    # the W warm-up steps and the K timed steps follow unchanged.
    t_spin, prewarm_steps = time.perf_counter(), 0
    while time.perf_counter() - t_spin < PREWARM_S:
        for _ in range(10):
            step()
        torch.cuda.synchronize()
        prewarm_steps += 10
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / steps

    # second pass: per-stage HIP events on the launch stream
    moe.moe_stage_timing_enable(True)
    per_step = np.zeros((steps, moe.N_STAGES))
    for i in range(steps):
        step()
        per_step[i] = moe.moe_stage_timing_read()
    moe.moe_stage_timing_enable(False)
    stage_ms = per_step.mean(axis=0)
    step_event_ms = per_step.sum(axis=1)          # one step as the sum of its stages' event times

    # routing statistics for the algorithmic byte count (which experts are touched)
    ids = torch.zeros((inp.T, inp.k), dtype=torch.int32, device="cuda")
    w = torch.zeros((inp.T, inp.k), dtype=torch.float32, device="cuda")
    moe.moe_layer_forward(*args[:13], ids, w, d.ws)
    torch.cuda.synchronize()
    touched = int(np.unique(ids.cpu().numpy()).size)

    T, H, I, E, k, S = inp.T, inp.H, inp.I, inp.E, inp.k, inp.S
    flops_layer = inp.useful_flops()
    rows = T * (k + S)
    gate_up_flops, down_flops = 4.0 * rows * H * I, 2.0 * rows * H * I
    # algorithmic bytes: the weights of every group that has a row, each operand row once, the result once
    gate_up_bytes = (touched + S) * 2.0 * I * H * 2 + T * H * 2 + rows * I * 2
    down_bytes = (touched + S) * 1.0 * I * H * 2 + rows * I * 2 + rows * H * 2
    layer_bytes = (touched + S) * 3.0 * I * H * 2 + E * H * 2 + 2.0 * T * H * 2
    hbm_bound = name == "C5"
    skinny = rows <= 40 * (E + S)
    kern = "ffn_skinny_kernel" if skinny else "ffn_tile_kernel"
    roof = kernel_roofline(name, kern + "<0>", hbm_bound, gate_up_flops, gate_up_bytes, stage_ms[2] * 1e-3)
    roof_down = kernel_roofline(name, kern + "<1>", hbm_bound, down_flops, down_bytes, stage_ms[3] * 1e-3)
    step_s = ms_per_step * 1e-3
    # the whole layer against the roofline its target is stated in: HBM for the decode config and for the pruned
    # prefill (its small groups re-read every expert's weights for a few rows), MFMA for the other prefill configs
    layer_hbm = name in ("C3", "C5")
    roof_layer = ({"bound": "hbm", "achieved": layer_bytes / step_s / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s"}
                  if layer_hbm else
                  {"bound": "mfma", "achieved": flops_layer / step_s / 1e12, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s"})
    roof_layer["frac"] = roof_layer["achieved"] / roof_layer["peak"]
    roof_layer["algorithmic_bytes"], roof_layer["algorithmic_flops"] = layer_bytes, flops_layer

    res = {
        "workload": name, "prewarm_steps": prewarm_steps, "weight_sets": weight_sets, "ms_per_step": ms_per_step, "tokens_per_s": T / (ms_per_step * 1e-3),
        "layer_tflops": flops_layer / (ms_per_step * 1e-3) / 1e12,
        "layer_frac_mfma_peak": flops_layer / (ms_per_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
        "layer_gbs": layer_bytes / (ms_per_step * 1e-3) / 1e9,
        "layer_frac_hbm_peak": layer_bytes / (ms_per_step * 1e-3) / 1e9 / PEAK_HBM_GBS,
        "experts_touched": touched, "roofline": roof, "roofline_down": roof_down, "roofline_layer": roof_layer,
        "stages_us": {n: float(v * 1e3) for n, v in zip(moe.STAGE_NAMES, stage_ms)},
        "step_event_us": {"median": float(np.median(step_event_ms) * 1e3), "min": float(step_event_ms.min() * 1e3)},
        "shape": {"T": T, "T_in": inp.T_in, "H": H, "E": E, "k": k, "I": I, "S": S},
    }
    if with_cpu_baseline:
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            cores = os.cpu_count() or 1
        # bounded sample: whole-layer oracle passes over the same inputs until about 10 s of CPU time are spent
        reps, t0 = 0, time.perf_counter()
        from oracle import moe_oracle
        while reps < 1 or (time.perf_counter() - t0 < 10.0 and reps < 20):
            moe_oracle.moe_layer_forward(inp.x, inp.keep_idx, inp.w_router, inp.w_gate, inp.w_up, inp.w_down, inp.k,
                                         inp.norm_topk, inp.ws_gate, inp.ws_up, inp.ws_down)
            reps += 1
        dt = (time.perf_counter() - t0) / reps
        res["cpu_baseline"] = {"value": T / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
                               "sample": f"{reps} passes of the whole {name} layer ({T} tokens each) through the numpy "
                                         f"fp32 oracle, {dt:.2f} s per pass"}
    return res


def measure_compress(name, steps, warmup, with_cpu_baseline):
    """The affinity-aware token compressor (moe_token_compress) on a synthetic workload: time per call, algorithmic
    bytes (attention rows + prefix routing ids in, index list out) against the HBM peak, and the oracle beside it.
    The kernels are latency-bound at these sizes (1.5 MB of input), which the roofline fraction shows."""
    import numpy as np
    import torch
    from paper_2605_05899_amd import moe, synth

    c = synth.make_compress_config(name)
    n_heads, N = c.A.shape
    L, _, k = c.R.shape
    dA, dR = torch.from_numpy(c.A).cuda(), torch.from_numpy(c.R).cuda()
    K_keep = int(np.floor(c.beta * N))
    keep = torch.empty(K_keep, dtype=torch.int32, device="cuda")
    ws = moe.alloc_compress_workspace(N, c.E)
    args = (dA, n_heads, N, dR, L, k, c.E, c.alpha, c.beta, c.lam, keep, None, None, ws)
    for _ in range(max(warmup, 50)):
        moe.moe_token_compress(*args)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        moe.moe_token_compress(*args)
    torch.cuda.synchronize()
    us = (time.perf_counter() - t0) * 1e6 / steps
    nbytes = c.A.nbytes + c.R.nbytes + K_keep * 4
    res = {"workload": name, "shape": {"N": N, "n_heads": n_heads, "L": L, "k": k, "E": c.E, "alpha": c.alpha,
                                      "beta": c.beta, "lambda": c.lam, "kept": K_keep},
           "us_per_call": us, "visual_tokens_per_s": N / (us * 1e-6),
           "roofline": {"bound": "hbm", "achieved": nbytes / (us * 1e-6) / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                        "frac": nbytes / (us * 1e-6) / 1e9 / PEAK_HBM_GBS, "traffic": None,
                        "kernel": ("compress_prepare_kernel + compress_select_kernel"
                                   if N < moe.moe_compress_wide_min_tokens(-1)
                                   else "compress_prepare_kernel + the wide_* chain (11 launches)"),
                        "algorithmic_bytes": nbytes}}
    if with_cpu_baseline:
        from oracle import compress_oracle as CO
        reps, t0 = 0, time.perf_counter()
        while reps < 1 or (time.perf_counter() - t0 < 3.0 and reps < 50):
            CO.token_compress(c.A, c.R, c.E, c.alpha, c.beta, c.lam)
            reps += 1
        dt = (time.perf_counter() - t0) / reps
        res["cpu_baseline"] = {"value": N / dt, "unit": "visual tokens/s", "cores": 1, "kind": "oracle",
                               "sample": f"{reps} passes of the {name} workload ({N} tokens) through the Python/numpy "
                                         f"oracle, {dt * 1e3:.0f} ms per pass"}
    return res


def measure_predictor_features(steps, warmup):
    """Feature construction of the lookahead predictor (Eq. 6-7) and its target (Eq. 9) at the size of the C3/C4
    stream after compression: hidden states [8192, 2048] pooled over 2016 retained rows, a routing histogram over
    4 layers x 2016 tokens x 8 ids, the target over a window of 5 layers. Mean pooling is the HBM-bound part."""
    import numpy as np
    import torch
    from paper_2605_05899_amd import moe, synth

    H, E, K, k = 2048, 128, 2016, 8
    rng = np.random.default_rng(5)
    hid = torch.from_numpy(synth.f32_to_bf16(rng.standard_normal((8192, H)).astype(np.float32)).view(np.int16)).cuda()
    keep = torch.from_numpy(np.sort(rng.choice(8064, size=K, replace=False)).astype(np.int32)).cuda()
    ids = torch.from_numpy(rng.integers(0, E, size=(5, K, k)).astype(np.int32)).cuda()
    x = torch.zeros(E + H, dtype=torch.float32, device="cuda")
    g = torch.zeros(E, dtype=torch.float32, device="cuda")
    ws = torch.empty(moe.moe_mean_pool_workspace_bytes(H), dtype=torch.uint8, device="cuda")
    # the predictor network at a plausible size: input [h_r ; h_h ; h_v] = 128 + 2048 + 1152, bottleneck 1024 -> 256
    D, D1, D2, B = E + H + 1152, 1024, 256, 20
    rnd = lambda *shape: torch.from_numpy((rng.standard_normal(shape) / np.sqrt(shape[-1])).astype(np.float32)).cuda()
    xin, W1, W2, Wo = rnd(D), rnd(D1, D), rnd(D2, D1), rnd(E, D2)
    s1, t1, s2, t2 = rnd(D1) + 1, rnd(D1), rnd(D2) + 1, rnd(D2)
    yv = torch.zeros(E, dtype=torch.float32, device="cuda")
    top = torch.zeros(B, dtype=torch.int32, device="cuda")
    wsp = torch.empty(moe.moe_predictor_workspace_bytes(D1, D2), dtype=torch.uint8, device="cuda")
    calls = {
        "predictor_mlp_top20": lambda: moe.moe_predictor_forward(xin, D, W1, s1, t1, D1, W2, s2, t2, D2, Wo, E, B, yv, top,
                                                                 wsp),
        "mean_pool": lambda: moe.moe_mean_pool(hid, 8192, H, keep, K, x[E:], ws),
        "routing_histogram": lambda: moe.moe_routing_histogram(ids, 4 * K * k, E, x[:E]),
        "lookahead_target": lambda: moe.moe_lookahead_target(ids, 5, K * k, E, 0.8, g),
    }
    res = {}
    for name, fn in calls.items():
        for _ in range(max(warmup, 50)):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        res[name + "_us"] = (time.perf_counter() - t0) * 1e6 / steps
    nbytes = K * H * 2 + K * 4 + H * 4
    s = res["mean_pool_us"] * 1e-6
    res["roofline"] = {"bound": "hbm", "achieved": nbytes / s / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                       "frac": nbytes / s / 1e9 / PEAK_HBM_GBS, "traffic": None,
                       "kernel": "mean_pool_partial_kernel + mean_pool_finish_kernel", "algorithmic_bytes": nbytes}
    res["shape"] = {"rows": 8192, "H": H, "K": K, "E": E, "history_layers": 4, "window": 5, "k": k,
                    "mlp": [D, D1, D2, E], "top_B": B}
    return res


def measure_expert_cache():
    """The slab cache's transfer path at the size of the C4 model's experts (9.4 MB slabs): host-to-device rate of a
    burst of prefetches on the transfer stream, host time per cache call, and the same burst while the compute stream
    runs the C4 layer (both streams busy, as in the paper's pipeline)."""
    import numpy as np
    import torch
    from paper_2605_05899_amd import harness, moe, synth

    H, I, E, n_fetch = 2048, 768, 64, 48
    slab_bytes = 3 * I * H * 2
    host = torch.empty((E, slab_bytes), dtype=torch.uint8).pin_memory()
    host.random_(0, 255)
    pool = torch.empty(n_fetch * slab_bytes, dtype=torch.uint8, device="cuda")
    trans, comp = torch.cuda.Stream(), torch.cuda.Stream()
    addr = lambda l, e: host.data_ptr() + e * slab_bytes

    def burst(background=None):
        cache = moe.ExpertCache(1, E, slab_bytes, n_fetch, pool)
        items = [(0, e, 1.0 - e / E) for e in range(n_fetch)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        started = cache.predict(items, addr, trans)
        t_call = time.perf_counter() - t0
        if background:
            with torch.cuda.stream(comp):
                for _ in range(8):
                    background()
        trans.synchronize()
        dt = time.perf_counter() - t0
        t1 = time.perf_counter()
        cache.acquire(0, list(range(0, n_fetch, 6)), addr, trans, comp)
        t_acq = time.perf_counter() - t1
        torch.cuda.synchronize()
        cache.close()
        return len(started) * slab_bytes / dt / 1e9, t_call / n_fetch * 1e6, t_acq * 1e6

    burst()
    alone = [burst() for _ in range(3)]
    inp = synth.make_config("C4")
    d = harness.DeviceLayer(inp, torch, moe)
    args = d.layer_args()
    layer = lambda: moe.moe_layer_forward(*args, stream=comp)
    busy = [burst(layer) for _ in range(3)]
    return {"slab_MB": slab_bytes / 1e6, "experts_per_burst": n_fetch,
            "h2d_GBps": max(a[0] for a in alone), "h2d_GBps_while_layer_runs": max(b[0] for b in busy),
            "predict_host_us_per_expert": min(a[1] for a in alone), "acquire_host_us_8_hits": min(a[2] for a in alone)}


def measure_prefetch_pipeline():
    """Compute-stream stall per layer of a four-layer stack in decode steps (4 tokens, 64 experts, top-4, slabs of
    9.4 MB like the C4 model's experts) whose experts live in pinned host memory behind a cache of 160 slabs (of 256
    experts), for three sources of the lookahead list (paper Sec. 3.4.2): none (every absent expert fetched on demand),
    the library's predictor MLP with random weights (a list no better than chance), and a stand-in that names the
    next layer's true experts with recall 0.9. Every step routes a fresh token batch, so the set of experts a layer
    needs drifts from step to step; four steps fill the cache, sixteen are measured."""
    import numpy as np
    import torch
    from paper_2605_05899_amd import harness, moe, pipeline, synth

    n_layers, T, H, E, k, I, n_slabs, budget, n_warm, n_steps = 4, 4, 2048, 64, 4, 768, 160, 14, 4, 16
    layers = [synth.make_small(900 + l, T, H, E, k, I, 0) for l in range(n_layers)]
    rng_x = np.random.default_rng(13)
    batches = [[harness.bf16_dev(synth.f32_to_bf16(rng_x.standard_normal((T, H)).astype(np.float32)), torch)
                for _ in range(n_layers)] for _ in range(n_warm + n_steps)]
    out = {"shape": {"layers": n_layers, "T": T, "H": H, "E": E, "k": k, "I": I, "slab_MB": 3 * I * H * 2 / 1e6,
                     "n_slabs": n_slabs, "list_length": budget, "warm_steps": n_warm, "steps": n_steps}}
    for name, mode, recall in (("demand_only", "demand", 0.0), ("mlp_random_weights", "mlp", 0.0),
                               ("standin_recall_0.9", "standin", 0.9)):
        stack = pipeline.CachedLayerStack(torch, moe, layers, n_slabs=n_slabs, budget=budget)
        try:
            if mode == "mlp":
                stack.set_random_mlp(11)
            rng = np.random.default_rng(12)
            stats, per_layer = pipeline.StackStats(), []
            for i, xs in enumerate(batches):
                stack.x = xs
                truth = stack.true_experts()
                if i == n_warm:
                    stats, before = pipeline.StackStats(), stack.cache.stats()
                if i >= n_warm:
                    per_layer += [len(t) for t in truth]
                stack.run_pass(mode, stats, truth=truth, recall=recall, rng=rng)
            after = stack.cache.stats()
            s = stats.summary({kk: after[kk] - before[kk] for kk in after})
            out[name] = {kk: s[kk] for kk in ("stall_us_mean", "stall_us_max", "experts_demanded", "demand_misses",
                                              "experts_listed", "prefetch_copies_started", "cache_hits",
                                              "cache_evictions", "cache_refused", "wall_ms")}
            out[name]["experts_per_layer_mean"] = float(np.mean(per_layer))
        finally:
            stack.close()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="C4", choices=["C1", "C2", "C3", "C4", "C5", "P1", "P2", "P3", "PF"],
                    help="C1..C5: the MoE layer workloads; P1..P3: the token compressor alone; PF: the predictor's "
                         "feature construction alone")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-also", action="store_true", help="skip the extra decode (C5) measurement")
    ap.add_argument("--weight-sets", type=int, default=None,
                    help="distinct device copies of the layer's weights the steps rotate over (default: 2 for the "
                         "weight-streaming configs C3 and C5, 1 otherwise)")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one 1 GiB device-to-device copy first (reference kernel of known size for "
                         "scaling rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: this build is single-GPU by design (one MoE layer forward on one MI355X); "
              "run it with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(3)

    if a.calib_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")      # 1 GiB
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if a.config == "PF":
        r = measure_predictor_features(a.steps, a.warmup)
        line = {"metric": "mean_pool_GBps", "value": r["roofline"]["achieved"], "unit": "GB/s", "n_gpus": 1,
                "steps": a.steps, "warmup": a.warmup, "ms_per_step": r["mean_pool_us"] * 1e-3,
                "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
                "config": {"workload": "PF", **r["shape"]}, "roofline": r["roofline"],
                "routing_histogram_us": r["routing_histogram_us"], "lookahead_target_us": r["lookahead_target_us"],
                "predictor_mlp_top20_us": r["predictor_mlp_top20_us"]}
        print(json.dumps(line))
        return
    if a.config.startswith("P"):
        r = measure_compress(a.config, a.steps, a.warmup, not a.no_cpu_baseline)
        line = {"metric": "token_compress_visual_tokens_per_s", "value": r["visual_tokens_per_s"],
                "unit": "visual tokens/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
                "ms_per_step": r["us_per_call"] * 1e-3, "higher_is_better": True, "scaling": "weak",
                "vs_baseline": None, "dtype": "f32", "data": "synthetic",
                "config": {"workload": a.config, **r["shape"]}, "roofline": r["roofline"]}
        if "cpu_baseline" in r:
            line["cpu_baseline"] = r["cpu_baseline"]
        print(json.dumps(line))
        return
    if a.weight_sets is not None and a.weight_sets < 1:
        ap.error("--weight-sets must be at least 1")
    main_res = measure(a.config, a.steps, a.warmup, not a.no_cpu_baseline, a.weight_sets)
    line = {
        "metric": "moe_layer_tokens_per_s", "value": main_res["tokens_per_s"], "unit": "tokens/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": main_res["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": a.config, **main_res["shape"], "experts_touched": main_res["experts_touched"]},
        "layer_tflops": main_res["layer_tflops"], "layer_frac_mfma_peak": main_res["layer_frac_mfma_peak"],
        "layer_gbs": main_res["layer_gbs"], "layer_frac_hbm_peak": main_res["layer_frac_hbm_peak"],
        "roofline": main_res["roofline"], "roofline_down": main_res["roofline_down"],
        "roofline_layer": main_res["roofline_layer"], "stages_us": main_res["stages_us"],
        "step_event_us": main_res["step_event_us"],
        "prewarm_steps": main_res["prewarm_steps"], "weight_sets": main_res["weight_sets"],
    }
    if "cpu_baseline" in main_res:
        line["cpu_baseline"] = main_res["cpu_baseline"]
    if a.config == "C4" and not a.no_also:
        # the other four workloads of the headline metric, same method, no CPU-oracle leg
        keys = ("ms_per_step", "tokens_per_s", "layer_tflops", "layer_frac_mfma_peak", "layer_gbs",
                "layer_frac_hbm_peak", "experts_touched", "roofline", "roofline_down", "roofline_layer", "stages_us",
                "step_event_us", "weight_sets", "prewarm_steps", "shape")
        line["also"] = {}
        for other in ("C1", "C2", "C3", "C5"):
            r = measure(other, max(a.steps, 50), a.warmup, False)
            line["also"][other] = {k: r[k] for k in keys}
    if not a.no_also:
        line.setdefault("also", {})["token_compress_P2"] = measure_compress("P2", max(a.steps, 200), a.warmup,
                                                                            not a.no_cpu_baseline)
        # the long-video size, which takes the compressor's many-workgroup path
        line["also"]["token_compress_P3"] = measure_compress("P3", max(a.steps, 200), a.warmup, False)
        line["also"]["predictor_features"] = measure_predictor_features(max(a.steps, 200), a.warmup)
        line["also"]["expert_cache"] = measure_expert_cache()
        line["also"]["expert_cache"]["prefetch_pipeline"] = measure_prefetch_pipeline()
    print(json.dumps(line))


if __name__ == "__main__":
    main()
