#!/usr/bin/env python3
"""Benchmark of the LongFlow fused decode step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg3] [--valu|--split|--unit]
    python bench.py --report            # every workload + the uncompressed twin, as a table

A "step" is one decode step of the whole workload: every layer's cache advances by one
token (insert + attention + scores + eviction), i.e. `layers` C-ABI calls.  Inputs are
seeded synthetic tensors already resident in HBM.  Default mode prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published peak HBM3E bandwidth
DEFAULT_STEPS = {0: 512, 1: 1024, 2: 100, 3: 256, 4: 50}

# HBM bytes per launch of the streaming kernel as measured EARLIER with rocprofv3 --pmc
# (FETCH_SIZE / WRITE_SIZE, scaled by copy kernels of known size) and recorded under profiles/.
# A constant of this file, not a measurement of the run that prints it: the JSON line says so.
MEASURED_TRAFFIC = {
    ("cfg3_bf16_b64_28x4_d128_n8192_l28", "unit_mfma_kernel"): {"read_bytes": 1058529 * 1024, "write_bytes": 1076 * 1024,
                                                                "source": "profiles/unit_mfma_kernel_cfg3.txt"},
    ("cfg2_bf16_b32_28x4_d128_n4096", "unit_mfma_kernel"): {"read_bytes": 269157 * 1024, "write_bytes": 5954 * 1024,
                                                            "source": "profiles/unit_mfma_kernel_cfg2.txt"},
    ("cfg4_bf16_b128_40x8_d128_n16384", "unit_mfma_kernel"): {"read_bytes": 8458762 * 1024, "write_bytes": 3264 * 1024,
                                                              "source": "profiles/unit_mfma_kernel_cfg4.txt"},
    # the four launches of an unfused step together
    ("cfg3_bf16_b64_28x4_d128_n8192_l28", "unfused+unit_mfma_kernel"): {
        "read_bytes": 1585817 * 1024, "write_bytes": 9386 * 1024, "source": "profiles/unfused_comparison_path_cfg3_cfg4.txt"},
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cfg3", help="cfg0..cfg4 (BASELINE.json configs)")
    ap.add_argument("--valu", action="store_true", help="vector-ALU kernel instead of matrix cores")
    ap.add_argument("--split", action="store_true", help="force the split-K path")
    ap.add_argument("--unit", action="store_true", help="force the one-workgroup-per-unit fused path")
    ap.add_argument("--unfused", action="store_true",
                    help="bf16/head_dim 128: the unfused comparison path (accumulated attention weights, Fig. 1)")
    ap.add_argument("--plain", action="store_true",
                    help="plain decode attention over the full cache (LF_FLAG_ATTENTION_ONLY): no insert, score or eviction")
    ap.add_argument("--fill", action="store_true",
                    help="time filling one empty cache of the workload's geometry to the brim: one longflow_fill_steps call "
                         "against the same tokens as consecutive decode steps")
    ap.add_argument("--compress", action="store_true",
                    help="time longflow_compress_prompt: a prompt of --prompt-len tokens into one empty cache of the "
                         "workload's geometry (observation window --window, pooling width --pool-width)")
    ap.add_argument("--prompt-len", type=int, default=0, help="--compress: prompt tokens (default 4 x budget)")
    ap.add_argument("--window", type=int, default=32)
    ap.add_argument("--pool-width", type=int, default=7)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one 1 GiB device copy (a kernel of known traffic, to scale rocprofv3 byte counters)")
    ap.add_argument("--pool", type=int, default=0,
                    help="distinct input steps cycled through (0 = one per executed step, no repeats)")
    ap.add_argument("--report", action="store_true", help="all workloads and the uncompressed twin, as a table")
    ap.add_argument("--no-also", dest="also", action="store_false",
                    help="default run (cfg3) only: skip the cfg4 block that is measured after it in the same process")
    ap.add_argument("--streams", type=int, default=1,
                    help="HIP streams the independent layer caches are spread over in the timed pass (default 1: "
                         "all calls back-to-back on one stream)")
    ap.add_argument("--also-streams", type=int, default=0,
                    help="time the same steps once more with the layer calls spread over this many streams "
                         "(extra JSON fields; off by default so that a kernel trace of the default run holds "
                         "no overlapped launches)")
    return ap.parse_args()


def kernel_name(wl, flags):
    """Which kernel family the library will run for this workload (asked of the library itself)."""
    from paper_2603_11504_amd import longflow as lf
    cfg = lf.make_config(wl.batch, wl.q_heads, wl.kv_heads, wl.head_dim, wl.budget, wl.dtype, flags)
    name = lf.PATH_KERNELS[lf.longflow_plan_info(cfg).path]
    if flags & lf.LF_FLAG_MAX_FREE:
        name += "+max_free"
    return "unfused+" + name if flags & lf.LF_FLAG_UNFUSED_ACCUM else name


def cpu_baseline(wl, cache0, t_next, dev, target_s=12.0, rule="longflow"):
    """The float64 oracle, as it stands, timed on this host on a bounded sample of units, fed with
    the workload's own seeded step inputs (W.device_step, steps t_next onwards, layer 0)."""
    import numpy as np
    import torch
    from oracle import longflow_oracle as oracle
    from paper_2603_11504_amd import workloads as W

    G, D, N = wl.group, wl.head_dim, wl.budget
    threads = oracle.num_threads()
    nu = min(wl.units, max(4 * threads, 64))
    rng = np.random.default_rng(wl.seed)
    units = np.sort(rng.choice(wl.units, size=nu, replace=False))
    sel = torch.as_tensor(units, device=cache0.k_cache.device)
    n = cache0.valid_count
    ku = cache0.k_cache.reshape(wl.units, N, D)[sel][:, : n - 1].reshape(nu, 1, n - 1, D)
    vu = cache0.v_cache.reshape(wl.units, N, D)[sel][:, : n - 1].reshape(nu, 1, n - 1, D)

    def inputs(t, pick):
        q, k, v = W.device_step(wl, t, dev, 0)
        return (W.to_f64(q.reshape(wl.units, G, D)[pick]), W.to_f64(k.reshape(wl.units, 1, D)[pick]),
                W.to_f64(v.reshape(wl.units, 1, D)[pick]))

    ora = oracle.OracleCache(nu, G, 1, D, N, rule=rule)
    ora.init(W.to_f64(ku), W.to_f64(vu))
    steps, t_total = 0, 0.0
    while t_total < target_s and steps < 4096:
        q, k, v = inputs(t_next + steps, sel)
        t0 = time.perf_counter()
        ora.step(q, k, v)
        t_total += time.perf_counter() - t0
        steps += 1
    full_step_s = t_total / (nu * steps) * wl.units * wl.layers      # linear extrapolation
    # one unit alone: the oracle's loop over units has nothing to spread, so one core does the work
    one = oracle.OracleCache(1, G, 1, D, N, rule=rule)
    one.init(W.to_f64(ku[:1]), W.to_f64(vu[:1]))
    s1, t1 = 0, 0.0
    while t1 < target_s / 6 and s1 < 256:
        q, k, v = inputs(t_next + s1, sel[:1])
        t0 = time.perf_counter()
        one.step(q, k, v)
        t1 += time.perf_counter() - t0
        s1 += 1
    single_step_s = t1 / s1 * wl.units * wl.layers
    return {"value": wl.batch / full_step_s, "unit": "tokens/s", "cores": min(threads, nu), "kind": "oracle",
            "sample": f"{nu} of {wl.units * wl.layers} (layer,batch,kv-head) units x {steps} steps at n={n}, "
                      f"the workload's seeded step inputs, {t_total:.1f} s, scaled linearly to the full step",
            "ms_per_step": full_step_s * 1e3,
            "single_core_ms_per_step": single_step_s * 1e3,
            "single_core_tokens_per_s": wl.batch / single_step_s,
            "single_core_sample": f"1 unit x {s1} steps, {t1:.1f} s, scaled linearly"}


def measure(wl, flags, steps, warmup, pool=0, with_cpu=False, calibrate_copy=False,
            streams=1, also_streams=0, also_grouped=False):
    """Build the resident state, warm up, time `steps` steps, then the same again with kernel events."""
    import torch
    from paper_2603_11504_amd import longflow as lf
    from paper_2603_11504_amd import workloads as W

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    dt = W.torch_dtype(wl)
    attention_only = bool(flags & lf.LF_FLAG_ATTENTION_ONLY)

    # one cache per layer, pre-filled to N-1 rows where the workload says so (to N for plain attention)
    caches = []
    for layer in range(wl.layers):
        k0, v0 = W.device_prefill(wl, dev, layer)
        caches.append(lf.LongFlowCache(wl.batch, wl.q_heads, wl.kv_heads, wl.head_dim, wl.budget, dtype=dt,
                                       flags=flags, device=dev, k_init=k0, v_init=v0))
        del k0, v0
    # empty-start workloads fill first so that the timed steps are evicting steps
    fill = 0 if attention_only else wl.budget - wl.n_init - 1
    warm = max(warmup, 1) + max(fill, 0)
    # every executed step gets its own q/k/v (repeating inputs would plant bit-identical
    # rows in the cache, i.e. exact score ties that the real workload does not have)
    passes = 2 + (1 if also_streams > 1 else 0) + (1 if also_grouped else 0)
    npool = pool if pool > 0 else warm + passes * steps
    # per step one stacked tensor per kind, [layers, ...]: a layer's call takes its slice,
    # the grouped call takes the whole
    inputs = []
    for t in range(npool):
        per_layer = [W.device_step(wl, t, dev, layer) for layer in range(wl.layers)]
        inputs.append(tuple(torch.stack([x[i] for x in per_layer]) for i in range(3)))
        del per_layer
    torch.cuda.synchronize()

    def run(nsteps, t0=0, marks=None, nstreams=1):
        # marks: nsteps + 1 events, recorded on the launch stream at every step boundary
        # the layer caches are independent: with nstreams > 1 their calls go round-robin to
        # several streams, so one call's tail overlaps the next call's start
        pool_s = [torch.cuda.Stream(device=dev) for _ in range(nstreams)] if nstreams > 1 else None
        if pool_s:
            for s_ in pool_s:
                s_.wait_stream(torch.cuda.current_stream())
        if marks is not None:
            marks[0].record()
        for t in range(t0, t0 + nsteps):
            for layer, c in enumerate(caches):
                q, k, v = (x[layer] for x in inputs[t % npool])
                if pool_s:
                    with torch.cuda.stream(pool_s[layer % nstreams]):
                        c.decode_step(q, k, v)
                else:
                    c.decode_step(q, k, v)
            if marks is not None:
                marks[t - t0 + 1].record()
        if pool_s:
            for s_ in pool_s:
                torch.cuda.current_stream().wait_stream(s_)

    run(warm)
    torch.cuda.synchronize()
    assert all(c.valid_count == wl.budget for c in caches)
    if calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).random_()   # elementwise kernel: writes 1 GiB
        dst = torch.empty_like(src)
        dst.copy_(src)                                                        # blit kernel: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    # ---- the timed pass: exactly `steps` steps between two synchronisations.  One event per step
    # boundary on the launch stream gives the spread of the individual steps (p10 / median / p90).
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)] if streams == 1 else None
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(steps, warm, marks, nstreams=streams)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) / steps * 1e3
    calls = steps * wl.layers
    step_us = sorted(marks[i].elapsed_time(marks[i + 1]) * 1e3 for i in range(steps)) if marks else None

    # ---- the kernel pass: the same number of steps again with HIP events around every launch
    # (recorded by the library on the launch stream).  Its own wall time is taken too: the kernel
    # durations of a pass can only add up to less than the wall time of THAT pass.
    for c in caches:
        c.profile_begin(steps)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(steps, warm + steps)
    torch.cuda.synchronize()
    kernel_pass_ms_per_step = (time.perf_counter() - t0) / steps * 1e3
    ksum = 0.0
    for c in caches:
        ms, n = c.profile_end()
        assert n == steps
        ksum += ms
    kernel_us = ksum / calls * 1e3
    assert kernel_us * wl.layers <= kernel_pass_ms_per_step * 1e3 * 1.0005, \
        f"kernel time {kernel_us * wl.layers:.1f} us per step exceeds the wall time {kernel_pass_ms_per_step * 1e3:.1f} us of the same pass"
    ms_per_step_multi = None
    if also_streams > 1 and wl.layers > 1 and npool >= warm + 3 * steps:
        t0 = time.perf_counter()
        run(steps, warm + 2 * steps, nstreams=also_streams)
        torch.cuda.synchronize()
        ms_per_step_multi = (time.perf_counter() - t0) / steps * 1e3

    ms_per_step_grouped = None
    if also_grouped and npool >= warm + passes * steps:
        # all layer caches in one launch per step (they are independent in this benchmark)
        group = lf.LongFlowGroup(caches)
        base = warm + (passes - 1) * steps
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for t in range(base, base + steps):
            q, k, v = inputs[t % npool]
            group.decode_step(q, None if attention_only else k, None if attention_only else v)
        torch.cuda.synchronize()
        ms_per_step_grouped = (time.perf_counter() - t0) / steps * 1e3
        group.close()

    bytes_call = wl.kv_bytes_per_call()
    kname = kernel_name(wl, flags)
    res = {
        "ms_per_step": ms_per_step, "warm": warm, "calls": calls, "kernel_us": kernel_us, "kernel": kname,
        "bytes_call": bytes_call, "tokens_per_s": wl.batch / (ms_per_step * 1e-3),
        "step_GBs": bytes_call * wl.layers / (ms_per_step * 1e-3) / 1e9,
        "kernel_GBs": bytes_call / (kernel_us * 1e-6) / 1e9, "step_us_sorted": step_us,
        "kernel_pass_ms_per_step": kernel_pass_ms_per_step,
        "ms_per_step_multi": ms_per_step_multi, "ms_per_step_grouped": ms_per_step_grouped,
    }
    if with_cpu:
        res["cpu_baseline"] = cpu_baseline(wl, caches[0], npool, dev, rule="accumulated_attention"
                                           if flags & lf.LF_FLAG_UNFUSED_ACCUM else "longflow")
    for c in caches:
        c.close()
    del caches, inputs
    torch.cuda.empty_cache()
    return res


KERNEL_PATHS = {"unit_mfma_kernel": "fused one-launch, matrix cores",
                "split_mfma_kernel": "split-K, matrix cores",
                "split_mfma32_kernel": "split-K, matrix cores in fp32",
                "split_valu_kernel": "split-K, vector ALU"}


def summary(wl, r):
    """The per-workload figures of the JSON line: per-call time, spread of the steps, roofline block."""
    kname = r["kernel"]
    out = {
        "us_per_call": r["ms_per_step"] * 1e3 / wl.layers,
        "step_hbm_GBs": r["step_GBs"],
        "step_hbm_frac": r["step_GBs"] / HBM_PEAK_GBS,
    }
    s = r.get("step_us_sorted")
    if s:
        out["us_per_step_p10"], out["us_per_step_median"], out["us_per_step_p90"] = \
            s[len(s) // 10], s[len(s) // 2], s[(9 * len(s)) // 10]
    # kernel durations come from a second pass of the same length (HIP events around every launch);
    # that pass's own wall time stands beside them: kernel_us * calls_per_step <= it, by construction
    out["kernel_us"] = r["kernel_us"]
    out["kernel_pass"] = {"ms_per_step": r["kernel_pass_ms_per_step"],
                          "kernel_ms_per_step": r["kernel_us"] * wl.layers * 1e-3,
                          "kernel_le_wall": r["kernel_us"] * wl.layers * 1e-3 <= r["kernel_pass_ms_per_step"]}
    roof = {"bound": "hbm", "kernel": kname, "achieved": r["kernel_GBs"], "peak": HBM_PEAK_GBS,
            "unit": "GB/s", "frac": r["kernel_GBs"] / HBM_PEAK_GBS,
            "bytes_per_launch": r["bytes_call"], "avg_launch_us": r["kernel_us"], "traffic": None}
    t = MEASURED_TRAFFIC.get((wl.name, kname))
    if t:
        roof["traffic"] = t["read_bytes"] + t["write_bytes"]
        roof["traffic_read_bytes"], roof["traffic_write_bytes"] = t["read_bytes"], t["write_bytes"]
        roof["traffic_source"] = ("static: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of an earlier run of this command, "
                                  "recorded in " + t["source"] + "; not measured by the run that prints this line")
    out["roofline"] = roof
    return out


def gpu_clocks():
    """Clocks as found (nothing is pinned), right after the timed work: the current levels in the
    driver's sysfs tables (plain file reads: no child process is started from a process that holds the GPU)."""
    import glob
    out = {}
    try:
        for name in ("pp_dpm_sclk", "pp_dpm_mclk", "pp_dpm_fclk"):
            for path in sorted(glob.glob("/sys/class/drm/card*/device/" + name))[:1]:
                cur = [ln.split(":", 1)[1].replace("*", "").strip() for ln in open(path).read().splitlines() if ln.strip().endswith("*")]
                if cur:
                    out[name[len("pp_dpm_"):]] = cur[0]
    except Exception:
        return None
    return out or None


def fill_bench(a):
    """Fill phase: N tokens into an empty cache, in bulk and step by step (one layer of the workload)."""
    import torch
    from paper_2603_11504_amd import longflow as lf
    from paper_2603_11504_amd import workloads as W
    wl = W.scaled(W.CONFIGS[int(a.workload.replace("cfg", ""))], layers=1, n_init=0)
    dev = torch.device("cuda:0")
    dt = W.torch_dtype(wl)
    T = wl.budget
    g = torch.Generator(device=dev).manual_seed(wl.seed)
    q = torch.randn((T, wl.batch, wl.q_heads, wl.head_dim), device=dev, dtype=torch.float32, generator=g).to(dt)
    k = torch.randn((T, wl.batch, wl.kv_heads, wl.head_dim), device=dev, dtype=torch.float32, generator=g).to(dt)
    v = torch.randn((T, wl.batch, wl.kv_heads, wl.head_dim), device=dev, dtype=torch.float32, generator=g).to(dt)
    out = torch.empty_like(q)

    def fresh():
        return lf.LongFlowCache(wl.batch, wl.q_heads, wl.kv_heads, wl.head_dim, wl.budget, dtype=dt, device=dev)

    def timed(fn):
        c = fresh()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        fn(c)
        torch.cuda.synchronize()
        dt_s = time.perf_counter() - t0
        assert c.valid_count == wl.budget
        c.close()
        return dt_s

    def bulk(c):
        c.fill_steps(q, k, v, out=out)

    def steps(c):
        for t in range(T):
            c.decode_step(q[t], k[t], v[t], out=out[t])

    timed(bulk)                                     # warm-up (code objects, allocator)
    t_bulk = min(timed(bulk) for _ in range(3))
    t_steps = timed(steps)
    esz = wl.elem_bytes
    row = 2 * wl.units * wl.head_dim * esz          # K and V row of every unit
    bytes_steps = row * T * (T + 1) // 2            # step t reads t + 1 rows
    print(json.dumps({
        "metric": "fill_tokens_per_s", "unit": "tokens/s", "value": wl.batch * T / t_bulk,
        "config": {"workload": wl.name + "_fill_from_empty", "batch": wl.batch, "q_heads": wl.q_heads,
                   "kv_heads": wl.kv_heads, "head_dim": wl.head_dim, "budget": wl.budget, "tokens_per_sequence": T},
        "bulk_s": t_bulk, "step_by_step_s": t_steps, "speedup": t_steps / t_bulk,
        "step_by_step_tokens_per_s": wl.batch * T / t_steps,
        "step_by_step_hbm_GBs": bytes_steps / t_steps / 1e9,
        "dtype": "f32" if wl.dtype == "f32" else "bf16", "data": "synthetic", "n_gpus": 1}))


def compress_bench(a):
    """One-shot compression of a prompt longer than the budget (one layer of the workload's geometry).
    The dominant kernels are the two multi-query passes over the prompt's keys (softmax states, then
    votes); their arithmetic is the logits, 2 x T x head_dim x (window x group) multiply-adds per unit and pass."""
    import torch
    from paper_2603_11504_amd import longflow as lf
    from paper_2603_11504_amd import workloads as W
    wl = W.scaled(W.CONFIGS[int(a.workload.replace("cfg", ""))], layers=1, n_init=0)
    dev = torch.device("cuda:0")
    T = a.prompt_len or 4 * wl.budget
    Wn, keep = a.window, wl.budget - 1
    qw, kp, vp = W.device_prompt(wl, T, Wn, dev)
    times = []
    for it in range(1 + max(a.steps or 5, 1)):
        c = lf.LongFlowCache(wl.batch, wl.q_heads, wl.kv_heads, wl.head_dim, wl.budget, dtype=W.torch_dtype(wl), device=dev)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        c.compress_prompt(qw, kp, vp, keep, a.pool_width, want_pooled=False)
        e1.record()
        torch.cuda.synchronize()
        assert c.valid_count == keep
        if it:
            times.append(e0.elapsed_time(e1))
        c.close()
    ms = sorted(times)[len(times) // 2]
    flops = 2 * 2.0 * T * wl.head_dim * Wn * wl.group * wl.units          # both passes
    print(json.dumps({
        "metric": "prompt_tokens_per_s", "unit": "tokens/s", "value": wl.batch * T / (ms * 1e-3),
        "config": {"workload": wl.name + "_compress_prompt", "batch": wl.batch, "q_heads": wl.q_heads, "kv_heads": wl.kv_heads,
                   "head_dim": wl.head_dim, "budget": wl.budget, "prompt_tokens": T, "window": Wn, "pool": a.pool_width, "keep": keep},
        "ms_per_call": ms, "ms_min": min(times), "calls": len(times),
        "roofline": {"bound": "mfma", "kernel": "compress_stats_kernel + compress_votes_kernel", "achieved": flops / (ms * 1e-3) / 1e12,
                     "peak": 2500.0, "unit": "TFLOP/s", "frac": flops / (ms * 1e-3) / 1e12 / 2500.0,
                     "flops_per_call": flops, "note": "whole call (six kernels) in the denominator; see profiles/ for the split"},
        "dtype": "bf16", "data": "synthetic", "n_gpus": 1}))


def report(a):
    """Table over all BASELINE workloads plus the uncompressed twin of cfg4 (plain attention
    over all 81920 tokens, the kernel-level analogue of the paper's FullKV comparison)."""
    from paper_2603_11504_amd import longflow as lf
    from paper_2603_11504_amd import workloads as W
    rows = [(W.CONFIGS[i], 0, DEFAULT_STEPS[i]) for i in range(5)]
    twin = W.scaled(W.CONFIGS[4], name="cfg4_uncompressed_twin_n81920", budget=81920, n_init=81920)
    rows.append((twin, lf.LF_FLAG_ATTENTION_ONLY, 10))
    # plain attention with the running softmax reference (default) and as Alg. 1 prints it (max-free), A/B
    AO, MF = lf.LF_FLAG_ATTENTION_ONLY, lf.LF_FLAG_ATTENTION_ONLY | lf.LF_FLAG_MAX_FREE
    c3 = W.CONFIGS[3]
    for rep in range(2):
        rows.append((W.scaled(c3, name=f"cfg3_plain_attention_run{rep}", n_init=c3.budget), AO, 64))
        rows.append((W.scaled(c3, name=f"cfg3_plain_attention_max_free_run{rep}", n_init=c3.budget), MF, 64))
    rows.append((W.scaled(twin, name="cfg4_uncompressed_twin_n81920_max_free"), MF, 10))
    # the geometry of the paper's own kernel measurement (Fig. 1: Qwen3-8B, batch 128, 3200 slots)
    fig1 = W.scaled(W.CONFIGS[4], name="paper_fig1_geometry_b128_32x8_n3200", q_heads=32, kv_heads=8,
                    budget=3200, n_init=3199)
    rows.append((fig1, 0, 100))
    # the unfused comparison path of that figure (accumulated attention weights, one eviction per
    # step: plain attention kernel, then separate importance kernels) on the same workloads
    UNF = lf.LF_FLAG_UNFUSED_ACCUM
    rows.append((W.scaled(fig1, name=fig1.name + "_unfused"), UNF, 100))
    for i in (2, 3, 4):
        rows.append((W.scaled(W.CONFIGS[i], name=W.CONFIGS[i].name + "_unfused"), UNF, DEFAULT_STEPS[i]))
    # fp32 caches: the matrix-core kernel in fp32 arithmetic against its vector-ALU twin
    for nm, B, Hq, N, st in (("f32_b64_8x4_d128_n4096", 64, 8, 4096, 50), ("f32_b128_28x4_d128_n8192", 128, 28, 8192, 20)):
        wl32 = W.Workload(nm, "f32", B, Hq, 4, 128, N, N - 1, st, sink_scale=4.0, seed=W.BASE_SEED + 7)
        rows.append((wl32, 0, st))
        rows.append((W.scaled(wl32, name=nm + "_vector_alu"), lf.LF_FLAG_FORCE_VALU, st))
    # the small workloads again as 28 independent caches, for the one-launch-per-step column
    for i in range(3):
        rows.append((W.scaled(W.CONFIGS[i], name=W.CONFIGS[i].name + "_x28", layers=28), 0, DEFAULT_STEPS[i]))
    print(f"{'workload':44s} {'kernel':26s} {'us/step p10':>11s} {'median':>9s} {'p90':>9s} {'us/call':>9s} "
          f"{'GB/s step':>10s} {'% peak':>7s} {'GB/s kernel':>11s} {'% peak':>7s} {'tokens/s':>10s} "
          f"{'grouped us/call':>15s} {'% peak':>7s}")
    for wl, flags, steps in rows:
        if a.steps:
            steps = a.steps
        r = measure(wl, flags, steps, a.warmup, also_grouped=wl.layers > 1 and not flags & (lf.LF_FLAG_UNFUSED_ACCUM | lf.LF_FLAG_MAX_FREE))
        s = r["step_us_sorted"]
        p10, med, p90 = s[len(s) // 10], s[len(s) // 2], s[(9 * len(s)) // 10]
        print(f"{wl.name:44s} {r['kernel']:26s} {p10:11.1f} {med:9.1f} {p90:9.1f} {r['ms_per_step'] * 1e3 / wl.layers:9.1f} "
              f"{r['step_GBs']:10.1f} {100 * r['step_GBs'] / HBM_PEAK_GBS:7.1f} {r['kernel_GBs']:11.1f} "
              f"{100 * r['kernel_GBs'] / HBM_PEAK_GBS:7.1f} {r['tokens_per_s']:10.0f} " + (
                  f"{g * 1e3 / wl.layers:15.1f} {100 * r['bytes_call'] * wl.layers / (g * 1e-3) / 1e9 / HBM_PEAK_GBS:7.1f}"
                  if (g := r.get('ms_per_step_grouped')) else f"{'-':>15s} {'-':>7s}"), flush=True)


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the (batch, KV head) units are independent and would shard without exchange); "
              f"--gpus {a.gpus} is not supported", file=sys.stderr)
        sys.exit(2)
    from paper_2603_11504_amd import longflow as lf
    from paper_2603_11504_amd import workloads as W

    if a.report:
        report(a)
        return
    if a.fill:
        fill_bench(a)
        return
    if a.compress:
        compress_bench(a)
        return
    idx = int(a.workload.replace("cfg", ""))
    wl = W.CONFIGS[idx]
    steps = a.steps if a.steps is not None else DEFAULT_STEPS[idx]
    flags = lf.LF_FLAG_FORCE_VALU if a.valu else 0
    flags |= lf.LF_FLAG_FORCE_SPLIT if a.split else 0
    flags |= lf.LF_FLAG_FORCE_UNIT if a.unit else 0
    flags |= lf.LF_FLAG_UNFUSED_ACCUM if a.unfused else 0
    if a.plain:
        flags |= lf.LF_FLAG_ATTENTION_ONLY
        wl = W.scaled(wl, name=wl.name + "_plain_attention", n_init=wl.budget)
    r = measure(wl, flags, steps, a.warmup, pool=a.pool, with_cpu=not a.no_cpu_baseline,
                calibrate_copy=a.calibrate_copy, streams=a.streams, also_streams=a.also_streams if a.streams == 1 else 0,
                also_grouped=a.streams == 1 and wl.layers > 1 and not a.unfused and not a.plain)
    kname = r["kernel"]
    out = {
        "metric": "decode_tokens_per_s",
        "value": r["tokens_per_s"],
        "unit": "tokens/s",
        "n_gpus": 1, "steps": steps, "warmup": r["warm"], "ms_per_step": r["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if wl.dtype == "f32" else "bf16",   # bf16 operands, f32 accumulation
        "data": "synthetic",
        "config": {"workload": wl.name, "batch": wl.batch, "q_heads": wl.q_heads, "kv_heads": wl.kv_heads,
                   "head_dim": wl.head_dim, "budget": wl.budget, "layers": wl.layers,
                   "calls_per_step": wl.layers, "streams": a.streams,
                   "kernel_path": ("unfused comparison path (insert, attention, accumulate, decide) around: "
                                   if a.unfused else "plain attention, no by-products: " if a.plain else "") +
                                  KERNEL_PATHS[kname.split("+")[-1]]},
    }
    out.update(summary(wl, r))
    out["gpu_clocks"] = gpu_clocks()
    if r.get("ms_per_step_multi"):
        # the same steps with the independent layer calls spread over several streams (tails overlap)
        out["also_streams"] = a.also_streams
        out["ms_per_step_multi_stream"] = r["ms_per_step_multi"]
        out["step_hbm_frac_multi_stream"] = r["bytes_call"] * wl.layers / (r["ms_per_step_multi"] * 1e-3) / 1e9 / HBM_PEAK_GBS
    if r.get("ms_per_step_grouped"):
        # the same steps with all layer caches served by one launch per step
        out["ms_per_step_grouped"] = r["ms_per_step_grouped"]
        out["step_hbm_frac_grouped"] = r["bytes_call"] * wl.layers / (r["ms_per_step_grouped"] * 1e-3) / 1e9 / HBM_PEAK_GBS
    if "cpu_baseline" in r:
        out["cpu_baseline"] = r["cpu_baseline"]
    if a.also and a.workload == "cfg3" and flags == 0 and a.streams == 1:
        # the other workload the bandwidth target names, measured by this same process right after:
        # one cache, batch 128, 16384 slots (8 GiB of K and V per call)
        w4 = W.CONFIGS[4]
        r4 = measure(w4, 0, DEFAULT_STEPS[4], a.warmup)
        blk = {"workload": w4.name, "batch": w4.batch, "q_heads": w4.q_heads, "kv_heads": w4.kv_heads,
               "head_dim": w4.head_dim, "budget": w4.budget, "layers": w4.layers, "steps": DEFAULT_STEPS[4],
               "warmup": r4["warm"], "ms_per_step": r4["ms_per_step"], "tokens_per_s": r4["tokens_per_s"],
               "kernel_path": KERNEL_PATHS[r4["kernel"].split("+")[-1]]}
        blk.update(summary(w4, r4))
        out["also"] = [blk]
    print(json.dumps(out))


if __name__ == "__main__":
    main()
