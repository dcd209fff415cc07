#!/usr/bin/env python3
"""Decode throughput of one layer window on one MI355X.

A step = one pass of the whole hot path (every layer of the window: Q4_K projections with fused
RMSNorm / SwiGLU / residuals, RoPE + fp16 KV append, GQA attention) over one batch of T tokens
of seeded synthetic input that is already resident in HBM.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config c3] [--no-cpu-baseline] [--copy-calibration]
  python bench.py --batch B ...   a side measurement: B independent sequences, one token each per step
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X published HBM3E bandwidth


def gate_up_traffic_bytes():
    """HBM bytes of one gate/up launch of config 3 (one token) as the committed counter summary states them:
    rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE, each scaled by what the same counter reads for a plain 256 MiB copy
    (profiles/gemv_q4k_persistent_c3_hbm_traffic.txt, the "gate/up projections" row).  None if the file or the row is
    not there."""
    import re
    try:
        with open(os.path.join(ROOT, "profiles", "gemv_q4k_persistent_c3_hbm_traffic.txt")) as f:
            for line in f:
                if line.startswith("gate/up projections"):
                    m = re.search(r"\)\s+[0-9.]+\s+([0-9][0-9 ]+[0-9])\s+\(read", line)
                    return int(m.group(1).replace(" ", "")) if m else None
    except OSError:
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="c3")
    ap.add_argument("--layers", type=int, default=0, help="override the number of layers (debugging)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-configs", action="store_true", help="config 3 only: skip the short runs of configs 1, 2 and 4")
    ap.add_argument("--batch", type=int, default=0,
                    help="side measurement: B sequences of the config's context length, one token each per step")
    ap.add_argument("--format", default="", choices=["", "q5_k", "q6_k", "q8_0", "f16", "f32"],
                    help="side measurement: the mat-vec of another weight format at the output layer's and the down projection's shape")
    ap.add_argument("--mix", action="store_true",
                    help="side measurement: the config's window with the V and down projections of every other layer in Q6_K "
                         "(a common mix of a \"Q4K\" model), against the oracle")
    ap.add_argument("--prefill", type=int, default=0,
                    help="prompt processing: the config's window for this many prompt tokens in one call (time to the first token)")
    ap.add_argument("--generate", type=int, default=0,
                    help="with --prefill P: after the prompt call, this many one-token steps; reports both times (the paper's TTFT and TPOT, "
                         "for this window)")
    ap.add_argument("--device-profile", action="store_true",
                    help="side measurement: the device-profiler quantities of the paper's latency model on this GPU, and the "
                         "model's estimate of the config's window step next to the measured one")
    ap.add_argument("--halda", action="store_true",
                    help="side measurement (CPU only, no GPU needed): the scheduler's time for rings of 4 to 32 devices and an "
                         "80-layer model (the paper: 10-12 ms)")
    ap.add_argument("--launch-cost", action="store_true",
                    help="side measurement: one-token Q4_K mat-vecs of 8192 columns and 2048 to 114688 rows, cold weights; a straight "
                         "line through time against bytes gives the fixed cost of a launch and the rate of its streaming phase")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run three plain 256 MiB device copies first (reference kernel of known traffic for counter runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: the library has no multi-GPU path (run with --gpus 1)")
    if args.halda:
        return bench_halda(args)

    import numpy as np
    import torch
    import paper_2504_08791_amd as prima
    from workloads import synth
    from workloads.configs import CONFIGS

    cfg = CONFIGS[args.config]
    if args.layers:
        cfg = cfg.with_(n_layers=args.layers)
    if args.batch:
        return bench_batch(args, cfg)
    if args.format:
        return bench_format(args)
    if args.prefill and args.generate:
        return bench_generate(args, cfg)
    if args.prefill:
        return bench_prefill(args, cfg)
    if args.device_profile:
        return bench_device_profile(args, cfg)
    if args.launch_cost:
        return bench_launch_cost(args)
    if args.mix:
        return bench_mix(args, cfg)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    want_cpu = not args.no_cpu_baseline
    if args.config == "c0":
        return bench_c0(args, cfg)
    main_run = run_window_config(args, cfg, args.steps, args.warmup, want_cpu, True, args.copy_calibration)
    out = main_run["line"]
    if args.config == "c3" and not args.layers and not args.no_other_configs:
        # the other benchmark configurations, shorter: config 1 (12 layers), config 2 (16 layers, 4 tokens verified
        # jointly) and config 4's shape at 20 of its 80 layers with the output layer, 8 tokens verified jointly
        others = {}
        for name, layers in (("c1", 0), ("c2", 0), ("c4k8", 20)):
            ocfg = CONFIGS[name].with_(n_layers=layers) if layers else CONFIGS[name]
            r = run_window_config(args, ocfg, 20, 5, False, False, False)["line"]
            others[name] = {"workload": r["config"]["workload"], "tokens_per_step": ocfg.T, "ms_per_step": r["ms_per_step"],
                            "median_ms_per_step": r["median_ms_per_step"], "tokens_per_s": r["value"],
                            "window_hbm_gbps": r["window_hbm_gbps"], "window_hbm_frac": r["window_hbm_frac"],
                            "per_launch_us": r["per_launch_us"], "gate_up_frac": r["roofline"]["frac"]}
        out["other_configs"] = others
    print(json.dumps(out), flush=True)


def cpu_model():
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def time_steps(step, stream, warmup, steps):
    """W untimed steps, then K steps between two events (the mean) with an event after every step (the median); all on
    `stream`, nothing waits in between."""
    import torch
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    t0 = time.perf_counter()
    evs[0].record(stream)
    for i in range(steps):
        step()
        evs[i + 1].record(stream)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    each = sorted(evs[i].elapsed_time(evs[i + 1]) for i in range(steps))
    median = each[steps // 2] if steps % 2 else 0.5 * (each[steps // 2 - 1] + each[steps // 2])
    return evs[0].elapsed_time(evs[steps]) / steps, median, wall_ms / steps


def run_window_config(args, cfg, steps, warmup, want_cpu, with_probe, copy_calibration):
    """Builds the window of `cfg` in HBM (and walks the oracle over the same layers when asked), times it, measures
    every kind of launch on its own, and returns the JSON line as a dict."""
    import numpy as np
    import torch
    import paper_2504_08791_amd as prima
    from workloads import synth

    d = cfg.dims
    dev = torch.device("cuda:0")
    cap = cfg.n_past + cfg.T
    x_host = synth.window_input(cfg)

    # --- build the window in HBM, one layer at a time; the oracle walks the same layers on the host ---
    if want_cpu:
        import oracle
    dev_layers = []
    h_ref = x_host.astype(np.float64)
    cpu_seconds = 0.0
    t_build = time.time()
    for l in range(cfg.n_layers):
        t = synth.layer_tensors(cfg, l, kv_cap=cap)
        dev_layers.append({k: torch.from_numpy(v).to(dev) for k, v in t.items()})
        if want_cpu:
            t0 = time.perf_counter()
            h_ref = oracle.layer(d, t, h_ref, cfg.n_past)     # appends to the host copy of the cache only
            cpu_seconds += time.perf_counter() - t0
        del t
    print(f"[bench] built {cfg.n_layers} layers in {time.time() - t_build:.1f} s "
          f"(oracle: {cpu_seconds:.1f} s)", file=sys.stderr, flush=True)

    win = prima.Window(d, dev_layers, cap, T_max=cfg.T)
    x = torch.from_numpy(x_host).to(dev)
    y = torch.empty_like(x)
    stream = torch.cuda.current_stream()
    # a configuration with an output layer (config 4): final RMSNorm + lm_head follow the window in every step
    head = None
    if cfg.vocab:
        out_t = synth.output_layer_tensors(cfg)
        head = {k: torch.from_numpy(v).to(dev) for k, v in out_t.items()}
        logits = torch.empty((cfg.T, cfg.vocab), dtype=torch.float32, device=dev)
        head_ws = torch.empty(max(256, prima.lm_head_workspace_bytes(d, cfg.vocab, cfg.T)), dtype=torch.uint8, device=dev)
        if want_cpu:
            t0 = time.perf_counter()
            logits_ref = oracle.lm_head(d, out_t["g_final"], out_t["w_lm"], h_ref)
            cpu_seconds += time.perf_counter() - t0
        del out_t

    def step():
        win.decode(x, cfg.n_past, x_out=y)
        if head is not None:
            prima.lm_head(d, head["g_final"], head["w_lm"], y, logits, head_ws)

    if copy_calibration:
        src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    ms_per_step, median_ms, wall_ms_step = time_steps(step, stream, warmup, steps)
    tokens_per_s = cfg.T / (ms_per_step * 1e-3)
    bytes_step = cfg.bytes_per_step()   # the output layer's bytes included when there is one

    # --- what a plain linear read reaches on this device (4 GiB, far beyond the last-level cache) ---
    stream_read_gbps = None
    stream_read_nt_gbps = None
    if with_probe:
        probe = torch.empty(4 * 1024 ** 3, dtype=torch.uint8, device=dev)
        probe.zero_()
        sink = torch.zeros(1, dtype=torch.int32, device=dev)
        for _ in range(2):
            prima.stream_read_probe(probe, sink)
        p0, p1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        p0.record(stream)
        for _ in range(5):
            prima.stream_read_probe(probe, sink)
        p1.record(stream)
        torch.cuda.synchronize()
        stream_read_gbps = probe.numel() * 5 / (p0.elapsed_time(p1) * 1e-3) / 1e9
        # the same read with non-temporal loads, the way the one-token mat-vec requests its weights
        for _ in range(2):
            prima.stream_read_probe(probe, sink, nt=True)
        p0.record(stream)
        for _ in range(5):
            prima.stream_read_probe(probe, sink, nt=True)
        p1.record(stream)
        torch.cuda.synchronize()
        stream_read_nt_gbps = probe.numel() * 5 / (p0.elapsed_time(p1) * 1e-3) / 1e9
        del probe

    # --- per kind of launch: each replayed on its own, once per layer, between two HIP events on the
    #     same stream (the dominant kernel is the gate/up projection) ---
    n_prof = 5
    acc = {}
    for _ in range(n_prof):
        _, kinds = win.decode_profiled(x, cfg.n_past, x_out=y)
        for k, (ms, n) in kinds.items():
            a = acc.setdefault(k, [0.0, 0])
            a[0] += ms
            a[1] += n
    per_launch_us = {k: (v[0] / v[1] * 1e3) for k, v in acc.items() if v[1]}
    gate_up_bytes = 2 * d.ffn * (d.e // 256) * 144      # algorithmic bytes of one gate/up launch
    gu_us = per_launch_us["gate_up"]
    achieved = gate_up_bytes / (gu_us * 1e-6) / 1e9
    qd, kvd = d.n_q_heads * d.head_dim, d.n_kv_heads * d.head_dim
    kind_bytes = {"qkv": (qd + 2 * kvd) * (d.e // 256) * 144, "attn": d.kv_bytes_per_layer(cfg.n_past + cfg.T),
                  "wo": d.e * (qd // 256) * 144, "gate_up": gate_up_bytes, "down": d.e * (d.ffn // 256) * 144}

    out = {
        "metric": "decode tokens/s per layer window; achieved HBM GB/s vs MI355X peak",
        "value": round(tokens_per_s, 2),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {
            "workload": f"{cfg.name}: {cfg.n_layers}-layer window, e={d.e}, Hq/Hkv={d.n_q_heads}/{d.n_kv_heads}, "
                        f"ffn={d.ffn}, T={cfg.T}, n_kv={cfg.n_past}, Q4_K weights, fp16 KV"
                        + (f", final RMSNorm + {cfg.vocab}-row Q4_K output layer" if cfg.vocab else ""),
            "tokens_per_step": cfg.T,
            "layers": cfg.n_layers,
            "kv_context": cfg.n_past,
        },
        "median_ms_per_step": round(median_ms, 4),
        "window_bytes_per_step": bytes_step,
        "window_hbm_gbps": round(bytes_step / (ms_per_step * 1e-3) / 1e9, 1),
        "window_hbm_frac": round(bytes_step / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
        "wall_ms_per_step": round(wall_ms_step, 4),
        "per_launch_us": {k: round(v, 2) for k, v in per_launch_us.items()},
        # every kind of launch against the same peak: algorithmic bytes of the launch / its duration / 8 TB/s
        "per_launch_hbm_frac": {k: round(kind_bytes[k] / (per_launch_us[k] * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4)
                                for k in kind_bytes if k in per_launch_us},
        "roofline": {
            "bound": "hbm",
            "kernel": f"gemv_q4k_persistent_kernel<{cfg.T}> as launched for the gate/up projections (RMSNorm in front, SwiGLU behind)",
            "achieved": round(achieved, 1),
            "peak": HBM_PEAK_GBPS,
            "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBPS, 4),
            "bytes_per_launch": gate_up_bytes,
            "avg_launch_us": round(gu_us, 2),
            "traffic": gate_up_traffic_bytes() if (cfg.name == "c3" and cfg.T == 1) else None,
        },
    }
    if stream_read_gbps is not None:
        out["plain_read_gbps"] = round(stream_read_gbps, 1)  # linear 128-bit read of 4 GiB: the practical ceiling
        out["plain_read_nt_gbps"] = round(stream_read_nt_gbps, 1)  # the same with non-temporal loads (as the one-token mat-vec reads its weights)
    if want_cpu:
        got = y.cpu().numpy().astype(np.float64)
        rms = np.sqrt((h_ref ** 2).mean(axis=1, keepdims=True))
        err = float((np.abs(got - h_ref) / np.maximum(np.abs(h_ref), np.maximum(rms, 1e-30))).max())
        out["max_rel_err_vs_oracle"] = err
        if head is not None:
            gl = logits.cpu().numpy().astype(np.float64)
            rms = np.sqrt((logits_ref ** 2).mean(axis=1, keepdims=True))
            out["max_rel_err_logits_vs_oracle"] = float((np.abs(gl - logits_ref) / np.maximum(np.abs(logits_ref), np.maximum(rms, 1e-30))).max())
        out["cpu_baseline"] = {
            "value": round(cfg.T / cpu_seconds, 4),
            "unit": "tokens/s",
            "cores": oracle.num_threads(),
            "cpu_model": cpu_model(),
            "kind": "oracle",
            "sample": f"the whole {cfg.n_layers}-layer window, {cfg.T} token(s), once ({cpu_seconds:.1f} s of CPU time; "
                      "tensor generation excluded)",
        }
        # config 0 (one 8B-shaped layer, one token) on one thread and on all of them
        from workloads.configs import CONFIGS as _C
        c0 = _C["c0"]
        t0l = synth.layer_tensors(c0, 0)
        x0 = synth.window_input(c0).astype(np.float64)
        n_thr = oracle.num_threads()
        res = {}
        for label, thr in (("all_threads", n_thr), ("one_thread", 1)):
            oracle.set_num_threads(thr)
            tt = time.perf_counter()
            oracle.layer(c0.dims, {k: (v.copy() if k.endswith("cache") else v) for k, v in t0l.items()}, x0, c0.n_past)
            res[label] = round(1.0 / (time.perf_counter() - tt), 3)
        oracle.set_num_threads(n_thr)
        out["cpu_baseline"]["config0_layer_tokens_per_s"] = res
    del dev_layers, win
    torch.cuda.empty_cache()
    return {"line": out}


def bench_c0(args, cfg):
    """Config 0 (one 8B-shaped layer, 125 MB): the layer fits the 256 MB last-level cache, so the same layer timed
    again and again measures that cache.  Cold: six copies of the layer (750 MB) taken in rotation, one per step;
    warm: one copy every step.  Launch-bound either way (five launches for 15.6 us of traffic at the peak rate)."""
    import numpy as np
    import torch
    import paper_2504_08791_amd as prima
    from workloads import synth

    d = cfg.dims
    dev = torch.device("cuda:0")
    cap = cfg.n_past + cfg.T
    host = synth.layer_tensors(cfg, 0, kv_cap=cap)
    copies = 6
    wins = [prima.Window(d, [{k: torch.from_numpy(v).to(dev) for k, v in host.items()}], cap, T_max=cfg.T) for _ in range(copies)]
    x = torch.from_numpy(synth.window_input(cfg)).to(dev)
    y = torch.empty_like(x)
    stream = torch.cuda.current_stream()
    counter = [0]

    def cold():
        wins[counter[0] % copies].decode(x, cfg.n_past, x_out=y)
        counter[0] += 1

    def warm():
        wins[0].decode(x, cfg.n_past, x_out=y)

    cold_ms, cold_med, wall = time_steps(cold, stream, args.warmup, args.steps)
    warm_ms, warm_med, _ = time_steps(warm, stream, args.warmup, args.steps)
    bytes_step = cfg.bytes_per_step()
    out = {
        "metric": "decode tokens/s per layer window; achieved HBM GB/s vs MI355X peak", "value": round(1e3 / cold_ms, 1), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(cold_ms, 5), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"c0: one layer, e={d.e}, ffn={d.ffn}, T=1, n_kv={cfg.n_past}; cold = {copies} copies of the layer in rotation "
                               f"({copies * bytes_step / 1e6:.0f} MB, beyond the 256 MB last-level cache)", "tokens_per_step": 1, "layers": 1},
        "cold": {"ms_per_step": round(cold_ms, 5), "median_ms_per_step": round(cold_med, 5), "window_hbm_gbps": round(bytes_step / cold_ms / 1e6, 1),
                 "window_hbm_frac": round(bytes_step / cold_ms / 1e6 / HBM_PEAK_GBPS, 4)},
        "warm_cache_resident": {"ms_per_step": round(warm_ms, 5), "median_ms_per_step": round(warm_med, 5),
                                "note": "the same 125 MB layer every step: served by the last-level cache, not an HBM figure"},
        "window_bytes_per_step": bytes_step, "wall_ms_per_step": round(wall, 5),
    }
    if not args.no_cpu_baseline:
        import oracle
        ref = oracle.layer(d, host, synth.window_input(cfg).astype(np.float64), cfg.n_past)
        got = y.cpu().numpy().astype(np.float64)
        rms = np.sqrt((ref ** 2).mean(axis=1, keepdims=True))
        out["max_rel_err_vs_oracle"] = float((np.abs(got - ref) / np.maximum(np.abs(ref), rms)).max())
    print(json.dumps(out), flush=True)


def bench_batch(args, cfg):
    """B independent sequences (each with the config's context in its own caches) advance by one token per step."""
    import numpy as np
    import torch
    import paper_2504_08791_amd as prima
    from workloads import synth

    d, B = cfg.dims, args.batch
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    cap = cfg.n_past + 1
    n_past = [cfg.n_past] * B
    want_cpu = not args.no_cpu_baseline
    host_layers, dev_layers = [], []
    for l in range(cfg.n_layers):
        t = synth.layer_tensors(cfg.with_(n_past=0), l, kv_cap=1)   # weights and gains; the window's own caches stay unused
        dev_layers.append({k: torch.from_numpy(v).to(dev) for k, v in t.items()})
        dev_layers[-1]["k_cache"] = torch.zeros((d.n_kv_heads, cap, d.head_dim), dtype=torch.float16, device=dev)
        dev_layers[-1]["v_cache"] = dev_layers[-1]["k_cache"]
        if want_cpu:
            host_layers.append(t)
    caches = synth.batch_caches(cfg, cfg.n_layers, n_past, cap)
    dev_caches = [[(torch.from_numpy(k).to(dev), torch.from_numpy(v).to(dev)) for k, v in per_layer] for per_layer in caches]
    win = prima.Window(d, dev_layers, cap, T_max=B)
    x_host = synth.batch_input(cfg, B)
    x = torch.from_numpy(x_host).to(dev)
    y = torch.empty_like(x)
    stream = torch.cuda.current_stream()
    for _ in range(args.warmup):
        win.decode_batch(x, n_past, dev_caches, x_out=y)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(args.steps):
        win.decode_batch(x, n_past, dev_caches, x_out=y)
    e1.record(stream)
    torch.cuda.synchronize()
    ms_per_step = e0.elapsed_time(e1) / args.steps
    out = {
        "metric": "decode tokens/s per layer window, batch of independent sequences",
        "value": round(B / (ms_per_step * 1e-3), 2), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name} shape: {cfg.n_layers}-layer window, {B} sequences x 1 token, n_kv={cfg.n_past} each, "
                               "Q4_K weights, fp16 KV", "tokens_per_step": B, "layers": cfg.n_layers, "kv_context": cfg.n_past},
    }
    if want_cpu:
        import oracle
        t0 = time.perf_counter()
        ref = oracle.window_batch(d, host_layers, caches, x_host.astype(np.float64), n_past)
        cpu_seconds = time.perf_counter() - t0
        got = y.cpu().numpy().astype(np.float64)
        rms = np.sqrt((ref ** 2).mean(axis=1, keepdims=True))
        out["max_rel_err_vs_oracle"] = float((np.abs(got - ref) / np.maximum(np.abs(ref), np.maximum(rms, 1e-30))).max())
        out["cpu_baseline"] = {"value": round(B / cpu_seconds, 4), "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
                               "sample": f"the whole step once ({cpu_seconds:.1f} s of CPU time)"}
    print(json.dumps(out), flush=True)


def bench_prefill(args, cfg):
    """Prompt processing (the paper's time to the first token, Sec. 4.1, for this device's window): T prompt tokens
    through all layers in one call, empty caches.  A step is one such call."""
    import numpy as np
    import torch
    import paper_2504_08791_amd as prima
    from workloads import synth

    d, T = cfg.dims, args.prefill
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    cfg = cfg.with_(T=T, n_past=0)
    want_cpu = not args.no_cpu_baseline
    dev_layers, host0 = [], None
    for l in range(cfg.n_layers):
        t = synth.layer_tensors(cfg, l, kv_cap=T)
        dev_layers.append({k: torch.from_numpy(v).to(dev) for k, v in t.items()})
        if l == 0 and want_cpu:
            host0 = t
    win = prima.Window(d, dev_layers, T, T_max=1)
    x_host = synth.window_input(cfg)
    x = torch.from_numpy(x_host).to(dev)
    y = torch.empty_like(x)
    stream = torch.cuda.current_stream()
    for _ in range(args.warmup):
        win.prefill(x, 0, x_out=y)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(args.steps):
        win.prefill(x, 0, x_out=y)
    e1.record(stream)
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / args.steps
    qd, kvd = d.n_q_heads * d.head_dim, d.n_kv_heads * d.head_dim
    weights = d.e * (qd + 2 * kvd) + qd * d.e + 3 * d.ffn * d.e
    flops_step = 2.0 * weights * T * cfg.n_layers
    # the dominant launch on its own: the gate projection's matrix product (RMSNorm in front), between two events
    h = torch.randn((T, d.e), device=dev)
    g = torch.empty((T, d.ffn), device=dev)
    ws = torch.empty(prima._ffi.lib().prima_gemm_workspace_bytes(T, d.e), dtype=torch.uint8, device=dev)
    wg, gain = dev_layers[0]["wgate"], dev_layers[0]["g_ffn"]
    for _ in range(3):
        prima.q4k_gemm(wg, h, gain=gain, eps=d.rms_eps, y=g, workspace=ws)
    p0, p1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    p0.record(stream)
    for i in range(20):
        prima.q4k_gemm(dev_layers[i % cfg.n_layers]["wgate"], h, gain=gain, eps=d.rms_eps, y=g, workspace=ws)
    p1.record(stream)
    torch.cuda.synchronize()
    gate_us = p0.elapsed_time(p1) / 20 * 1e3
    gate_flops = 2.0 * d.ffn * d.e * T
    achieved = gate_flops / (gate_us * 1e-6) / 1e12
    out = {
        "metric": "prompt tokens/s per layer window (time to the first token of this window = ms_per_step)",
        "value": round(T / (ms * 1e-3), 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f16 x f16 -> f32",
        "data": "synthetic",
        "config": {"workload": f"{cfg.name} shape: {cfg.n_layers}-layer window, e={d.e}, ffn={d.ffn}, {T} prompt tokens, empty caches, "
                               "Q4_K weights, fp16 KV", "tokens_per_step": T, "layers": cfg.n_layers},
        "window_tflops": round(flops_step / (ms * 1e-3) / 1e12, 1),
        "roofline": {
            "bound": "mfma",
            "kernel": "prima_q4k_gemm as called for the gate projection (token scales, activation split and q4k_gemm_kernel; RMSNorm in front)",
            "achieved": round(achieved, 1), "peak": 2500.0, "unit": "TFLOP/s", "frac": round(achieved / 2500.0, 4),
            "flops_per_launch": gate_flops, "avg_launch_us": round(gate_us, 1),
            "mfma_passes": 2,   # every activation enters as hi + lo: the matrix cores do twice the algorithmic work
            "traffic": None,
        },
    }
    if want_cpu:
        import oracle
        n_s = min(64, T)
        win1 = prima.Window(d, [dict(dev_layers[0], k_cache=torch.zeros_like(dev_layers[0]["k_cache"]),
                                     v_cache=torch.zeros_like(dev_layers[0]["v_cache"]))], T, T_max=1)
        got = win1.prefill(x[:n_s].contiguous(), 0).cpu().numpy().astype(np.float64)
        t0 = time.perf_counter()
        ref = oracle.layer(d, host0, x_host[:n_s].astype(np.float64), 0)
        cpu_seconds = time.perf_counter() - t0
        rms = np.sqrt((ref ** 2).mean(axis=1, keepdims=True))
        out["max_rel_err_vs_oracle"] = float((np.abs(got - ref) / np.maximum(np.abs(ref), np.maximum(rms, 1e-30))).max())
        out["cpu_baseline"] = {"value": round(n_s / (cpu_seconds * cfg.n_layers), 4), "unit": "tokens/s", "cores": oracle.num_threads(),
                               "kind": "oracle", "sample": f"layer 0 for the first {n_s} prompt tokens ({cpu_seconds:.1f} s of CPU time), "
                                                           f"scaled to {cfg.n_layers} layers"}
    print(json.dumps(out), flush=True)


def bench_generate(args, cfg):
    """A prompt of P tokens through the window in one call, then N one-token steps (Sec. 4.1 reports both: time to the first
    token and time per output token).  A step is the whole sequence prompt + N tokens; `value` is the decode rate."""
    import torch
    import paper_2504_08791_amd as prima
    from workloads import synth

    d, P, N = cfg.dims, args.prefill, args.generate
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    cfg = cfg.with_(T=P, n_past=0)
    cap = P + N
    dev_layers = []
    for l in range(cfg.n_layers):
        t = synth.layer_tensors(cfg, l, kv_cap=cap)
        dev_layers.append({k: torch.from_numpy(v).to(dev) for k, v in t.items()})
    win = prima.Window(d, dev_layers, cap, T_max=1)
    x = torch.from_numpy(synth.window_input(cfg)).to(dev)
    nxt = torch.from_numpy(synth.batch_input(cfg, 1)).to(dev)
    y, y1 = torch.empty_like(x), torch.empty_like(nxt)
    stream = torch.cuda.current_stream()

    def sequence(ev=None):
        win.prefill(x, 0, x_out=y)
        if ev is not None:
            ev.record(stream)
        for i in range(N):
            win.decode(nxt, P + i, x_out=y1)

    for _ in range(args.warmup):
        sequence()
    torch.cuda.synchronize()
    ttft, total = 0.0, 0.0
    for _ in range(args.steps):
        e0, e1, e2 = (torch.cuda.Event(enable_timing=True) for _ in range(3))
        e0.record(stream)
        sequence(e1)
        e2.record(stream)
        torch.cuda.synchronize()
        ttft += e0.elapsed_time(e1)
        total += e0.elapsed_time(e2)
    ttft /= args.steps
    total /= args.steps
    tpot = (total - ttft) / N
    out = {
        "metric": "output tokens/s per layer window after a prompt (1000 / TPOT of this window); TTFT of this window alongside",
        "value": round(1e3 / tpot, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(total, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name} shape: {cfg.n_layers}-layer window, {P} prompt tokens in one call, then {N} one-token steps; "
                               "Q4_K weights, fp16 KV", "tokens_per_step": P + N, "layers": cfg.n_layers},
        "ttft_ms": round(ttft, 3), "tpot_ms": round(tpot, 4),
    }
    print(json.dumps(out), flush=True)


def bench_mix(args, cfg):
    """The config's window with matrices in two formats: V and down projections of every other layer in Q6_K, the rest
    Q4_K.  One token step timed as the main measurement is; bytes are those of the tensors as stored."""
    import numpy as np
    import torch
    import paper_2504_08791_amd as prima
    from paper_2504_08791_amd import profiler
    from workloads import synth

    d = cfg.dims
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    cap = cfg.n_past + cfg.T
    formats = [({"wv": "q6_k", "wdown": "q6_k"} if l % 2 == 0 else {}) for l in range(cfg.n_layers)]
    want_cpu = not args.no_cpu_baseline
    x_host = synth.window_input(cfg)
    h = x_host.astype(np.float64)
    dev_layers, cpu_seconds = [], 0.0
    for l in range(cfg.n_layers):
        t = synth.layer_tensors(cfg, l, kv_cap=cap, formats=formats[l])
        dev_layers.append({k: torch.from_numpy(v).to(dev) for k, v in t.items()})
        if want_cpu:
            import oracle
            t0 = time.perf_counter()
            h = oracle.layer(d, t, h, cfg.n_past, formats=formats[l])
            cpu_seconds += time.perf_counter() - t0
        del t
    win = prima.Window(d, dev_layers, cap, T_max=cfg.T, formats=formats)
    x = torch.from_numpy(x_host).to(dev)
    y = torch.empty_like(x)
    stream = torch.cuda.current_stream()
    for _ in range(args.warmup):
        win.decode(x, cfg.n_past, x_out=y)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(args.steps):
        win.decode(x, cfg.n_past, x_out=y)
    e1.record(stream)
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / args.steps
    step_bytes = sum(profiler.model_profile(d, f)["b"] for f in formats) + cfg.n_layers * d.kv_bytes_per_layer(cfg.n_past + cfg.T)
    out = {
        "metric": "decode tokens/s per layer window, matrices in two formats", "value": round(cfg.T / (ms * 1e-3), 2), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: {cfg.n_layers}-layer window, T={cfg.T}, n_kv={cfg.n_past}; V and down projections of every "
                               "other layer in Q6_K, the rest Q4_K; fp16 KV", "tokens_per_step": cfg.T, "layers": cfg.n_layers},
        "window_bytes_per_step": step_bytes, "window_hbm_gbps": round(step_bytes / (ms * 1e-3) / 1e9, 1),
        "window_hbm_frac": round(step_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
    }
    if want_cpu:
        got = y.cpu().numpy().astype(np.float64)
        rms = np.sqrt((h ** 2).mean(axis=1, keepdims=True))
        out["max_rel_err_vs_oracle"] = float((np.abs(got - h) / np.maximum(np.abs(h), np.maximum(rms, 1e-30))).max())
        out["cpu_baseline"] = {"value": round(cfg.T / cpu_seconds, 4), "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
                               "sample": f"the whole window once ({cpu_seconds:.1f} s of CPU time; tensor generation excluded)"}
    print(json.dumps(out), flush=True)


def bench_halda(args):
    """Scheduling latency of Halda (Sec. 3.3: 10-12 ms on 4 to 32 devices) on seeded synthetic rings: devices of mixed
    operating systems and GPUs, an 80-layer model (its divisors below 80 that leave every device a layer are the candidate
    numbers of rounds).  Algorithm 1 as the paper gives it, and with this repository's refinement over the set assignment
    behind it.  Runs on the CPU alone."""
    import statistics
    from paper_2504_08791_amd import halda
    from workloads.lda import random_instance

    def objects(model, devices):
        mo = halda.Model(L=model["L"], flops=dict(model["flops"]), flops_out=dict(model["flops_out"]), b=model["b"], b_i=model["b_i"],
                         b_o=model["b_o"], V=model["V"], kv_bytes_per_token=model["kv"], n_kv=model["n_kv"], c_cpu=model["c_cpu"],
                         c_gpu=model["c_gpu"])
        ds = [halda.Device(name=f"d{m}", os=d["os"], gpu=d["gpu"], uma=d["uma"], d_avail=d["d_avail"], d_gpu_avail=d["d_gpu_avail"],
                           d_swapout=d["swap_cap"], s_disk=d["s_disk"], s_cpu=dict(d["s_cpu"]), s_gpu=dict(d["s_gpu"]), T_cpu=d["T_cpu"],
                           T_gpu=d["T_gpu"], t_kv_cpy_cpu=d["t_kv_cpy_cpu"], t_kv_cpy_gpu=d["t_kv_cpy_gpu"], t_ram_vram=d["t_ram_vram"],
                           t_vram_ram=d["t_vram_ram"], t_comm=d["t_comm"]) for m, d in enumerate(devices)]
        return mo, ds

    halda.halda(*objects(*random_instance(1, n_devices=4, L=80)))  # the solver's first call loads it
    rows, plain_all = [], []
    for M in (4, 8, 16, 32):
        plain, refined = [], []
        for seed in range(5):
            mo, ds = objects(*random_instance(1000 + seed, n_devices=M, L=80))
            t0 = time.perf_counter()
            halda.halda(mo, ds, refine=False)
            t1 = time.perf_counter()
            halda.halda(mo, ds, refine=True)
            t2 = time.perf_counter()
            plain.append((t1 - t0) * 1e3)
            refined.append((t2 - t1) * 1e3)
        plain_all += plain
        rows.append({"devices": M, "algorithm_1_ms": round(statistics.median(plain), 2), "with_refinement_ms": round(statistics.median(refined), 1)})
    value = statistics.median(plain_all)
    print(json.dumps({
        "metric": "Halda scheduling latency (Algorithm 1), median over rings of 4, 8, 16 and 32 devices, 80 layers", "value": round(value, 2),
        "unit": "ms", "n_gpus": 0, "steps": 20, "warmup": 1, "higher_is_better": False, "vs_baseline": round(value / 11.0, 3),
        "baseline": "10-12 ms on 4-32 devices (Sec. 3.3); vs_baseline = value / 11 ms", "dtype": "f64", "data": "synthetic",
        "config": {"workload": "seeded rings of mixed devices (workloads/lda.py), 80-layer model, HiGHS through scipy.optimize.milp"},
        "cpu_model": cpu_model(), "by_ring_size": rows}))


def bench_launch_cost(args):
    """Time of a one-token mat-vec launch against its bytes: launches of 8192 columns and a growing number of rows,
    every launch on weights that the launches before it did not touch (nothing comes from the last-level cache),
    enqueued back to back as in a window.  The least-squares line t = t0 + bytes / rate separates what a launch costs
    whatever its size (hand-over from the launch before, prologue, tail) from the rate of its streaming phase."""
    import numpy as np
    import torch
    import paper_2504_08791_amd as prima

    dev = torch.device("cuda:0")
    cols = 8192
    stream = torch.cuda.current_stream()
    x = torch.randn((1, cols), device=dev)
    points = []
    for rows in (2048, 4096, 8192, 10240, 16384, 32768, 57344, 114688):
        nbytes = rows * (cols // 256) * 144
        copies = max(3, int(700_000_000 // nbytes) + 1)
        Ws = [torch.randint(0, 60, (rows, cols // 256, 144), dtype=torch.uint8, device=dev) for _ in range(copies)]
        y = torch.empty((1, rows), device=dev)
        ws = torch.empty(max(256, prima.gemv_workspace_bytes(rows, cols, 1)), dtype=torch.uint8, device=dev)
        for i in range(copies):
            prima.q4k_gemv(Ws[i], x, y=y, workspace=ws)
        torch.cuda.synchronize()
        n = max(args.steps, 2 * copies)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for i in range(n):
            prima.q4k_gemv(Ws[i % copies], x, y=y, workspace=ws)
        e1.record(stream)
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / n
        points.append((nbytes, us))
        del Ws
    b = np.array([p[0] for p in points], float)
    t = np.array([p[1] for p in points], float)
    slope, t0 = np.polyfit(b, t, 1)
    print(json.dumps({
        "metric": "fixed cost of a one-token Q4_K mat-vec launch (us) and the rate of its streaming phase",
        "value": round(float(t0), 2), "unit": "us", "n_gpus": 1, "steps": args.steps, "warmup": 0, "higher_is_better": False,
        "dtype": "i8 x i8 -> i32", "data": "synthetic",
        "config": {"workload": "Q4_K mat-vec, 8192 columns, 2048 to 114688 rows, one token, cold weights, launches back to back"},
        "stream_rate_gbps": round(1e-3 / float(slope), 1),
        "points": [{"rows": int(nb // ((cols // 256) * 144)), "MB": round(nb / 1e6, 1), "us": round(u, 2),
                    "line_us": round(float(t0 + slope * nb), 2)} for nb, u in points]}))


def bench_device_profile(args, cfg):
    """The GPU-side inputs of the paper's latency model (App. A.3) measured on this device with the library's own
    kernels, the model's estimate for one step of the config's window (all layers on the GPU, one window), and the
    measured step."""
    import torch
    import paper_2504_08791_amd as prima
    from paper_2504_08791_amd import profiler
    from workloads import synth

    d = cfg.dims
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    dp = profiler.device_profile(d)
    mp = profiler.model_profile(d)
    est = profiler.estimate_latency(mp, dp, cfg.n_layers, cfg.n_past + cfg.T)
    cap = cfg.n_past + cfg.T
    dev_layers = [{k: torch.from_numpy(v).to(dev) for k, v in synth.layer_tensors(cfg, l, kv_cap=cap).items()} for l in range(cfg.n_layers)]
    win = prima.Window(d, dev_layers, cap, T_max=cfg.T)
    x = torch.from_numpy(synth.window_input(cfg)).to(dev)
    y = torch.empty_like(x)
    stream = torch.cuda.current_stream()
    for _ in range(args.warmup):
        win.decode(x, cfg.n_past, x_out=y)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(args.steps):
        win.decode(x, cfg.n_past, x_out=y)
    e1.record(stream)
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / args.steps
    out = {
        "metric": "device-profiler quantities of the latency model; estimated vs measured window step", "value": round(ms, 4),
        "unit": "ms per step (measured)", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 4),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: {cfg.n_layers}-layer window, T={cfg.T}, n_kv={cfg.n_past}, Q4_K weights"},
        "device_profile": {
            "s_gpu_tflops": {q: round(v / 1e12, 3) for q, v in dp["s_gpu"].items()}, "matvec_shape": dp["matvec_shape"],
            "T_gpu_gbps": round(dp["T_gpu"] / 1e9, 1), "T_gpu_volume_bytes": dp["T_gpu_volume_bytes"],
            "t_kv_cpy_us": round(dp["t_kv_cpy"] * 1e6, 2), "t_ram_vram_us": round(dp["t_ram_vram"] * 1e6, 2),
            "t_vram_ram_us": round(dp["t_vram_ram"] * 1e6, 2)},
        "model_profile": {"flops_per_layer": mp["flops"], "b": mp["b"], "kv_bytes_per_token": mp["kv_bytes_per_token"]},
        "estimate_ms": {k: round(v * 1e3, 4) for k, v in est.items()},
        "estimate_over_measured": round(est["T"] * 1e3 / ms, 3),
        "max_of_terms_over_measured": round(max(est["T_comp"], est["T_mem"]) * 1e3 / ms, 3),
    }
    print(json.dumps(out), flush=True)


def bench_format(args):
    """Mat-vec of one of the other weight formats, one token: the output layer of config 4 (128256 x 8192, the tensor a
    "Q4K" model most often keeps in another format) with the final RMSNorm in front, and the down projection's shape
    (8192 x 28672).  Each launch reads a copy that the previous launches did not touch (the smaller matrix would
    otherwise sit in the 256 MB last-level cache)."""
    import numpy as np
    import torch
    import paper_2504_08791_amd as prima
    from workloads import synth
    from workloads.configs import CONFIGS

    fmt = args.format
    cfg = CONFIGS["c4k1"]
    d = cfg.dims
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    stream = torch.cuda.current_stream()
    res = {}
    g_host = synth.gain_f32(cfg.config_id, 0, "g_final", d.e)
    g = torch.from_numpy(g_host).to(dev)
    for name, rows, cols, with_norm in (("output_layer", cfg.vocab, d.e, True), ("down_projection", d.e, d.ffn, False)):
        nbytes = prima.fmt_tensor_bytes(fmt, rows, cols)
        W_host = synth.fmt_tensor(cfg.config_id, 0, "w_lm" if with_norm else "wdown", fmt, rows, cols)
        copies = [torch.from_numpy(W_host).to(dev)]
        while len(copies) * nbytes < 1_200_000_000:
            copies.append(copies[0].clone())
        x_host = synth.normal_f32(cfg.config_id, 0, "x_in", (1, cols))
        x = torch.from_numpy(x_host).to(dev)
        y = torch.empty((1, rows), dtype=torch.float32, device=dev)

        def launch(i):
            if with_norm:
                prima.lm_head_fmt(d, fmt, g, copies[i % len(copies)], rows, x, logits=y)
            else:
                prima.fmt_gemv(fmt, copies[i % len(copies)], rows, cols, x, y=y)
        for i in range(args.warmup):
            launch(i)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for i in range(args.steps):
            launch(i)
        e1.record(stream)
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / args.steps
        res[name] = {"rows": rows, "cols": cols, "bytes_per_launch": nbytes, "avg_launch_us": round(us, 2),
                     "gbps": round(nbytes / us / 1e3, 1), "frac_of_8000": round(nbytes / us / 1e3 / 8000.0, 4)}
        if not args.no_cpu_baseline:
            import oracle
            launch(0)
            got = y.cpu().numpy().astype(np.float64)[0]
            sample = np.unique(np.concatenate([np.arange(0, 2048), np.arange(rows - 2048, rows)]))
            # the sampled rows as a tensor of their own: plane by plane (the planes of a tensor are row-major)
            n, nb = rows * cols // 256, cols // 256
            per_block = {"q5_k": [16, 128, 32], "q6_k": [128, 64, 16, 2], "q8_0": [256, 16], "f16": [512], "f32": [1024]}[fmt]
            parts, off = [], 0
            for pb in per_block:
                plane = W_host[off:off + n * pb].reshape(rows, nb * pb)
                parts.append(plane[sample].reshape(-1))
                off += n * pb
            Ws = np.concatenate(parts)
            xin = x_host.astype(np.float64)
            t0 = time.perf_counter()
            if with_norm:
                ref = oracle.lm_head_fmt(d, fmt, g_host, Ws, len(sample), xin)[0]
            else:
                ref = oracle.fmt_gemv(fmt, Ws, len(sample), cols, xin)[0]
            cpu_seconds = time.perf_counter() - t0
            rms = np.sqrt((ref ** 2).mean())
            res[name]["max_rel_err_vs_oracle_sampled_rows"] = float((np.abs(got[sample] - ref) / np.maximum(np.abs(ref), rms)).max())
            res[name]["cpu_oracle_rows_per_s"] = round(len(sample) / cpu_seconds, 1)
            res[name]["cpu_cores"] = oracle.num_threads()
        del copies
    o = res["output_layer"]
    out = {
        "metric": f"weight streaming of the {fmt} mat-vec (one token), GB/s vs MI355X peak", "value": o["gbps"], "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(o["avg_launch_us"] / 1e3, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"output layer of config 4 ({cfg.vocab} x {d.e}) in {fmt}, final RMSNorm in front, T=1; "
                               f"also the down projection's shape ({d.e} x {d.ffn})"},
        "roofline": {"bound": "hbm", "kernel": "fmt_gemv_kernel (output layer launch)", "achieved": o["gbps"], "peak": 8000.0,
                     "unit": "GB/s", "frac": o["frac_of_8000"], "bytes_per_launch": o["bytes_per_launch"],
                     "avg_launch_us": o["avg_launch_us"], "traffic": None},
        "shapes": res,
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
