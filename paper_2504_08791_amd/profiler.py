"""Model profiler and device profiler for one GPU: the quantities the paper's latency model takes as inputs
(App. A.3, "Layer-to-device assignment: from latency analysis to vectorized model").

model_profile(): counts, per layer and for the output layer, the floating-point operations by weight format
(f^q) and the bytes (b, b_o, b_i), and the KV bytes per cached token 2 (h_k e_k + h_v e_v).  Pure arithmetic on
the model's dimensions.

device_profile(): measures on the current GPU, through the library's own entry points, the per-format
throughput s^{gpu,q} (operations of a one-token mat-vec per second), the practical read throughput T^{gpu} (the
library's linear-read operator at a data volume like a tensor's), the KV copy time t^{kv_cpy,gpu}
(2 (h_k e_k + h_v e_v) bytes, device to device) and the hidden-state copies t^{ram-vram}, t^{vram-ram} (4e bytes).

estimate_latency(): the paper's T^comp + T^mem for a device that runs all its layers on the GPU
(l_m = l_m^gpu; the CPU, disk and network terms belong to other devices of the ring or to the host).
"""
import time

FORMAT_BITS = {"q4_k": 4.5, "q5_k": 5.5, "q6_k": 6.5625, "q8_0": 8.5, "f16": 16.0, "f32": 32.0}
MATRICES = ("wq", "wk", "wv", "wo", "wgate", "wup", "wdown")


def _shapes(dims):
    qd, kvd = dims.n_q_heads * dims.head_dim, dims.n_kv_heads * dims.head_dim
    return {"wq": (qd, dims.e), "wk": (kvd, dims.e), "wv": (kvd, dims.e), "wo": (dims.e, qd),
            "wgate": (dims.ffn, dims.e), "wup": (dims.ffn, dims.e), "wdown": (dims.e, dims.ffn)}


def model_profile(dims, formats=None, vocab=0, out_format="q4_k", in_format="q4_k"):
    """Per token: {"flops": {q: f^q}, "b": bytes of a layer's matrices, "flops_out": {q: f_out^q}, "b_o", "b_i",
    "kv_bytes_per_token": 2 (h_k e_k + h_v e_v)}.  formats: dict matrix name -> format (default Q4_K).
    A multiply-add counts as two operations; only the products with the weight matrices are counted (the cost of
    attention enters the latency model through the KV bytes)."""
    formats = formats or {}
    flops = {q: 0 for q in FORMAT_BITS}
    b = 0
    for name, (rows, cols) in _shapes(dims).items():
        q = formats.get(name, "q4_k")
        flops[q] += 2 * rows * cols
        b += int(rows * cols * FORMAT_BITS[q] / 8)
    flops_out = {q: 0 for q in FORMAT_BITS}
    flops_out[out_format] = 2 * vocab * dims.e
    return {"flops": flops, "b": b, "flops_out": flops_out,
            "b_o": int(vocab * dims.e * FORMAT_BITS[out_format] / 8), "b_i": int(vocab * dims.e * FORMAT_BITS[in_format] / 8),
            "kv_bytes_per_token": 2 * 2 * dims.n_kv_heads * dims.head_dim}


def estimate_latency(mp, dp, n_layers, n_kv, windows=1, output_on_gpu=False):
    """Seconds per token of a device with n_layers layers, all on the GPU, n_kv cached tokens, `windows` windows
    per token: the paper's computation and memory-access terms.  mp: model_profile(), dp: device_profile() (or
    any dict with "s_gpu" {q: ops/s}, "T_gpu" bytes/s, "t_kv_cpy", "t_ram_vram", "t_vram_ram" seconds).
    Returns a dict of the terms and their sum."""
    def comp(flops):
        return sum(f / dp["s_gpu"][q] for q, f in flops.items() if f)
    t_comp = n_layers * comp(mp["flops"]) + (comp(mp["flops_out"]) if output_on_gpu else 0.0)
    t_kv_cpy = n_layers * dp["t_kv_cpy"]
    t_dev_cpy = windows * (dp["t_ram_vram"] + dp["t_vram_ram"])
    t_dev_load = (n_layers * (mp["b"] + mp["kv_bytes_per_token"] * n_kv) + (mp["b_o"] if output_on_gpu else 0)) / dp["T_gpu"]
    return {"T_comp": t_comp, "T_kv_cpy": t_kv_cpy, "T_dev_cpy": t_dev_cpy, "T_dev_load": t_dev_load,
            "T_mem": t_kv_cpy + t_dev_cpy + t_dev_load, "T": t_comp + t_kv_cpy + t_dev_cpy + t_dev_load}


def device_profile(dims, formats=("q4_k", "q5_k", "q6_k", "q8_0", "f16", "f32"), reps=20):
    """Measures the GPU-side inputs of the latency model on the current device (see the module text).
    Mat-vec shape: the gate projection's (ffn x e), one token, every launch on a copy of the tensor that the
    launches before it did not touch (nothing comes from the last-level cache that a real step would stream)."""
    import torch
    from . import (fmt_gemv, fmt_tensor_bytes, gemv_workspace_bytes, q4k_gemv, stream_read_probe)

    dev = torch.device("cuda")
    rows, cols = dims.ffn, dims.e
    stream = torch.cuda.current_stream()

    def timed(fn, n):
        for i in range(3):
            fn(i)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for i in range(n):
            fn(i)
        e1.record(stream)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / n

    out = {"s_gpu": {}, "matvec_shape": [rows, cols]}
    x = torch.randn((1, cols), device=dev)
    y = torch.empty((1, rows), device=dev)
    for q in formats:
        nbytes = fmt_tensor_bytes(q, rows, cols)
        copies = max(2, int(600_000_000 // nbytes) + 1)
        # timing only: byte values that keep every scale finite (no special values slow a multiply-add, but infinities would)
        Ws = [torch.randint(0, 60, (nbytes,), dtype=torch.uint8, device=dev) for _ in range(copies)]
        if q == "q4_k":
            ws = torch.empty(max(256, gemv_workspace_bytes(rows, cols, 1)), dtype=torch.uint8, device=dev)
            W3 = [w.view(rows, cols // 256, 144) for w in Ws]
            sec = timed(lambda i: q4k_gemv(W3[i % copies], x, y=y, workspace=ws), reps)
        else:
            sec = timed(lambda i: fmt_gemv(q, Ws[i % copies], rows, cols, x, y=y), reps)
        out["s_gpu"][q] = 2.0 * rows * cols / sec
        del Ws
    # read throughput at a tensor-like volume (the gate and up matrices of a layer in Q4_K), cold
    vol = 2 * fmt_tensor_bytes("q4_k", rows, cols)
    bufs = [torch.empty(vol, dtype=torch.uint8, device=dev).random_(0, 255) for _ in range(max(2, int(600_000_000 // vol) + 1))]
    sink = torch.zeros(1, dtype=torch.int32, device=dev)
    # with non-temporal loads, the way the library requests weights that a launch reads once
    out["T_gpu"] = vol / timed(lambda i: stream_read_probe(bufs[i % len(bufs)], sink, nt=True), reps)
    out["T_gpu_plain_loads"] = vol / timed(lambda i: stream_read_probe(bufs[i % len(bufs)], sink), reps)
    out["T_gpu_volume_bytes"] = vol
    del bufs
    # KV copy: the new token's K and V rows of one layer, device to device
    kv = 2 * 2 * dims.n_kv_heads * dims.head_dim
    src, dst = torch.empty(kv, dtype=torch.uint8, device=dev), torch.empty(kv, dtype=torch.uint8, device=dev)
    out["t_kv_cpy"] = timed(lambda i: dst.copy_(src, non_blocking=True), 200)
    # hidden state in and out of the device: 4e bytes, pinned host memory, each copy waited for (as a window would)
    h_host = torch.empty(dims.e, dtype=torch.float32).pin_memory()
    h_dev = torch.empty(dims.e, dtype=torch.float32, device=dev)

    def wall(fn, n):
        fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            fn()
        return (time.perf_counter() - t0) / n

    def to_dev():
        h_dev.copy_(h_host, non_blocking=True)
        torch.cuda.synchronize()

    def to_host():
        h_host.copy_(h_dev, non_blocking=True)
        torch.cuda.synchronize()
    out["t_ram_vram"] = wall(to_dev, 200)
    out["t_vram_ram"] = wall(to_host, 200)
    return out
