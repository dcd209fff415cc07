"""Test infrastructure, not product code: the token latency of a layer-to-device assignment written out term by
term from the latency analysis (App. A.3), and its minimum by exhaustive search.

Only tests import this.  It shares nothing with the scheduler it checks: no set assignment, no linearised
coefficients, no integer program.  The disk term keeps its max(), the layer counts keep the remainder R, and
the search simply tries every (w, n).

Devices and the model are plain dicts (keys below), so that no class of the product is needed here.
  model:  L, flops {q: f}, flops_out {q: f}, b, b_i, b_o, V, kv (= 2 (h_k e_k + h_v e_v)), n_kv, c_cpu, c_gpu
  device: os ("macos" | "linux" | "android"), gpu (None | "cuda" | "metal"), uma, d_avail, d_gpu_avail,
          swap_cap (= min(bytes_can_swap, swap_avail)), s_disk, s_cpu {q: ops/s}, s_gpu {q: ops/s}, T_cpu, T_gpu,
          t_kv_cpy_cpu, t_kv_cpy_gpu, t_ram_vram, t_vram_ram, t_comm
Device 0 is the head (m = 1 in the paper).
"""
import itertools


def layer_counts(L, w, n):
    """l_m, l_m^gpu and the number of windows W_m of every device (App. A.3, computation latency and device
    copy time): floor(L / W) full rounds, then the remainder R = L mod W handed out in ring order."""
    W = sum(w)
    full, R = divmod(L, W)
    l, lg, nw = [], [], []
    before = 0                                       # sum over j < m of min(w_j, R)
    for wm, nm in zip(w, n):
        left = max(0, R - before)
        l.append(full * wm + min(wm, left))
        lg.append(full * nm + min(nm, left))
        nw.append(full + min(1, left))
        before += min(wm, R)
    return l, lg, nw


def _seconds(flops, s):
    return sum(f / s[q] for q, f in flops.items() if f)


def device_latency(model, dev, m, l, lg, nw):
    """T_m^comp + T_m^mem + T_m^disk + T_m^comm for one device (App. A.3), l layers of which lg on the GPU."""
    head = m == 0
    kvb = model["kv"] * model["n_kv"]                # KV bytes of one layer
    io = (model["b_i"] / model["V"] + model["b_o"]) if head else 0.0
    lookup = model["b_i"] / model["V"]
    cpu_layers = l - lg
    t_comp = cpu_layers * _seconds(model["flops"], dev["s_cpu"]) if cpu_layers else 0.0
    if lg:
        t_comp += lg * _seconds(model["flops"], dev["s_gpu"])
    if head:
        t_comp += _seconds(model["flops_out"], dev["s_cpu"])
    t_mem = cpu_layers * dev["t_kv_cpy_cpu"] + lg * dev["t_kv_cpy_gpu"]
    t_mem += nw * (dev["t_ram_vram"] + dev["t_vram_ram"]) * (0 if dev["uma"] else 1)
    t_mem += (cpu_layers / dev["T_cpu"] + (lg / dev["T_gpu"] if lg else 0.0)) * (model["b"] + kvb) + io / dev["T_cpu"]
    if dev["os"] == "macos" and dev["gpu"] != "metal":
        reload = l * model["b"] + io + kvb * l + model["c_cpu"] - dev["d_avail"]
        t_disk = max(reload, lookup) / dev["s_disk"]
    elif dev["os"] == "macos":
        need = l * model["b"] + io + kvb * l + model["c_cpu"] + model["c_gpu"]
        whole = (l * model["b"] + io) if need > dev["d_gpu_avail"] else 0.0
        t_disk = max(whole, lookup) / dev["s_disk"]
    else:
        need = cpu_layers * model["b"] + io + kvb * cpu_layers + model["c_cpu"]
        swapout = 0.0
        if dev["os"] == "android":
            swapout = min(max(0.0, need - dev["d_avail"]), dev["swap_cap"])
        t_disk = max(need - dev["d_avail"] - swapout, lookup) / dev["s_disk"]
    t_comm = nw * dev["t_comm"]
    return t_comp + t_mem + t_disk + t_comm


def token_latency(model, devices, w, n):
    """T = sum over devices of T_m (App. A.3; the sum, not the maximum, is what the method minimises)."""
    l, lg, nw = layer_counts(model["L"], w, n)
    return sum(device_latency(model, dev, m, l[m], lg[m], nw[m]) for m, dev in enumerate(devices))


def overflows(model, dev, m, l, lg):
    """Does device m need more memory than it has (the conditions of Cases 1-3, App. A.3)?"""
    kvb = model["kv"] * model["n_kv"]
    io = (model["b_i"] / model["V"] + model["b_o"]) if m == 0 else 0.0
    if dev["os"] == "macos" and dev["gpu"] == "metal":
        return l * (model["b"] + kvb) + io + model["c_cpu"] + model["c_gpu"] > dev["d_gpu_avail"]
    if dev["os"] == "macos":
        return l * (model["b"] + kvb) + io + model["c_cpu"] > dev["d_avail"]
    extra = dev["swap_cap"] if dev["os"] == "android" else 0.0
    return (l - lg) * (model["b"] + kvb) + io + model["c_cpu"] > dev["d_avail"] + extra


def gpu_fits(model, dev, m, lg):
    """VRAM (or Metal working-set) limit on the GPU layers (App. A.3, the last two constraints)."""
    if dev["gpu"] is None:
        return lg == 0
    room = dev["d_gpu_avail"] - model["c_gpu"] - (model["b_o"] if (dev["gpu"] == "metal" and m == 0) else 0.0)
    return lg * (model["b"] + model["kv"] * model["n_kv"]) <= room


def compositions(total, parts):
    """All ways to write total as an ordered sum of `parts` positive integers."""
    if parts == 1:
        yield (total,)
        return
    for first in range(1, total - parts + 2):
        for rest in compositions(total - first, parts - 1):
            yield (first,) + rest


def brute_force(model, devices, s_disk_threshold=0.0, no_overflow=()):
    """The best (T, w, n, k) over every w with sum(w) a divisor W of L (k = L / W < L rounds, every window
    filled: the method's own restriction, Sec. 3.2), every n <= w within the GPU memory, and no overflow on a
    device whose disk is at or below the threshold (Case 4) or that is listed in no_overflow."""
    L, M = model["L"], len(devices)
    best = None
    for k in range(1, L):
        if L % k or L // k < M:
            continue
        for w in compositions(L // k, M):
            ranges = [range(0, wm + 1) if dev["gpu"] else range(0, 1) for wm, dev in zip(w, devices)]
            for n in itertools.product(*ranges):
                l, lg, _ = layer_counts(L, w, n)
                ok = True
                for m, dev in enumerate(devices):
                    if not gpu_fits(model, dev, m, lg[m]):
                        ok = False
                        break
                    if (dev["s_disk"] <= s_disk_threshold or m in no_overflow) and overflows(model, dev, m, l[m], lg[m]):
                        ok = False
                        break
                if not ok:
                    continue
                T = token_latency(model, devices, w, n)
                if best is None or T < best[0]:
                    best = (T, list(w), list(n), k)
    return best
