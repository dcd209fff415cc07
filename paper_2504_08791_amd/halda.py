"""Halda: layer windows w_m and GPU layers n_m for a ring of heterogeneous devices (Sec. 3.2, Sec. 3.3,
Algorithm 1; latency model and its vectorised form: App. A.3).

Host-side scheduling, no GPU work: the consumer of the model profiler's f^q, b, b_i, b_o and of the device
profiler's s^{gpu,q}, T^{gpu}, t^{kv_cpy}, t^{ram-vram}, t^{vram-ram} (profiler.py measures the GPU-side ones on
the current device; device_from_profile() turns them into a Device).

The layer-to-device assignment problem is an integer linear-fractional program whose coefficients depend on
which devices overflow their memory (sets M1..M4).  Halda (i) fixes the number of rounds k = L / W for every
divisor of L, which leaves an integer linear program per k (solved with HiGHS through scipy.optimize.milp),
and (ii) iterates: sets from the latest (w, n, k), programs for every k, best (w, n), sets again, until the
sets stop changing, with a calibration step that forces the slowest-disk overflowing device to stop
overflowing while some GPU still has free memory.

Readings of the paper taken here (each also noted where it applies):
  * the memory inequalities are non-strict, as in the problem's definition in Sec. 3.2 (App. A.3 prints them
    strict; with integer variables and real bounds the two differ only at exact ties);
  * d_m^swapout enters as its cap min(bytes_can_swap, swap_avail): in set M3 the overflow exceeds the cap, in
    set M4 the need must fit below d_avail + cap, so the cap is the constant of both inequalities;
  * "cuda" names any GPU backend with private memory (HIP on an MI355X as well), "metal" a GPU that shares
    the host's memory;
  * a calibration step whose programs are all infeasible (the other devices cannot hold the layers without
    overflowing) is undone and that device is not forced again;
  * device selection drops every device whose window is one layer and schedules again, keeping the result
    only if its predicted latency is lower.
"""
from dataclasses import dataclass, field, replace

import numpy as np

FORMATS = ("q4_k", "q5_k", "q6_k", "q8_0", "f16", "f32")


@dataclass
class Model:
    """What the model profiler reports (App. A.3): per layer the operations by weight format f^q and the weight
    bytes b; for the output layer f_out^q and b_o; the input table's bytes b_i and the vocabulary V; the KV bytes
    per cached token and layer 2 (h_k e_k + h_v e_v); the cached tokens n_kv; the compute buffers c^cpu, c^gpu."""
    L: int
    flops: dict
    flops_out: dict
    b: float
    b_i: float
    b_o: float
    V: int
    kv_bytes_per_token: float
    n_kv: int
    c_cpu: float = 0.0
    c_gpu: float = 0.0

    @property
    def b_prime(self):
        """b' = b + 2 (h_k e_k + h_v e_v) n_kv: a layer's weights and its KV cache (App. A.3)."""
        return self.b + self.kv_bytes_per_token * self.n_kv


@dataclass
class Device:
    """What the device profiler reports for device m (App. A.3).  os: "macos" | "linux" | "android";
    gpu: None | "cuda" | "metal"; uma: CPU and GPU share memory (no hidden-state copies)."""
    name: str
    os: str
    gpu: str = None
    uma: bool = False
    d_avail: float = 0.0            # RAM available, bytes
    d_gpu_avail: float = 0.0        # d^avail_{m,cuda} or d^avail_{m,metal}
    d_swapout: float = 0.0          # Android: min(bytes that can be swapped out, swap space left)
    s_disk: float = 1.0             # bytes/s (random reads on macOS, sequential on Linux)
    s_cpu: dict = field(default_factory=dict)   # q -> operations/s
    s_gpu: dict = field(default_factory=dict)
    T_cpu: float = 1.0              # bytes/s from RAM into registers
    T_gpu: float = 1.0
    t_kv_cpy_cpu: float = 0.0
    t_kv_cpy_gpu: float = 0.0
    t_ram_vram: float = 0.0
    t_vram_ram: float = 0.0
    t_comm: float = 0.0

    def __post_init__(self):
        if self.os not in ("macos", "linux", "android"):
            raise ValueError(f"unknown os {self.os!r}")
        if self.gpu not in (None, "cuda", "metal"):
            raise ValueError(f"unknown gpu backend {self.gpu!r}")
        if self.gpu == "metal" and self.os != "macos":
            raise ValueError("metal needs macos")


def device_from_profile(dp, name="gpu0", d_gpu_avail=288e9, host=None):
    """A Device for the GPU that profiler.device_profile() measured: Linux host, private GPU memory.
    host: optional dict of the CPU-side quantities (d_avail, s_disk, s_cpu, T_cpu, t_kv_cpy_cpu, t_comm)."""
    host = dict(host or {})
    return Device(name=name, os="linux", gpu="cuda", uma=False, d_gpu_avail=d_gpu_avail,
                  d_avail=host.get("d_avail", 0.0), s_disk=host.get("s_disk", 1.0),
                  s_cpu=host.get("s_cpu", {}), T_cpu=host.get("T_cpu", 1.0),
                  t_kv_cpy_cpu=host.get("t_kv_cpy_cpu", 0.0), t_comm=host.get("t_comm", 0.0),
                  s_gpu=dict(dp["s_gpu"]), T_gpu=dp["T_gpu"], t_kv_cpy_gpu=dp["t_kv_cpy"],
                  t_ram_vram=dp["t_ram_vram"], t_vram_ram=dp["t_vram_ram"])


def valid_rounds(L, M=1):
    """The k of Algorithm 1: divisors of L other than L itself, for which W = L / k leaves every one of the M
    devices at least one layer."""
    return [k for k in range(1, L) if L % k == 0 and L // k >= M] if L > 1 else []


def _per_layer_seconds(flops, s):
    total = 0.0
    for q, f in flops.items():
        if f:
            if not s.get(q):
                return float("inf")
            total += f / s[q]
    return total


def coefficients(model, dev):
    """alpha_m, beta_m, xi_m (App. A.3): seconds per CPU layer, the change when a layer moves to the GPU, and
    seconds per window (hidden-state copies unless memory is shared, plus one hop of the ring)."""
    bp = model.b_prime
    cpu = _per_layer_seconds(model.flops, dev.s_cpu) + dev.t_kv_cpy_cpu + bp / dev.T_cpu
    alpha = cpu
    if dev.gpu is None:
        beta = 0.0
    else:
        beta = _per_layer_seconds(model.flops, dev.s_gpu) + dev.t_kv_cpy_gpu + bp / dev.T_gpu - cpu
    xi = (dev.t_ram_vram + dev.t_vram_ram) * (0.0 if dev.uma else 1.0) + dev.t_comm
    return alpha, beta, xi


def _b_cio(model, m):
    """b^cio_m = (b_i / V + b_o) [m is the head] + c^cpu (App. A.3)."""
    return ((model.b_i / model.V + model.b_o) if m == 0 else 0.0) + model.c_cpu


def _ram_budget(model, dev, m):
    """Bytes left for layers in the memory that device m's CPU layers (or, with Metal, all its layers) use."""
    if dev.os == "macos":
        if dev.gpu == "metal":
            return dev.d_gpu_avail - _b_cio(model, m) - model.c_gpu
        return dev.d_avail - _b_cio(model, m)
    return dev.d_avail + (dev.d_swapout if dev.os == "android" else 0.0) - _b_cio(model, m)


def _gpu_budget(model, dev, m):
    if dev.gpu == "cuda":
        return dev.d_gpu_avail - model.c_gpu
    if dev.gpu == "metal":
        return dev.d_gpu_avail - model.c_gpu - (model.b_o if m == 0 else 0.0)
    return 0.0


def assign_sets(model, devices, w, n, k, forced=(), s_disk_threshold=0.0):
    """Cases 1-4 of App. A.3 for l_m = k w_m, l_m^gpu = k n_m: the set (1..4) of every device."""
    sets = []
    for m, dev in enumerate(devices):
        if m in forced or dev.s_disk <= s_disk_threshold:
            sets.append(4)
            continue
        layers = k * (w[m] - n[m]) if dev.os != "macos" else k * w[m]
        over = layers * model.b_prime > _ram_budget(model, dev, m)
        if not over:
            sets.append(4)
        elif dev.os == "macos":
            sets.append(2 if dev.gpu == "metal" else 1)
        else:
            sets.append(3)
    return sets


def objective_terms(model, devices, sets):
    """a, b, c and kappa of the vectorised objective (App. A.3) for a set assignment."""
    bp = model.b_prime
    a, b, c = [], [], []
    for dev, s in zip(devices, sets):
        alpha, beta, xi = coefficients(model, dev)
        if s == 1:
            a.append(alpha + bp / dev.s_disk); b.append(0.0)
        elif s == 2:
            a.append(alpha + model.b / dev.s_disk); b.append(beta)
        elif s == 3:
            a.append(alpha + bp / dev.s_disk); b.append(beta - bp / dev.s_disk)
        else:
            a.append(alpha); b.append(beta)
        c.append(xi)
    head = devices[0]
    kappa = (_per_layer_seconds(model.flops_out, head.s_cpu) + (model.b_i / model.V + model.b_o) / head.T_cpu
             + model.b_i / model.V / head.s_disk + (model.b_o / head.s_disk if sets[0] != 4 else 0.0))
    for dev, s in zip(devices, sets):
        if s in (1, 3):
            kappa += (model.c_cpu - dev.d_avail - (dev.d_swapout if dev.os == "android" else 0.0)) / dev.s_disk
    return np.array(a), np.array(b), np.array(c), kappa


def predicted_latency(model, devices, sets, w, n):
    """The objective of Sec. 3.2 for one (w, n): L (a.w + b.n + e.c) / (e.w) + kappa."""
    a, b, c, kappa = objective_terms(model, devices, sets)
    w, n = np.asarray(w, float), np.asarray(n, float)
    return model.L * (a @ w + b @ n + c.sum()) / w.sum() + kappa


def solve_fixed_k(model, devices, sets, k):
    """The integer linear program of Sec. 3.3 for one k (W = L / k).  Returns (T, w, n) or None if infeasible."""
    from scipy.optimize import Bounds, LinearConstraint, milp

    M, L = len(devices), model.L
    W = L // k
    a, b, c, kappa = objective_terms(model, devices, sets)
    if not (np.all(np.isfinite(a)) and np.all(np.isfinite(a + b))):
        # a device that cannot run some format on its CPU must hold every layer on its GPU; keep the program finite
        a = np.where(np.isfinite(a), a, 1e30)
        b = np.where(np.isfinite(b), b, -1e30 + 1.0)
    scale = W / (L * model.b_prime)
    rows, lo, hi = [], [], []

    def add(cw, cn, m, lower, upper):
        r = np.zeros(2 * M)
        r[m], r[M + m] = cw, cn
        rows.append(r); lo.append(lower); hi.append(upper)

    r = np.zeros(2 * M)
    r[:M] = 1.0
    rows.append(r); lo.append(W); hi.append(W)                        # every window filled: e.w = W
    for m, (dev, s) in enumerate(zip(devices, sets)):
        add(-1.0, 1.0, m, -np.inf, 0.0)                               # n_m <= w_m
        z = scale * _ram_budget(model, dev, m)
        if s in (1, 2):
            add(1.0, 0.0, m, z, np.inf)                               # overflowing: all layers count
        elif s == 3:
            add(1.0, -1.0, m, z, np.inf)                              # overflowing: CPU layers count
        elif dev.os == "macos":
            add(1.0, 0.0, m, -np.inf, z)
        else:
            add(1.0, -1.0, m, -np.inf, z)
    ub_n = [min(L, max(0.0, np.floor(scale * _gpu_budget(model, dev, m) + 1e-9))) if dev.gpu else 0.0
            for m, dev in enumerate(devices)]
    bounds = Bounds(np.concatenate([np.ones(M), np.zeros(M)]), np.concatenate([np.full(M, float(L)), np.array(ub_n)]))
    res = milp(c=np.concatenate([k * a, k * b]), constraints=LinearConstraint(np.array(rows), np.array(lo), np.array(hi)),
               integrality=np.ones(2 * M), bounds=bounds)
    if not res.success:
        return None
    x = np.rint(res.x).astype(int)
    w, n = x[:M], x[M:]
    return float(k * (a @ w + b @ n + c.sum()) + kappa), w.tolist(), n.tolist()


def initial_windows(model, devices):
    """w proportional to each device's memory budget, summing to L (k = 1), every device at least one layer."""
    mem = np.array([(dev.d_gpu_avail if (dev.os == "macos" and dev.gpu == "metal") else
                     dev.d_avail + (dev.d_swapout if dev.os == "android" else 0.0)) for dev in devices], float)
    mem = np.maximum(mem, 1.0)
    L, M = model.L, len(devices)
    if M > L:
        raise ValueError("more devices than layers")
    w = np.maximum(1, np.floor(L * mem / mem.sum()).astype(int))
    while w.sum() > L:
        w[int(np.argmax(w))] -= 1
    order = np.argsort(-mem)
    i = 0
    while w.sum() < L:
        w[order[i % M]] += 1
        i += 1
    return w.tolist()


@dataclass
class Schedule:
    w: list
    n: list
    k: int
    T: float
    sets: list
    forced: list
    iterations: int
    devices: list = None          # indices into the devices handed in (device selection drops some)


def _overflow_set(dev):
    return (2 if dev.gpu == "metal" else 1) if dev.os == "macos" else 3


def _best_over_rounds(model, devices, sets, rounds):
    found = None
    for kk in rounds:
        sol = solve_fixed_k(model, devices, sets, kk)
        if sol is not None and (found is None or sol[0] < found[0]):
            found = (sol[0], sol[1], sol[2], kk, list(sets))
    return found


def halda(model, devices, s_disk_threshold=0.0, max_iterations=None, refine=True):
    """Algorithm 1.  devices[0] is the head (it holds the input table and the output layer).

    refine: after Algorithm 1 has converged, flip one device (or, up to 8 devices, a pair) between "overflows"
    and "does not overflow" and keep a flip whose programs give a lower latency, until none does.  This is not in the paper:
    Algorithm 1 only ever moves a device out of the overflowing sets (its calibration step), so a device that
    the memory-proportional start puts in set M4 can never be tried as overflowing, nor the reverse without a
    GPU having room.  refine=False gives the paper's algorithm alone.

    Every program's constraints make its own set assignment true of its solution, so each solution's objective
    is the latency model's prediction for it and solutions of different iterations compare; the schedule
    returned is the one with the lowest prediction among them (the last one, whenever calibration helps)."""
    M, L = len(devices), model.L
    rounds = valid_rounds(L, M)
    if not rounds:
        raise ValueError("no valid number of rounds: L needs a divisor k < L with L / k >= the number of devices")
    w, n = initial_windows(model, devices), [0] * M
    forced, barred = set(), set()
    sets_prev, best, held, last_forced, it = None, None, None, None, 0
    limit = max_iterations or 4 * M + 8
    while it < limit:
        it += 1
        k = L // sum(w)
        sets = assign_sets(model, devices, w, n, k, forced, s_disk_threshold)
        if sets == sets_prev:
            break
        found = _best_over_rounds(model, devices, sets, rounds)
        if found is None:
            if held is None:
                break
            # the calibration went too far (the rest of the ring cannot take the layers): undo it, bar that device
            # and go on from the solution held back, which may still call for another device to be forced
            forced.discard(last_forced)
            barred.add(last_forced)
            found, sets = held, held[4]
            held = last_forced = None
        elif best is None or found[0] < best[0]:
            best = found
        T, w_new, n_new, k_new, _ = found
        # calibration: some GPU has room for one more layer while a device (that one or another) overflows
        scale = (L // k_new) / (L * model.b_prime)
        free_vram = [m for m, dev in enumerate(devices) if dev.gpu and n_new[m] + 1 <= scale * _gpu_budget(model, dev, m)]
        overflowing = [m for m in range(M) if sets[m] != 4]
        candidates = [m for m in overflowing if m not in barred]
        if candidates and free_vram:
            last_forced = min(candidates, key=lambda m: devices[m].s_disk)
            forced.add(last_forced)
            held = found
            sets_prev = sets
            continue
        held = last_forced = None
        sets_prev = sets
        w, n = w_new, n_new
    if refine:
        base = best[4] if best is not None else assign_sets(model, devices, w, n, L // sum(w), forced, s_disk_threshold)

        def flipped(sets, ms):
            trial = list(sets)
            for m in ms:
                if sets[m] == 4 and devices[m].s_disk <= s_disk_threshold:
                    return None                                # a slow disk never overflows (Case 4)
                trial[m] = _overflow_set(devices[m]) if sets[m] == 4 else 4
            return trial

        moves = [(m,) for m in range(M)]
        if M <= 8:                                             # exchanges: one device starts to overflow, another stops
            moves += [(i, j) for i in range(M) for j in range(i + 1, M)]
        improved = True
        while improved:
            improved = False
            for ms in moves:
                trial = flipped(base, ms)
                if trial is None:
                    continue
                found = _best_over_rounds(model, devices, trial, rounds)
                if found is not None and (best is None or found[0] < best[0] * (1 - 1e-12)):
                    best, base, improved = found, trial, True
                    break
    if best is None:
        raise RuntimeError("no feasible assignment: the devices cannot hold the model under the set assignments tried")
    T, w, n, k, sets = best
    return Schedule(w=w, n=n, k=k, T=T, sets=sets, forced=sorted(forced), iterations=it, devices=list(range(M)))


def select_devices(model, devices, s_disk_threshold=0.0, keep=()):
    """Device selection (Sec. 3.3): devices that Halda leaves with a one-layer window are dropped and the rest
    scheduled again.  The head (index 0) and the indices in `keep` (relays the ring cannot lose) always stay."""
    alive = list(range(len(devices)))
    sched = halda(model, [devices[i] for i in alive], s_disk_threshold)
    while len(alive) > 1:
        weak = [j for j, wj in enumerate(sched.w) if wj <= 1 and alive[j] != 0 and alive[j] not in keep]
        if not weak:
            break
        trial_alive = [a for j, a in enumerate(alive) if j not in weak]
        try:
            trial = halda(model, [devices[i] for i in trial_alive], s_disk_threshold)
        except (ValueError, RuntimeError):
            break
        if trial.T >= sched.T:
            break
        alive, sched = trial_alive, trial
    return replace(sched, devices=alive)
