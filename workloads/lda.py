"""Seeded layer-to-device assignment instances (plain dicts: the keys oracle/lda.py documents), for the scheduler's tests
and its timing in bench.py.  Holds none of the method's arithmetic.

The sizes are those of a home cluster scaled down so that an exhaustive search finishes at once: a model of a
few layers, two to four devices of mixed operating systems, some with a GPU, memories from a fraction of the
model to several times it, disks from slow to fast (Table 2 and App. A.6 describe the real spread)."""
import numpy as np

FORMATS = ("q4_k", "q5_k", "q6_k", "q8_0", "f16", "f32")


def hand_model():
    return {"L": 4, "flops": {"q4_k": 100.0}, "flops_out": {"q4_k": 50.0}, "b": 1000.0, "b_i": 800.0, "b_o": 200.0, "V": 8,
            "kv": 10.0, "n_kv": 5, "c_cpu": 300.0, "c_gpu": 100.0}


def random_instance(seed, n_devices=None, L=None):
    rng = np.random.default_rng(seed)
    M = int(n_devices or rng.integers(2, 4))
    L = int(L or rng.choice([6, 8, 12]))
    b = 1.0e9
    model = {"L": L, "flops": {"q4_k": 2.0e9, "q6_k": 2.0e8}, "flops_out": {"q6_k": 5.0e8}, "b": b, "b_i": 4.0e8, "b_o": 4.0e8,
             "V": 32000, "kv": 4096.0, "n_kv": int(rng.integers(0, 2048)), "c_cpu": 1.0e8, "c_gpu": 1.5e8}
    devices = []
    for m in range(M):
        kind = rng.choice(["linux_cpu", "linux_cuda", "mac_metal", "mac_cpu", "android"], p=[0.2, 0.35, 0.2, 0.1, 0.15])
        cpu = float(rng.uniform(2e10, 3e11))
        dev = {"os": "linux", "gpu": None, "uma": False, "d_avail": float(rng.uniform(0.8, 1.2 * L) * b), "d_gpu_avail": 0.0,
               "swap_cap": 0.0, "s_disk": float(rng.choice([0.3e9, 1.0e9, 3.0e9])), "s_cpu": {q: cpu * f for q, f in zip(FORMATS, (1.0, 0.9, 0.8, 1.1, 0.7, 0.5))},
               "s_gpu": {}, "T_cpu": float(rng.uniform(1e10, 6e10)), "T_gpu": 1.0, "t_kv_cpy_cpu": float(rng.uniform(1e-6, 1e-5)),
               "t_kv_cpy_gpu": 0.0, "t_ram_vram": 0.0, "t_vram_ram": 0.0, "t_comm": float(rng.uniform(2e-3, 8e-3))}
        if kind in ("linux_cuda", "mac_metal"):
            gpu = float(rng.uniform(5e11, 5e12))
            dev["s_gpu"] = {q: gpu * f for q, f in zip(FORMATS, (1.0, 0.9, 0.8, 1.1, 1.5, 1.0))}
            dev["T_gpu"] = float(rng.uniform(1e11, 8e11))
            dev["t_kv_cpy_gpu"] = float(rng.uniform(5e-6, 2e-5))
        if kind == "linux_cuda":
            dev.update(gpu="cuda", d_gpu_avail=float(rng.uniform(1.5, 0.9 * L) * b), t_ram_vram=float(rng.uniform(1e-5, 1e-4)),
                       t_vram_ram=float(rng.uniform(1e-5, 1e-4)))
        elif kind == "mac_metal":
            dev.update(os="macos", gpu="metal", uma=True, d_gpu_avail=float(rng.uniform(1.5, 0.9 * L) * b))
        elif kind == "mac_cpu":
            dev.update(os="macos")
        elif kind == "android":
            dev.update(os="android", swap_cap=float(rng.uniform(0.0, 2.0) * b))
        devices.append(dev)
    return model, devices
