"""Pins of oracle/lda.py (the token latency of an assignment, written out from App. A.3) against values worked
by hand from the paper's formulas, the paper's own example of the ring, and invariants."""
import numpy as np
import pytest

from oracle import lda
import lda_cases


def _dev(**kw):
    d = {"os": "linux", "gpu": None, "uma": False, "d_avail": 0.0, "d_gpu_avail": 0.0, "swap_cap": 0.0, "s_disk": 50.0,
         "s_cpu": {"q4_k": 10.0}, "s_gpu": {}, "T_cpu": 50.0, "T_gpu": 1.0, "t_kv_cpy_cpu": 2.0, "t_kv_cpy_gpu": 0.0,
         "t_ram_vram": 0.0, "t_vram_ram": 0.0, "t_comm": 0.0}
    d.update(kw)
    return d


def test_ring_example_of_the_paper():
    """Sec. 3.1, the figure of the pipelined ring: 6 devices, 36 layers, window 2: 18 segments, every device
    takes 3 rounds and so 6 layers."""
    l, lg, nw = lda.layer_counts(36, [2] * 6, [0] * 6)
    assert l == [6] * 6 and nw == [3] * 6 and lg == [0] * 6


def test_layer_counts_with_a_remainder_by_hand():
    # L = 7, w = (3, 2): one full round (5 layers), R = 2 goes to the first device's window
    assert lda.layer_counts(7, [3, 2], [1, 2]) == ([5, 2], [2, 2], [2, 1])
    # L = 9, w = (3, 2): R = 4: three to the first device, one to the second; both get a second window
    assert lda.layer_counts(9, [3, 2], [0, 1]) == ([6, 3], [0, 2], [2, 2])


@pytest.mark.parametrize("seed", range(20))
def test_every_layer_is_assigned_once(seed):
    rng = np.random.default_rng(seed)
    M = int(rng.integers(1, 6))
    w = [int(v) for v in rng.integers(1, 7, M)]
    n = [int(rng.integers(0, wm + 1)) for wm in w]
    L = int(rng.integers(sum(w), 5 * sum(w)))
    l, lg, nw = lda.layer_counts(L, w, n)
    assert sum(l) == L
    assert all(0 <= g <= t for g, t in zip(lg, l))
    assert all(-(-t // wm) == k for t, wm, k in zip(l, w, nw))        # windows = ceil(layers / window size)


def test_two_linux_devices_by_hand():
    """Worked by hand from the four latency terms of App. A.3 (numbers chosen so every term is round).
    L = 4, w = (1, 1), n = (0, 1): two rounds, two layers each; device 1 runs both of its layers on the GPU.
      device 0 (head, CPU only): compute 2*100/10 + 50/10 = 25; memory 2*2 + 2*1050/50 + 300/50 = 52;
        disk max(2*1000 + 300 + 2*50 + 300 - 2000, 100)/50 = 14; network 2*7 = 14            -> 105
      device 1 (GPU): compute 2*100/100 = 2; memory 2*0.5 + 2*(3+4) + 2*1050/525 = 19;
        disk max(300 - 500, 100)/100 = 1; network 2*6 = 12                                    -> 34"""
    model = lda_cases.hand_model()
    d0 = _dev(d_avail=2000.0, t_comm=7.0)
    d1 = _dev(gpu="cuda", d_avail=500.0, d_gpu_avail=5000.0, s_disk=100.0, s_cpu={"q4_k": 20.0}, s_gpu={"q4_k": 100.0}, T_cpu=10.0,
              T_gpu=525.0, t_kv_cpy_cpu=1.0, t_kv_cpy_gpu=0.5, t_ram_vram=3.0, t_vram_ram=4.0, t_comm=6.0)
    assert lda.token_latency(model, [d0, d1], [1, 1], [0, 1]) == pytest.approx(139.0, abs=1e-9)
    l, lg, nw = lda.layer_counts(4, [1, 1], [0, 1])
    assert lda.device_latency(model, d0, 0, l[0], lg[0], nw[0]) == pytest.approx(105.0, abs=1e-9)
    assert lda.device_latency(model, d1, 1, l[1], lg[1], nw[1]) == pytest.approx(34.0, abs=1e-9)


def test_macos_with_metal_by_hand():
    """One device, L = 2, w = 2, n = 1, memory shared (no hidden-state copies even though their times are set).
    compute 10 + 100/50 + 5 = 17; memory 2 + 1 + 1050/50 + 1050/525 + 300/50 = 32.
    Needing 2*1000 + 300 + 2*50 + 300 + 100 = 2800 > 2000 bytes, the whole 2*1000 + 300 are reloaded every token:
    2300/50 = 46 -> 95.  With 3000 bytes nothing but the table row is read: 100/50 = 2 -> 51."""
    model = dict(lda_cases.hand_model(), L=2)
    mac = _dev(os="macos", gpu="metal", uma=True, d_gpu_avail=2000.0, s_gpu={"q4_k": 50.0}, T_gpu=525.0, t_kv_cpy_gpu=1.0,
               t_ram_vram=9.0, t_vram_ram=9.0)
    assert lda.token_latency(model, [mac], [2], [1]) == pytest.approx(95.0, abs=1e-9)
    assert lda.token_latency(model, [dict(mac, d_gpu_avail=3000.0)], [2], [1]) == pytest.approx(51.0, abs=1e-9)


def test_android_swaps_before_it_reloads_by_hand():
    """One device, L = 2, w = 2, CPU only: compute 20 + 5 = 25; memory 4 + 42 + 6 = 52.  It needs
    2*1000 + 300 + 100 + 300 = 2700 bytes and has 1000: with 500 bytes of swap 1200 are reloaded (24 s) -> 101;
    with 5000 bytes of swap nothing is (2 s for the table row) -> 79.  macOS without Metal in the same spot
    reloads 1700 bytes (34 s) -> 111, and so does Linux."""
    model = dict(lda_cases.hand_model(), L=2)
    phone = _dev(os="android", d_avail=1000.0, swap_cap=500.0)
    assert lda.token_latency(model, [phone], [2], [0]) == pytest.approx(101.0, abs=1e-9)
    assert lda.token_latency(model, [dict(phone, swap_cap=5000.0)], [2], [0]) == pytest.approx(79.0, abs=1e-9)
    assert lda.token_latency(model, [dict(phone, os="macos")], [2], [0]) == pytest.approx(111.0, abs=1e-9)
    assert lda.token_latency(model, [dict(phone, os="linux")], [2], [0]) == pytest.approx(111.0, abs=1e-9)


def test_moving_a_layer_to_the_gpu_changes_the_latency_by_beta():
    """Without memory pressure the latency is linear in n_m with slope k * beta_m, beta_m the difference of a
    layer's GPU and CPU seconds (App. A.3): here 2 rounds * ((100/100 + 0.5 + 1050/525) - (100/20 + 1 + 1050/10))."""
    model = lda_cases.hand_model()
    d0 = _dev(d_avail=1e9)
    d1 = _dev(gpu="cuda", d_avail=1e9, d_gpu_avail=1e9, s_cpu={"q4_k": 20.0}, s_gpu={"q4_k": 100.0}, T_cpu=10.0, T_gpu=525.0,
              t_kv_cpy_cpu=1.0, t_kv_cpy_gpu=0.5)
    t0 = lda.token_latency(model, [d0, d1], [1, 1], [0, 0])
    t1 = lda.token_latency(model, [d0, d1], [1, 1], [0, 1])
    assert t1 - t0 == pytest.approx(2 * ((1.0 + 0.5 + 2.0) - (5.0 + 1.0 + 105.0)), abs=1e-9)


def test_compositions_count():
    from math import comb
    for total, parts in ((6, 3), (8, 2), (5, 5), (7, 1)):
        got = list(lda.compositions(total, parts))
        assert len(got) == comb(total - 1, parts - 1) == len(set(got))
        assert all(sum(c) == total and min(c) >= 1 for c in got)
