"""Host logic of the model profiler and the latency estimate (App. A.3, computation and memory-access latency):
counts against what the tensors actually hold, the estimate against a case worked by hand."""
import numpy as np
import pytest

import oracle
from paper_2504_08791_amd import profiler
from workloads.configs import CONFIGS


def test_layer_bytes_and_operations_of_the_q4k_configs():
    for name in ("c0", "c1", "c3"):
        d = CONFIGS[name].dims
        mp = profiler.model_profile(d)
        assert mp["b"] == d.q4k_bytes_per_layer()                      # b of App. A.3, counted independently in workloads/
        weights = d.q4k_bytes_per_layer() * 256 // 144
        assert mp["flops"]["q4_k"] == 2 * weights and sum(mp["flops"].values()) == 2 * weights
        assert mp["kv_bytes_per_token"] * 100 == d.kv_bytes_per_layer(100)   # 2 (h_k e_k + h_v e_v) n_kv


def test_bytes_of_a_layer_with_several_formats_are_those_of_its_tensors():
    d = CONFIGS["c3"].dims
    formats = {"wv": "q6_k", "wdown": "q6_k", "wo": "q8_0", "wk": "f16"}
    mp = profiler.model_profile(d, formats, vocab=128256, out_format="q6_k")
    shapes = {"wq": (d.qd, d.e), "wk": (d.kvd, d.e), "wv": (d.kvd, d.e), "wo": (d.e, d.qd),
              "wgate": (d.ffn, d.e), "wup": (d.ffn, d.e), "wdown": (d.e, d.ffn)}
    assert mp["b"] == sum(oracle.fmt_tensor_bytes(formats.get(n, "q4_k"), r, c) for n, (r, c) in shapes.items())
    assert mp["b_o"] == oracle.fmt_tensor_bytes("q6_k", 128256, d.e)
    assert mp["flops"]["q6_k"] == 2 * (d.kvd * d.e + d.e * d.ffn) and mp["flops"]["f16"] == 2 * d.kvd * d.e
    assert mp["flops_out"] == {"q4_k": 0, "q5_k": 0, "q6_k": 2 * 128256 * d.e, "q8_0": 0, "f16": 0, "f32": 0}


def test_latency_estimate_worked_by_hand():
    # a made-up device and model with round numbers:
    #   per layer 4e9 operations in Q4_K and 1e9 in Q6_K, b = 3e8 bytes, 1000 KV bytes per cached token
    #   s(q4_k) = 2e12, s(q6_k) = 1e12 operations/s; T = 5e12 bytes/s; kv copy 2 us; copies in 10 us, out 12 us
    mp = {"flops": {"q4_k": 4e9, "q6_k": 1e9, "f32": 0}, "flops_out": {"q6_k": 2e9}, "b": 3e8, "b_o": 1e9,
          "kv_bytes_per_token": 1000}
    dp = {"s_gpu": {"q4_k": 2e12, "q6_k": 1e12, "f32": 1.0}, "T_gpu": 5e12, "t_kv_cpy": 2e-6, "t_ram_vram": 10e-6, "t_vram_ram": 12e-6}
    est = profiler.estimate_latency(mp, dp, n_layers=10, n_kv=2000, windows=2)
    # computation: 10 layers x (4e9/2e12 + 1e9/1e12) = 10 x 3 ms = 30 ms
    assert est["T_comp"] == pytest.approx(30e-3, rel=1e-12)
    # memory access: 10 x 2 us + 2 x 22 us + 10 x (3e8 + 2e6) / 5e12 = 20 us + 44 us + 604 us
    assert est["T_kv_cpy"] == pytest.approx(20e-6) and est["T_dev_cpy"] == pytest.approx(44e-6)
    assert est["T_dev_load"] == pytest.approx(604e-6, rel=1e-12)
    assert est["T"] == pytest.approx(30e-3 + 668e-6, rel=1e-12)
    # with the output layer on the GPU: + 2e9/1e12 = 2 ms of computation and 1e9/5e12 = 200 us of loading
    est2 = profiler.estimate_latency(mp, dp, n_layers=10, n_kv=2000, windows=2, output_on_gpu=True)
    assert est2["T"] - est["T"] == pytest.approx(2.2e-3, rel=1e-9)
