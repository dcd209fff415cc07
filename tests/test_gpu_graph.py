"""The window calls under HIP graph capture: they enqueue kernels on the stream they are given, allocate nothing,
never synchronise and clear their scratch with fill kernels (not memset nodes), so a step can be captured once and
replayed.  Each graph is replayed several times with eager work of the library and synchronisations in between, and
every replay must give the bits of the eager call."""
import copy

import numpy as np
import pytest
import torch

from workloads import synth
from workloads.configs import TINY

pytestmark = pytest.mark.gpu


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _windows(gpu_lib, cfg, cap, n):
    host = [synth.layer_tensors(cfg, l, kv_cap=cap) for l in range(cfg.n_layers)]
    return [gpu_lib.Window(cfg.dims, [{k: _dev(v) for k, v in t.items()} for t in copy.deepcopy(host)], cap, T_max=16) for _ in range(n)]


@pytest.mark.parametrize("T", [1, 4, 16])
def test_decode_step_replayed_from_a_graph(gpu_lib, T):
    cfg = TINY["t1"].with_(T=T, n_past=37)
    cap = 80
    eager, captured, other = _windows(gpu_lib, cfg, cap, 3)
    x = _dev(synth.window_input(cfg))
    want = eager.decode(x, cfg.n_past).clone()
    side = torch.cuda.Stream()
    y = torch.empty_like(x)
    with torch.cuda.stream(side):
        captured.decode(x, cfg.n_past, x_out=y)        # everything that is looked up once happens here, not under capture
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        captured.decode(x, cfg.n_past, x_out=y)
    x2 = _dev(synth.window_input(cfg.with_(config_id=cfg.config_id + 1)))
    for replay in range(4):
        y.fill_(float("nan"))
        other.decode(x2, 11 + replay)                  # the library's own eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, want), (T, replay)
        captured.check(T)


def test_prompt_call_replayed_from_a_graph(gpu_lib):
    cfg = TINY["t2"].with_(T=100, n_past=9)
    cap = 128
    eager, captured, other = _windows(gpu_lib, cfg, cap, 3)
    x = _dev(synth.window_input(cfg))
    gpu_lib.set_prefill_small_tokens(0)                # the matrix-product route
    try:
        want = eager.prefill(x, cfg.n_past).clone()
        side = torch.cuda.Stream()
        y = torch.empty_like(x)
        with torch.cuda.stream(side):
            captured.prefill(x, cfg.n_past, x_out=y)   # also allocates the binding's scratch for this size
        side.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            captured.prefill(x, cfg.n_past, x_out=y)
        x2 = _dev(synth.window_input(cfg.with_(config_id=cfg.config_id + 1)))
        for replay in range(3):
            y.fill_(float("nan"))
            other.prefill(x2, replay)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(y, want), replay
    finally:
        gpu_lib.set_prefill_small_tokens(gpu_lib.PREFILL_SMALL_TOKENS)
