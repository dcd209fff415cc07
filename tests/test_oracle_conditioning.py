"""Pins of the oracle-side conditioning bound (oracle.conditioning / layer_stepwise / window_conditioning), the only
excuse the window-level parity tests accept for a miss of the 2e-3 bar (tests/tolerance.py)."""
import numpy as np
import pytest

import oracle
from workloads import synth
from workloads.configs import TINY, ModelDims, WindowConfig


def _host(cfg, cap, formats=None):
    return [synth.layer_tensors(cfg, l, kv_cap=cap, formats=formats) for l in range(cfg.n_layers)]


@pytest.mark.parametrize("name", ["t0", "t1", "t2"])
def test_stepwise_layer_is_the_layer(name):
    """layer_stepwise composes the oracle's operators in the order of the definition; unperturbed it must return
    the bits of layer() and leave the same cache rows (a dropped residual, a swapped operand or a missed append
    would show here)."""
    cfg = TINY[name]
    cap = cfg.n_past + cfg.T
    a, b = _host(cfg, cap), _host(cfg, cap)
    x = synth.window_input(cfg).astype(np.float64)
    ya = oracle.window(cfg.dims, a, x, cfg.n_past)
    yb = oracle.window_stepwise(cfg.dims, b, x, cfg.n_past)
    assert np.array_equal(ya, yb)
    for ta, tb in zip(a, b):
        assert np.array_equal(ta["k_cache"], tb["k_cache"]) and np.array_equal(ta["v_cache"], tb["v_cache"])


def test_stepwise_layer_with_other_formats_is_the_layer():
    cfg = TINY["t1"]
    fm = {"wk": "q6_k", "wo": "q5_k", "wup": "f16", "wdown": "q8_0"}
    cap = cfg.n_past + cfg.T
    x = synth.window_input(cfg).astype(np.float64)
    ya = oracle.window(cfg.dims, _host(cfg, cap, fm), x, cfg.n_past, formats=[fm] * cfg.n_layers)
    yb = oracle.window_stepwise(cfg.dims, _host(cfg, cap, fm), x, cfg.n_past, formats=[fm] * cfg.n_layers)
    assert np.array_equal(ya, yb)


def test_every_stored_intermediate_is_offered_to_the_perturbation():
    cfg = TINY["t1"].with_(n_layers=1)
    d, T = cfg.dims, cfg.T
    seen = {}

    def spy(name, arr):
        seen[name] = arr.shape
        return arr
    oracle.window_stepwise(d, _host(cfg, cfg.n_past + T), synth.window_input(cfg).astype(np.float64), cfg.n_past, perturb=spy)
    assert seen == {"q": (T, d.qd), "k": (T, d.kvd), "v": (T, d.kvd), "q_rot": (T, d.qd), "k_rot": (T, d.kvd),
                    "o": (T, d.qd), "h": (T, d.e), "a": (T, d.ffn), "y": (T, d.e)}


def test_conditioning_of_a_linear_map_is_its_closed_form():
    """fn(x) = x A^T: the movement under x -> x (1 + eps s) is eps (x s) A^T exactly."""
    rng = np.random.default_rng(3)
    A = rng.standard_normal((7, 12))
    x = rng.standard_normal((2, 12))
    signs = [rng.integers(0, 2, size=x.shape) * 2.0 - 1.0 for _ in range(3)]
    eps = 2.0 ** -10
    got = oracle.conditioning(lambda v: v @ A.T, x, signs, eps=eps)
    base = x @ A.T
    rms = np.sqrt((base ** 2).mean(axis=1, keepdims=True))
    want = max(float((np.abs(eps * (x * s) @ A.T) / np.maximum(np.abs(base), rms)).max()) for s in signs)
    assert got == pytest.approx(want, rel=1e-9)
    assert oracle.conditioning(lambda v: v @ A.T, x, signs, eps=0.0) == 0.0


def test_a_smooth_window_moves_by_the_perturbation_itself():
    """The tiny windows are well conditioned: the result moves by a few eps, linearly in eps, so the 2e-3 bar
    stands for them (and for every case like them: no free pass)."""
    cfg = TINY["t0"]
    host = _host(cfg, cfg.n_past + cfg.T)
    x = synth.window_input(cfg).astype(np.float64)
    s1 = oracle.window_conditioning(cfg.dims, host, x, cfg.n_past, probes=2, singles=0, eps=2.0 ** -23)
    s16 = oracle.window_conditioning(cfg.dims, host, x, cfg.n_past, probes=2, singles=0, eps=2.0 ** -19)
    assert 1e-8 < s1 < 2e-6
    assert 12 < s16 / s1 < 20
    # the caches given to it are untouched
    again = _host(cfg, cfg.n_past + cfg.T)
    for a, b in zip(host, again):
        assert np.array_equal(a["k_cache"], b["k_cache"]) and np.array_equal(a["v_cache"], b["v_cache"])


def test_an_ill_conditioned_window_is_recognised():
    """A one-layer window of 13 tokens on an empty cache whose smallest top-2 logit gap is 0.89 (found by a
    randomised run): under perturbations of two fp32 roundings single fp16 roundings of appended K / V elements go
    the other way and the fp64 result itself moves by 3.6e-3, far more than a smooth window's few eps."""
    cfg = WindowConfig("s333", 1233, ModelDims(2048, 8, 8, 128, 1280, 1e6, rope_mode=0), 1, 13, 0)
    host = _host(cfg, 15)
    x = synth.window_input(cfg).astype(np.float64)
    _, taps = oracle.layer(cfg.dims, oracle._fresh(host)[0], x, 0, taps=True)
    assert 0.85 < taps["min_gap"] < 0.95
    spread = oracle.window_conditioning(cfg.dims, host, x, 0, seed=2504, eps=2.0 ** -22)
    assert 3e-3 < spread < 5e-3
    # the movement comes from the rounding boundaries, not from the random signs
    assert oracle.window_conditioning(cfg.dims, host, x, 0, probes=0, singles=0, eps=2.0 ** -22) == pytest.approx(spread)


def test_append_ties_finds_exactly_the_values_near_a_binary16_midpoint():
    """1 + 2^-11 is the midpoint of the binary16 neighbours 1 and 1 + 2^-10: values within eps of it are ties, are
    moved to its other side (so that they round to the other neighbour) and nothing else is touched."""
    eps = 2.0 ** -22
    mid = 1.0 + 2.0 ** -11
    v = np.array([mid * (1 - 0.5 * eps), mid * (1 + 0.5 * eps), mid * (1 + 3 * eps), 1.0, -mid * (1 - 0.25 * eps), 0.0, 3.14159])
    mask, moved, close = oracle._append_ties(v, eps)
    assert mask.tolist() == [True, True, False, False, True, False, False]
    f16 = lambda a: np.asarray(a).astype(np.float32).astype(np.float16).astype(np.float64)
    assert f16(v).tolist()[:2] == [1.0, 1.0 + 2.0 ** -10] and f16(moved).tolist()[:2] == [1.0 + 2.0 ** -10, 1.0]
    assert f16(v)[4] == -1.0 and f16(moved)[4] == -(1.0 + 2.0 ** -10)
    assert np.array_equal(moved[~mask], v[~mask])
    assert np.all(np.abs(moved - v) <= 2.0 * eps * np.abs(v) + 1e-300)
    assert close[0] == pytest.approx(0.5 * eps, rel=1e-3) and np.isinf(close[3])
