"""GPU parity of the many-token Q4_K matrix product (prompt processing) against the CPU oracle, through the C ABI.

Bar: max relative error <= 2e-3 (tests/metrics.rel_err), as for every hidden-state quantity; the kernel's own
arithmetic (22-bit activations, exact weights, fp32 sums) stays some orders below it, which is asserted too.
"""
import numpy as np
import pytest
import torch

import oracle
from metrics import rel_err

pytestmark = pytest.mark.gpu

HID_TOL = 2e-3
ARITH_TOL = 3e-6   # 22-bit activations and fp32 accumulation over at most 28672 columns: observed at most 1.7e-6


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _rand_q4k(rng, rows, nb):
    W = rng.integers(0, 256, size=(rows, nb, 144), dtype=np.uint8)
    dd = (1e-3 + 3e-3 * rng.random((rows * nb, 2), dtype=np.float32)).astype(np.float16)
    W.reshape(-1, 144)[:, 0:4] = dd.view(np.uint8).reshape(-1, 4)
    return W


def _oracle_product(W, a):
    """The oracle's mat-vec takes up to 64 tokens a call."""
    return np.concatenate([oracle.gemv(W, a[t:t + 64]) for t in range(0, a.shape[0], 64)], axis=0)


def test_gemm_shapes(gpu_lib):
    """Rows and tokens that are not multiples of the tiles (128 rows, 32 tokens), one to several super-blocks."""
    rng = np.random.default_rng(31)
    for rows, nb, T in [(1, 1, 1), (16, 1, 16), (130, 2, 33), (257, 3, 70), (1000, 5, 100), (64, 16, 31), (300, 8, 129)]:
        print("case", rows, nb, T, flush=True)
        W = _rand_q4k(rng, rows, nb)
        x = rng.standard_normal((T, nb * 256)).astype(np.float32)
        ref = _oracle_product(W, x.astype(np.float64))
        Wd, xd = _dev(W), _dev(x)
        got = gpu_lib.q4k_gemm(Wd, xd).cpu().numpy()
        again = gpu_lib.q4k_gemm(Wd, xd).cpu().numpy()
        assert got.shape == (T, rows)
        tol = ARITH_TOL if rows >= 16 else HID_TOL   # a lone output may be a sum that nearly cancels
        for t in range(T):
            assert rel_err(got[t], ref[t]) < tol, (rows, nb, T, t, rel_err(got[t], ref[t]))
        assert np.array_equal(got.view(np.uint32), again.view(np.uint32))


def test_gemm_rmsnorm_and_residual(gpu_lib):
    """RMSNorm in front, residual behind, strided rows of x, y and the residual."""
    rng = np.random.default_rng(32)
    rows, nb, T = 520, 4, 45
    W = _rand_q4k(rng, rows, nb)
    xfull = (rng.standard_normal((T, nb * 256 + 64)) * np.exp(rng.standard_normal((T, 1)) * 3)).astype(np.float32)
    gain = (1 + 0.2 * rng.standard_normal(nb * 256)).astype(np.float32)
    resid_full = rng.standard_normal((T, rows + 8)).astype(np.float32)
    eps = 1e-5
    x = xfull[:, :nb * 256]
    ref = _oracle_product(W, oracle.rmsnorm(x.astype(np.float64), gain, eps)) + resid_full[:, :rows].astype(np.float64)
    xd = _dev(xfull)[:, :nb * 256]
    rd = _dev(resid_full)[:, :rows]
    ybuf = torch.zeros((T, rows + 24), dtype=torch.float32, device="cuda")
    got = gpu_lib.q4k_gemm(_dev(W), xd, gain=_dev(gain), eps=eps, resid=rd, y=ybuf[:, :rows]).cpu().numpy()
    assert rel_err(got, ref) < ARITH_TOL, rel_err(got, ref)
    assert torch.all(ybuf[:, rows:] == 0)
    # the residual may be the output buffer
    ybuf2 = _dev(resid_full[:, :rows].copy())
    got2 = gpu_lib.q4k_gemm(_dev(W), xd, gain=_dev(gain), eps=eps, resid=ybuf2, y=ybuf2).cpu().numpy()
    assert np.array_equal(got.view(np.uint32), got2.view(np.uint32))


def test_gemm_wide_dynamic_range(gpu_lib):
    """Tokens of very different magnitude (each gets its own power-of-two scale), common-mode activations, zeros."""
    rng = np.random.default_rng(33)
    W = _rand_q4k(rng, 200, 8)
    x = np.concatenate([1e7 * (1 + 0.01 * rng.standard_normal((3, 2048))),
                        1e-9 * rng.standard_normal((3, 2048)),
                        rng.standard_normal((3, 2048)) * np.exp(4 * rng.standard_normal((3, 2048))),
                        np.zeros((2, 2048))]).astype(np.float32)
    ref = _oracle_product(W, x.astype(np.float64))
    got = gpu_lib.q4k_gemm(_dev(W), _dev(x)).cpu().numpy()
    for t in range(x.shape[0]):
        if np.abs(ref[t]).max() == 0:
            assert np.all(got[t] == 0)
        else:
            assert rel_err(got[t], ref[t]) < HID_TOL, (t, rel_err(got[t], ref[t]))
    assert np.all(np.isfinite(got))


def test_gemm_equals_the_decode_mat_vec(gpu_lib):
    """The same product from the decode kernel (integer digits) and from this one agree far inside the bar."""
    rng = np.random.default_rng(34)
    W = _rand_q4k(rng, 777, 6)
    x = rng.standard_normal((8, 6 * 256)).astype(np.float32)
    a = gpu_lib.q4k_gemm(_dev(W), _dev(x)).cpu().numpy()
    b = gpu_lib.q4k_gemv(_dev(W), _dev(x)).cpu().numpy()
    assert rel_err(a, b.astype(np.float64)) < ARITH_TOL


def test_gemm_model_shape_sampled(gpu_lib):
    """A 70B-shaped gate projection (28672 x 8192) with 512 tokens: sampled rows against the oracle."""
    rng = np.random.default_rng(35)
    rows, nb, T = 28672, 32, 512
    W = _rand_q4k(rng, rows, nb)
    x = rng.standard_normal((T, nb * 256)).astype(np.float32)
    print("case", rows, nb, T, flush=True)
    got = gpu_lib.q4k_gemm(_dev(W), _dev(x)).cpu().numpy()
    pick = np.unique(np.concatenate([[0, 15, 16, 127, 128, rows - 1], rng.integers(0, rows, 60)]))
    ref = _oracle_product(np.ascontiguousarray(W[pick]), x.astype(np.float64))
    assert rel_err(got[:, pick], ref) < ARITH_TOL, rel_err(got[:, pick], ref)


def test_gemm_k_divided_among_workgroups(gpu_lib):
    """Few rows x few tokens: with the larger workspace K is cut into shares that a second launch adds.  Both routes
    against the oracle (RMSNorm in front, residual in the output buffer, ragged rows and tokens), the same bits on a
    rerun, and nothing written beside the output."""
    from paper_2504_08791_amd import _ffi
    rng = np.random.default_rng(36)
    for rows, nb, T, want in [(64, 16, 31, 4), (300, 8, 129, 2), (1000, 40, 70, 10), (257, 64, 16, 16), (520, 33, 200, 8)]:
        print("case", rows, nb, T, flush=True)
        assert gpu_lib.gemm_ksplit(T, rows, nb * 256) == want
        W = _rand_q4k(rng, rows, nb)
        x = (rng.standard_normal((T, nb * 256)) * np.exp(rng.standard_normal((T, 1)))).astype(np.float32)
        gain = (1 + 0.2 * rng.standard_normal(nb * 256)).astype(np.float32)
        resid = rng.standard_normal((T, rows)).astype(np.float32)
        ref = _oracle_product(W, oracle.rmsnorm(x.astype(np.float64), gain, 1e-5)) + resid.astype(np.float64)
        Wd, xd, gd = _dev(W), _dev(x), _dev(gain)
        out = {}
        for split in (False, True):
            nbytes = gpu_lib.gemm_workspace_bytes(T, rows, nb * 256, ksplit=split)
            ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
            ybuf = torch.full((T, rows + 8), 7.0, dtype=torch.float32, device="cuda")
            ybuf[:, :rows] = _dev(resid)
            got = gpu_lib.q4k_gemm(Wd, xd, gain=gd, eps=1e-5, resid=ybuf[:, :rows], y=ybuf[:, :rows], workspace=ws)
            assert torch.all(ybuf[:, rows:] == 7.0)
            out[split] = got.cpu().numpy()
            for t in range(T):
                assert rel_err(out[split][t], ref[t]) < ARITH_TOL, (rows, nb, T, split, t, rel_err(out[split][t], ref[t]))
            ybuf[:, :rows] = _dev(resid)
            again = gpu_lib.q4k_gemm(Wd, xd, gain=gd, eps=1e-5, resid=ybuf[:, :rows], y=ybuf[:, :rows], workspace=ws).cpu().numpy()
            assert np.array_equal(out[split].view(np.uint32), again.view(np.uint32))
        assert not np.array_equal(out[False], out[True])      # the two routes add in different orders
        assert rel_err(out[True], out[False].astype(np.float64)) < ARITH_TOL


def test_gemm_k_divided_model_shape_sampled(gpu_lib):
    """A 70B-shaped down projection (8192 x 28672) against 128 tokens (8 shares of K): sampled rows against the oracle."""
    rng = np.random.default_rng(37)
    rows, nb, T = 8192, 112, 128
    assert gpu_lib.gemm_ksplit(T, rows, nb * 256) == 8
    W = _rand_q4k(rng, rows, nb)
    x = rng.standard_normal((T, nb * 256)).astype(np.float32)
    print("case", rows, nb, T, flush=True)
    got = gpu_lib.q4k_gemm(_dev(W), _dev(x)).cpu().numpy()
    pick = np.unique(np.concatenate([[0, 15, 16, 255, 256, rows - 1], rng.integers(0, rows, 40)]))
    ref = _oracle_product(np.ascontiguousarray(W[pick]), x.astype(np.float64))
    assert rel_err(got[:, pick], ref) < ARITH_TOL, rel_err(got[:, pick], ref)


def test_gemm_argument_errors(gpu_lib):
    from paper_2504_08791_amd import _ffi
    L = _ffi.lib()
    W = torch.zeros((16, 1, 144), dtype=torch.uint8, device="cuda")
    x = torch.zeros((4, 256), dtype=torch.float32, device="cuda")
    y = torch.zeros((4, 16), dtype=torch.float32, device="cuda")
    need = L.prima_gemm_workspace_bytes(4, 256)
    ws = torch.zeros(need, dtype=torch.uint8, device="cuda")
    p = lambda t: t.data_ptr()
    ok = lambda **k: L.prima_q4k_gemm(k.get("W", p(W)), k.get("rows", 16), k.get("cols", 256), k.get("x", p(x)), k.get("ldx", 256),
                                      k.get("T", 4), None, 0.0, None, 0, k.get("y", p(y)), k.get("ldy", 16), k.get("ws", p(ws)),
                                      k.get("wsb", need), None)
    assert ok() == 0
    assert _ffi.STATUS[ok(W=None)] == "PRIMA_E_NULL"
    assert _ffi.STATUS[ok(cols=255)] == "PRIMA_E_SHAPE"
    assert _ffi.STATUS[ok(ldy=15)] == "PRIMA_E_SHAPE"
    assert _ffi.STATUS[ok(T=0)] == "PRIMA_E_RANGE"
    assert _ffi.STATUS[ok(x=p(x) + 4)] == "PRIMA_E_ALIGN"
    assert _ffi.STATUS[ok(wsb=need - 1)] == "PRIMA_E_WORKSPACE"
    assert ok(rows=0) == 0
    torch.cuda.synchronize()
