"""prima_q4k_gemv_noalloc (the entry point for callers that cannot allocate: the scratch is a fixed array in the
library's device image) against prima_q4k_gemv on the same inputs: same kernels, same plan, so the same bits.
Two calls in a row, the second with a smaller input, both on shapes whose launch really uses the scratch
(K cut into slabs: partial sums and arrival counters in global memory); then the oracle on the second."""
import numpy as np
import pytest
import torch

import oracle
from metrics import rel_err
from workloads import synth

pytestmark = pytest.mark.gpu


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def test_noalloc_gemv_equals_gemv_on_two_calls_in_a_row(gpu_lib):
    prima = gpu_lib
    # (rows, cols, T): K = 28672 at one token runs as several slabs; so do 5 tokens at K = 8192 (fewer rows: smaller)
    cases = [(2048 + 7, 28672, 1), (512 + 3, 8192, 5)]
    outs = []
    for i, (rows, cols, T) in enumerate(cases):
        assert prima.gemv_workspace_bytes(rows, cols, T) <= prima._ffi.NOALLOC_SCRATCH_BYTES
        W = synth.q4k_tensor(900 + i, 0, "wdown", rows, cols)
        x = synth.normal_f32(900 + i, 0, "x_in", (T, cols))
        Wd, xd = _dev(W), _dev(x)
        want = prima.q4k_gemv(Wd, xd)
        got = torch.full((T, rows), float("nan"), dtype=torch.float32, device="cuda")
        before = torch.cuda.memory_allocated()
        prima.q4k_gemv_noalloc(Wd, xd, got)
        assert torch.cuda.memory_allocated() == before
        torch.cuda.synchronize()
        print(f"noalloc case {i}: {rows} x {cols}, T={T}", flush=True)
        assert torch.equal(got, want), (rows, cols, T)
        outs.append((W, x, got.cpu().numpy()))
    # and the second, smaller call against the oracle (the first call's leftovers in the array did no harm)
    W, x, got = outs[1]
    ref = oracle.gemv(W, x.astype(np.float64))
    assert rel_err(got, ref) < 2e-3


def test_noalloc_gemv_rejects_what_does_not_fit(gpu_lib):
    prima = gpu_lib
    rows, cols, T = 128256, 8192, 8      # the output layer at 8 tokens: 8 slabs of partial sums, far beyond the array
    assert prima.gemv_workspace_bytes(rows, cols, T) > prima._ffi.NOALLOC_SCRATCH_BYTES
    W = torch.zeros((16, cols // 256, 144), dtype=torch.uint8, device="cuda")
    x = torch.zeros((T, cols), dtype=torch.float32, device="cuda")
    y = torch.zeros((T, rows), dtype=torch.float32, device="cuda")
    lib = prima._ffi.lib()
    # (W is too small for the shape claimed: nothing may be launched, and nothing is: the size check comes first)
    rc = lib.prima_q4k_gemv_noalloc(W.data_ptr(), rows, cols, x.data_ptr(), cols, T, y.data_ptr(), rows, None)
    assert rc == 5  # PRIMA_E_WORKSPACE
