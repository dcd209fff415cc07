"""The hidden-state tolerance of the window-level parity tests, and the one mechanical excuse.

Bar: max relative error 2e-3 (metrics.rel_err).  A case that misses it is excused only by a bound computed from
the oracle alone: oracle.window_conditioning perturbs every intermediate that an implementation with FP32
activations has to store by a relative eps with random signs and reports how far the fp64 result itself moves
(with the benchmark's value distribution attention logits reach 1e4..1e6, the softmax sits one fp16 rounding of an
appended K/V element away from another mixture, and single such roundings move outputs by several 1e-3).  eps is
the accuracy class of the mat-vec on the path, which the operator-level tests assert separately:
  EPS_Q4K   two fp32 roundings (2^-22): the Q4_K mat-vec (exact integer sums, fp32 recombination; measured rms error
            1e-7 of the output's rms)
  EPS_GEMM  2^-21: the Q4_K matrix product of the prompt call (22-bit activations and a chain of fp32 roundings per
            super-block: measured rms error 2.2e-7, single outputs up to 1.7e-6)
  EPS_FP32  2^-20: the other formats' mat-vec (fp32 accumulation along K).
The perturbed evaluations: four with random signs everywhere, and the deterministic ones in which appended K / V
values that lie within eps of a binary16 rounding boundary are rounded the other way (all of them, and the twelve
closest one at a time).  A case passes when err <= 2e-3 or err <= 1.5 x the largest movement over these
evaluations; both numbers are printed.  Nothing from the GPU result enters the bound.
"""
import oracle

HID_TOL = 2e-3
EPS_Q4K = 2.0 ** -22
EPS_GEMM = 2.0 ** -21
EPS_FP32 = 2.0 ** -20
SLACK = 1.5

excused = []  # (label, err, bound) of every case that needed the excuse in this process


def check_hidden(label, err, dims, host_layers, x, n_past, formats=None, eps=EPS_Q4K):
    """Assert the hidden-state bar for one window case.  host_layers: the layers' tensors (cache rows >= n_past may
    hold anything: every oracle evaluation works on a copy and writes them before it reads them), or a callable
    that returns them (large windows are regenerated from their seeds only when the bound is needed)."""
    if err <= HID_TOL:
        return
    if callable(host_layers):
        host_layers = host_layers()
    spread = oracle.window_conditioning(dims, host_layers, x, n_past, formats=formats, seed=2504, eps=eps)
    bound = SLACK * spread
    print(f"{label}: err {err:.3e} misses {HID_TOL:g}; the oracle's own result moves by {spread:.3e} under perturbations of "
          f"{eps:.2e} of its stored intermediates -> bar {bound:.3e}", flush=True)
    assert err <= bound, (label, err, spread)
    excused.append((label, err, bound))
