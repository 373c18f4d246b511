"""Helpers shared by the GPU parity tests."""
import numpy as np
import torch

import oracle
from paper_2509_21841_amd import synth

O_MAXABS, O_RELL2, LSE_MAXABS = 2e-2, 5e-3, 1e-3   # bf16 inputs, fp32 accumulation


def widen(t: torch.Tensor) -> np.ndarray:
    """Device tensor (bf16 or f32) -> float64 numpy, exactly."""
    if t.dtype == torch.bfloat16:
        return oracle.bf16_bits_to_f64(synth.bf16_bits(t))
    return t.detach().cpu().to(torch.float64).numpy()


def assert_close(name, got, ref, maxabs=O_MAXABS, rell2=O_RELL2, bf16_out=True):
    """max-abs <= 2e-2 and relative-L2 <= 5e-3 over the tensor. The absolute bound is the stated one for every
    element with |ref| <= 4. Above that two things grow with the magnitude and the bound follows them: the error of
    the bf16 probabilities inside the sums is relative, so the bound scales as 2e-2 * |ref| / 4 (the same 0.5 %
    relative slack it grants at |ref| = 4); and a bf16 OUTPUT sits on a grid whose half-spacing is 1.6e-2 in [4,8),
    3.1e-2 in [8,16), ... -- what that exceeds the half-spacing below 4 (7.8e-3, already inside the 2e-2) is added.
    bf16_out=False for float32 results (accumulators, partial outputs), which carry no output rounding."""
    got = np.asarray(got, np.float64); ref = np.asarray(ref, np.float64)
    assert got.shape == ref.shape, (name, got.shape, ref.shape)
    assert np.isfinite(got).all(), f"{name}: non-finite values"
    if got.size == 0:
        return
    diff = np.abs(got - ref)
    bound = maxabs * np.maximum(1.0, np.abs(ref) / 4.0)
    if bf16_out:
        half_ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(ref), 1.0))) - 8.0)   # bf16: 8 significand bits
        bound = bound + np.maximum(0.0, half_ulp - 2.0 ** -7)
    worst = int(np.argmax(diff / bound))
    err = float(diff.ravel()[worst]); at = float(ref.ravel()[worst])
    den = float(np.linalg.norm(ref.ravel()))
    rel = float(np.linalg.norm((got - ref).ravel())) / den if den > 0 else float(diff.max())
    assert (diff <= bound).all() and rel <= rell2, \
        f"{name}: abs error {err:.3e} at ref {at:.3f} (bound {float(bound.ravel()[worst]):.3e}), rel-L2 {rel:.3e} (<= {rell2})"


def assert_lse_close(name, got, ref):
    got = np.asarray(got, np.float64); ref = np.asarray(ref, np.float64)
    inf = np.isneginf(ref)
    assert np.array_equal(np.isneginf(got), inf), f"{name}: -inf pattern differs"
    if (~inf).any():
        err = float(np.abs(got[~inf] - ref[~inf]).max())
        assert err <= LSE_MAXABS, f"{name}: LSE max-abs {err:.3e}"
