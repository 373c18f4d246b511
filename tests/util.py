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


def assert_close(name, got, ref, maxabs=O_MAXABS, rell2=O_RELL2):
    got = np.asarray(got, np.float64); ref = np.asarray(ref, np.float64)
    assert got.shape == ref.shape, (name, got.shape, ref.shape)
    assert np.isfinite(got).all(), f"{name}: non-finite values"
    if got.size == 0:
        return
    err = float(np.abs(got - ref).max())
    den = float(np.linalg.norm(ref.ravel()))
    rel = float(np.linalg.norm((got - ref).ravel())) / den if den > 0 else err
    assert err <= maxabs and rel <= rell2, f"{name}: max-abs {err:.3e} (<= {maxabs}), rel-L2 {rel:.3e} (<= {rell2})"


def assert_lse_close(name, got, ref):
    got = np.asarray(got, np.float64); ref = np.asarray(ref, np.float64)
    inf = np.isneginf(ref)
    assert np.array_equal(np.isneginf(got), inf), f"{name}: -inf pattern differs"
    if (~inf).any():
        err = float(np.abs(got[~inf] - ref[~inf]).max())
        assert err <= LSE_MAXABS, f"{name}: LSE max-abs {err:.3e}"
