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


def bf16_half_ulp(x):
    """Half the spacing of the bfloat16 grid (8 significand bits) at magnitude |x| >= 2^-126."""
    return 2.0 ** (np.floor(np.log2(np.maximum(np.abs(x), 2.0 ** -126))) - 8.0)


class StatedBoundNotMet(AssertionError):
    """The stated max-abs bound of 2e-2 fails on a FEW elements by a LITTLE while the relative-L2 bound holds: at most
    max(3, size / 10000) elements, each within 1.5 x the bound (plus the bf16 half-spacing at its magnitude for a bf16
    output). That is the tail of the rounding of the bf16 MFMA operands (P, dS carry 2^-9 relative error per term) and
    of the bf16 output grid (half-spacing 1.56e-2 on [4,8)) on sums over the 4-8 query heads of a GQA group -- not a
    wrong mask, index or descriptor, which shows as errors of order one and breaks the relative-L2 bound.
    Tests known to end here are marked xfail(strict=True, raises=StatedBoundNotMet) with the element counts in the
    reason: the stated bound is NOT met there, nothing else may fail (any other error raises a plain AssertionError,
    which the mark does not accept), and a change that makes them pass shows up as XPASS."""


def assert_close(name, got, ref, maxabs=O_MAXABS, rell2=O_RELL2, bf16_out=True):
    """The stated bounds: max-abs <= 2e-2 on EVERY element and relative-L2 <= 5e-3 over the tensor.

    One exception, forced by the output format alone: a bf16 result with |ref| >= 8 sits on a grid whose half-spacing
    (3.1e-2 on [8,16), 6.2e-2 on [16,32), ...) already exceeds 2e-2, so there -- and only there, and only for bf16
    outputs -- the bound is 2e-2 plus that half-spacing. Nothing scales with the magnitude otherwise; float32 results
    (partial outputs, running rows, gradient accumulators: bf16_out=False) get the flat bound everywhere.
    On failure the message counts the elements over their bound and names the worst one; the failure is a
    StatedBoundNotMet if it is the small tail that class describes, a plain AssertionError otherwise."""
    got = np.asarray(got, np.float64); ref = np.asarray(ref, np.float64)
    assert got.shape == ref.shape, (name, got.shape, ref.shape)
    assert np.isfinite(got).all(), f"{name}: non-finite values"
    if got.size == 0:
        return
    diff = np.abs(got - ref)
    bound = np.full(ref.shape, float(maxabs))
    if bf16_out:
        big = np.abs(ref) >= 8.0
        bound[big] += bf16_half_ulp(ref[big])
    den = float(np.linalg.norm(ref.ravel()))
    rel = float(np.linalg.norm((got - ref).ravel())) / den if den > 0 else float(diff.max())
    over = diff > bound
    if over.any() or rel > rell2:
        worst = int(np.argmax(diff - bound))
        msg = (f"{name}: {int(over.sum())} of {diff.size} elements over the max-abs bound; worst error "
               f"{float(diff.ravel()[worst]):.3e} at ref {float(ref.ravel()[worst]):.4f} (bound "
               f"{float(bound.ravel()[worst]):.3e}); largest error anywhere {float(diff.max()):.3e}; "
               f"rel-L2 {rel:.3e} (<= {rell2})")
        envelope = 1.5 * bound[over] + (bf16_half_ulp(ref[over]) if bf16_out else 0.0)
        tail_only = rel <= rell2 and int(over.sum()) <= max(3, diff.size // 10000) and bool((diff[over] <= envelope).all())
        raise (StatedBoundNotMet if tail_only else AssertionError)(msg)


class Checks:
    """Runs every comparison of a test before judging it: any plain failure fails the test with all messages; if the
    only failures are StatedBoundNotMet ones, that is what is raised (for the strict xfail marks to accept)."""

    def __init__(self):
        self.hard, self.soft = [], []

    def close(self, name, got, ref, **kw):
        try:
            assert_close(name, got, ref, **kw)
        except StatedBoundNotMet as e:
            self.soft.append(str(e))
        except AssertionError as e:
            self.hard.append(str(e))

    def lse(self, name, got, ref):
        try:
            assert_lse_close(name, got, ref)
        except AssertionError as e:
            self.hard.append(str(e))

    def finish(self):
        if self.hard:
            raise AssertionError("\n".join(self.hard + self.soft))
        if self.soft:
            raise StatedBoundNotMet("\n".join(self.soft))


def assert_lse_close(name, got, ref):
    got = np.asarray(got, np.float64); ref = np.asarray(ref, np.float64)
    inf = np.isneginf(ref)
    assert np.array_equal(np.isneginf(got), inf), f"{name}: -inf pattern differs"
    if (~inf).any():
        err = float(np.abs(got[~inf] - ref[~inf]).max())
        assert err <= LSE_MAXABS, f"{name}: LSE max-abs {err:.3e}"
