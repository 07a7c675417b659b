"""Helpers for the GPU tests: upload a workload.Problem, run the HIP library through its C ABI, compare."""
import numpy as np

from paper_2507_01663_amd.torch_util import DeviceProblem, bits_to_bf16  # noqa: F401  (the tests import them from here)

ABS_TOL = 1e-2      # max |out_gpu - out_ref| over all elements
REL_TOL = 1e-2      # per (b, h) row: ||out_gpu - out_ref||_2 / ||out_ref||_2
LSE_TOL = 1e-3      # |lse_gpu - lse_ref|


def compare(out, lse, ref_out, ref_lse, what="", abs_rel=0.0):
    """Asserts the three tolerances; returns the measured errors.  abs_rel widens the element-wise bound to
    ABS_TOL + abs_rel * |ref| for outputs that are not small: rounding the exact result to bf16 alone moves an
    element by up to 2**-9 of its magnitude, which passes ABS_TOL once |ref| > 5 (prompt prefill: the first tokens of a
    prompt average over few values; a decode step averages over hundreds and never gets there)."""
    assert np.isfinite(out).all(), what + ": non-finite output"
    empty = np.isneginf(ref_lse)
    assert (np.isneginf(lse) == empty).all(), what + ": -inf pattern of lse differs"
    d = out - ref_out
    abs_err = float(np.abs(d).max()) if d.size else 0.0
    num = np.sqrt((d * d).sum(axis=-1))
    den = np.sqrt((ref_out * ref_out).sum(axis=-1))
    rel = np.where(den > 0, num / np.maximum(den, 1e-300), num)
    rel_err = float(rel.max()) if rel.size else 0.0
    lse_err = float(np.abs(lse[~empty] - ref_lse[~empty]).max()) if (~empty).any() else 0.0
    excess = float((np.abs(d) - abs_rel * np.abs(ref_out)).max()) if d.size else 0.0
    assert excess <= ABS_TOL, "%s: max abs err %.3e (%.3e beyond the magnitude allowance)" % (what, abs_err, excess)
    assert rel_err <= REL_TOL, "%s: max row rel err %.3e" % (what, rel_err)
    assert lse_err <= LSE_TOL, "%s: max lse err %.3e" % (what, lse_err)
    return abs_err, rel_err, lse_err
