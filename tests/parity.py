"""Comparison rule shared by the GPU parity tests.

bf16 inputs, fp32 accumulation, one bf16 rounding of the output.  A result passes when BOTH
hold: every element is within 2e-2 absolute of the fp64 checker, and every (token, head)
row is within 1e-2 relative in the 2-norm.  With N(0,1) values and contexts of hundreds of
tokens the outputs are O(0.05), so the row-relative bound is the one with teeth; the
expected error is ~2^-9 per element from the output rounding plus the averaged-down
rounding of the bf16 softmax weights.
"""
import numpy as np

ABS_TOL = 2e-2
ROW_REL_TOL = 1e-2


def compare(got: np.ndarray, ref: np.ndarray, what: str = ""):
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.isfinite(got).all(), "%s: non-finite output" % what
    err = np.abs(got - ref)
    denom = np.linalg.norm(ref, axis=-1)
    rel = np.linalg.norm(got - ref, axis=-1) / np.where(denom > 0, denom, 1.0)
    worst = np.unravel_index(np.argmax(rel), rel.shape)
    msg = "%s: max abs %.3e, max row rel %.3e at %s" % (what, err.max(), rel.max(), worst)
    assert err.max() <= ABS_TOL, msg
    assert rel.max() <= ROW_REL_TOL, msg
    assert (err <= ABS_TOL + ROW_REL_TOL * np.abs(ref)).all(), msg
    return float(err.max()), float(rel.max())
