"""Helpers shared by the tests (no layer arithmetic)."""
import numpy as np


def scaled_err(got, want) -> float:
    """max_i |got_i - want_i| / (|want_i| + rms(want)).

    Element-wise relative error with the tensor's rms added to the denominator, so that outputs
    which happen to be near zero do not dominate; 0 for two empty or two all-zero tensors."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (got.shape, want.shape)
    if want.size == 0:
        return 0.0
    rms = float(np.sqrt(np.mean(want * want)))
    diff = np.abs(got - want)
    if rms == 0.0:
        return float(diff.max())
    return float((diff / (np.abs(want) + rms)).max())


def make_problem(oracle, lin, tensors):
    lay = lin.layout
    return oracle.Problem(tensors.x, tensors.W, tensors.A, tensors.B, lay.seg_off,
                          lay.seg_adapter, lay.scale, lay.rank)
