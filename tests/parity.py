"""The parity metric for parameter vectors, shared by the GPU tests.

"Maximum relative error" of a vector: max over columns of |gpu - ref| / max(|ref_c|, rms(ref)).
An entry at least as large as the vector's root mean square is measured against itself, a smaller
one against the rms.  Why the floor is the rms and not a small fraction of it: every update adds
terms of the size of the replicas' disagreement and of the gradient step, so fp32 rounding leaves
an absolute error of about 2^-24 times that size per operation whatever the entry's own value;
an entry that passes through zero keeps that absolute error, and against a floor of 1e-3 rms a
hundred steps of correctly rounded fp32 arithmetic already read as 1e-3.  `strict_rel_err` is that
harsher figure (floor 1e-3 rms); the tests print it beside the bar they assert.
"""
import numpy as np


def rel_err(got, ref, floor_frac=1.0):
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    floor = floor_frac * np.sqrt(np.mean(ref * ref)) + 1e-30
    return float(np.max(np.abs(got - ref) / np.maximum(np.abs(ref), floor)))


def strict_rel_err(got, ref):
    return rel_err(got, ref, 1e-3)
