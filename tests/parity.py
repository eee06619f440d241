"""Parity figures for parameter vectors, shared by the GPU tests.

Three figures, from the sharpest to the loosest:

* `forward_excess` - element by element, for ONE record run on identical inputs: the fp32 result may differ
  from the exactly rounded one by at most (n + 3) 2^-24 times the sum of the magnitudes of the n terms that
  were added (Higham's forward bound for a chain of n fused multiply-adds), plus the oracle's own final
  rounding.  No floor, no norm: every entry is judged against what was added to make it.  Asserted for every
  record of every per-record check.
* `strict_rel_err` - max_c |gpu - ref| / max(|ref_c|, 1e-3 rms(ref)): the "maximum relative error" of the
  target (1e-5 per step, 1e-4 per run), an entry below a thousandth of the vector's rms being measured against
  that thousandth.  Asserted on the five named workloads.
* `rel_err` - the same with the floor at rms(ref): for runs of seeded random modes and degenerate shapes,
  whose vectors can be a handful of entries, or pass through zero, where a floor of 1e-3 rms turns the
  absolute rounding error every fp32 path leaves (2^-24 of the terms per operation) into an arbitrary ratio.
"""
import numpy as np

EPS = 2.0 ** -24


def rel_err(got, ref, floor_frac=1.0):
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    floor = floor_frac * np.sqrt(np.mean(ref * ref)) + 1e-30
    return float(np.max(np.abs(got - ref) / np.maximum(np.abs(ref), floor)))


def strict_rel_err(got, ref):
    return rel_err(got, ref, 1e-3)


def forward_excess(got, ref, term_magnitudes, n_terms, extra=0.0):
    """max_c |got - ref|_c / bound_c with bound_c = (n_c + 3) 2^-24 term_magnitudes_c + 2^-24 |ref_c| + extra_c;
    at most 1 for a correct fp32 evaluation.  n_terms may be an array (a column's own number of terms)."""
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    bound = (np.asarray(n_terms, np.float64) + 3.0) * EPS * np.asarray(term_magnitudes, np.float64)
    bound = bound + EPS * np.abs(ref) + extra + 1e-37
    return float(np.max(np.abs(got - ref) / bound))
