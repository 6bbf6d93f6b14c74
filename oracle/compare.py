"""The parity metric for floating-point outputs.

Error of an output row is measured against the largest magnitude the oracle gives in
that row: max_n |got[m,n] - ref[m,n]| <= tol * max_n |ref[m,n]|; a row whose reference
is identically zero must be matched exactly.
"""
import numpy as np


def row_rel_error(got64, ref64):
    """Per-row max|got-ref| / max|ref| (inf where ref row is 0 and got is not)."""
    got64 = np.asarray(got64, dtype=np.float64)
    ref64 = np.asarray(ref64, dtype=np.float64)
    err = np.abs(got64 - ref64).max(axis=1)
    nrm = np.abs(ref64).max(axis=1)
    out = np.zeros_like(err)
    nz = nrm > 0
    out[nz] = err[nz] / nrm[nz]
    out[~nz & (err > 0)] = np.inf
    return out


def max_row_rel_error(got64, ref64):
    if got64.size == 0:
        return 0.0
    return float(row_rel_error(got64, ref64).max())
