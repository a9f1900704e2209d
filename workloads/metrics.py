"""Accuracy metrics of the paper's appendix "Datasets and Metrics" (accuracy metrics
paragraph): cosine similarity, relative L1 and RMSE of the flattened outputs, plus the
row-normalised max-abs error used as the parity bar of this repository."""
import numpy as np


def _flat64(x):
    return np.asarray(x, dtype=np.float64).ravel()


def cos_sim(o_test, o_ref):
    a, b = _flat64(o_test), _flat64(o_ref)
    den = np.sqrt((a * a).sum()) * np.sqrt((b * b).sum())
    return float((a * b).sum() / den) if den > 0 else 1.0


def rel_l1(o_test, o_ref):
    a, b = _flat64(o_test), _flat64(o_ref)
    den = np.abs(b).sum()
    return float(np.abs(a - b).sum() / den) if den > 0 else 0.0


def rmse(o_test, o_ref):
    a, b = _flat64(o_test), _flat64(o_ref)
    return float(np.sqrt(np.mean((a - b) ** 2)))


def max_abs_over_row_linf(o_test, o_ref):
    """max over rows of max_c |o_test - o_ref| / max_c |o_ref| (rows = last axis)."""
    a = np.asarray(o_test, dtype=np.float64)
    b = np.asarray(o_ref, dtype=np.float64)
    a = a.reshape(-1, a.shape[-1])
    b = b.reshape(-1, b.shape[-1])
    den = np.abs(b).max(axis=1)
    den = np.where(den > 0, den, 1.0)
    return float((np.abs(a - b).max(axis=1) / den).max())
