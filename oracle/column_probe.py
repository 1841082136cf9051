"""Hessian-column probe of the section "Banded Hessians".

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).  A column of the Hessian is
the Hessian-vector product with a vector that is 1 at one index and 0
elsewhere.  Its sparsity is summarised the way the paper tabulates it: the
fraction (here: the count) of entries whose absolute value is below each of a
list of thresholds, and a histogram of the absolute values with equal-width
bins.

Decisions taken in float32, the precision the column is produced in: an entry
counts as below a threshold t when |h_i| < t with both sides float32; the
histogram spans [0, max_i |h_i|] with n_bins equal bins, entry i falls in bin
floor(|h_i| * (n_bins / max)) with the quotient and the product each rounded to
float32, and the largest entry belongs to the last bin (so does an entry whose
product is not a number, which takes an infinite maximum).  A column of zeros
puts every entry in bin 0.  NaN entries are below no threshold and are left out of
the maximum and of the histogram.
"""
from __future__ import annotations

import numpy as np

from . import models


def hessian_column(model, params, inputs, labels, index):
    e = np.zeros(models.num_params(model))
    e[index] = 1.0
    return models.hvp(model, params, inputs, labels, e)


def column_stats(h, thresholds, n_bins):
    """h: the column as float32.  Returns (below[len(thresholds)] int64,
    max_abs float32, hist[n_bins] int64)."""
    a = np.abs(np.asarray(h, dtype=np.float32))
    thr = np.asarray(thresholds, dtype=np.float32)
    below = np.array([int(np.count_nonzero(a < t)) for t in thr], dtype=np.int64)
    ok = ~np.isnan(a)
    mx = np.float32(a[ok].max()) if ok.any() else np.float32(0.0)
    hist = np.zeros(n_bins, dtype=np.int64)
    if mx > 0:
        scale = np.float32(n_bins) / mx                       # float32 quotient
        with np.errstate(invalid="ignore"):
            prod = a[ok] * scale                               # float32 product
        idx = np.where(np.isnan(prod), n_bins - 1, np.minimum(np.floor(np.nan_to_num(prod, nan=0.0)), n_bins - 1))
        idx = idx.astype(np.int64)
        np.add.at(hist, idx, 1)
    else:
        hist[0] = int(ok.sum())
    return below, mx, hist
