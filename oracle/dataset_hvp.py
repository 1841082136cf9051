"""Dataset-averaged Hessian-vector product: the batch loop of Algorithm 1.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).  Algorithm 1 walks the
batches of the data set, takes the Hessian-vector product u_B of each batch's
mean loss, accumulates h += u_B * |B| with |B| the number of samples
(sequences) in the batch, counts N += |B| and returns h / N.  The steps are
taken in that order and notation here; the per-batch product is oracle.models.
"""
from __future__ import annotations

import numpy as np

from . import models


def hvp_dataset(model, params, batches, v):
    """batches: iterable of (inputs, labels), one entry per batch B; |B| is the
    leading dimension of inputs.  Returns (h / N, sum_B |B| L_B / N) in float64."""
    v = np.asarray(v, dtype=np.float64)
    h = np.zeros_like(v)
    N = 0
    loss = 0.0
    for inputs, labels in batches:
        size = int(np.asarray(inputs).shape[0])
        L_B, _, u_B, _ = models.loss_grad_hvp(model, params, inputs, labels, v)
        h += u_B * size
        loss += L_B * size
        N += size
    return h / N, loss / N


def split_batches(inputs, labels, micro_batch):
    """Consecutive batches of `micro_batch` samples; the last one may be smaller."""
    inputs, labels = np.asarray(inputs), np.asarray(labels)
    return [(inputs[i:i + micro_batch], labels[i:i + micro_batch]) for i in range(0, inputs.shape[0], micro_batch)]
