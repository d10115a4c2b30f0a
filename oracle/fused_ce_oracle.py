"""Plain fp64 reference of the fused in-place cross-entropy (paper section 4, "Fused In-Place Cross-Entropy"): the loss
of every row and the gradient of the logits that the operator leaves in their place.  Test infrastructure only.

The operator reaches a result with a plain definition, written out here: for a row z with target y,
loss = log(sum_j exp(z_j)) - z_y and d loss / d z_j = softmax(z)_j - [j == y]; rows with a negative target are ignored
(loss 0, gradient 0)."""
from __future__ import annotations

import numpy as np


def cross_entropy(logits, targets, grad_scale=1.0):
    """logits: [rows, vocab] (any float array, widened to fp64), targets: [rows] ints.  Returns (loss[rows], grad[rows, vocab])."""
    z = np.asarray(logits, dtype=np.float64)
    rows, vocab = z.shape
    loss = np.zeros(rows)
    grad = np.zeros_like(z)
    for i in range(rows):
        y = int(targets[i])
        if y < 0 or y >= vocab:
            continue
        m = z[i].max()
        e = np.exp(z[i] - m)
        s = e.sum()
        loss[i] = m + np.log(s) - z[i, y]
        grad[i] = e / s
        grad[i, y] -= 1.0
        grad[i] *= grad_scale
    return loss, grad
