"""Pins of the cross-entropy oracle (CPU): a library routine in fp64 (torch.nn.functional.cross_entropy and autograd),
closed forms, invariants and finite differences."""
import numpy as np
import torch

from oracle import fused_ce_oracle as orc


def test_against_torch_autograd_fp64():
    rng = np.random.default_rng(0)
    z = rng.normal(size=(7, 40)) * 3
    y = rng.integers(0, 40, size=7)
    y[3] = -1                                     # ignored row
    loss, grad = orc.cross_entropy(z, y, grad_scale=0.25)
    zt = torch.tensor(z, dtype=torch.float64, requires_grad=True)
    lt = torch.nn.functional.cross_entropy(zt, torch.tensor(y), reduction="none", ignore_index=-1)
    (lt.sum() * 0.25).backward()
    assert np.allclose(loss, lt.detach().numpy(), rtol=0, atol=1e-12)
    assert np.allclose(grad, zt.grad.numpy(), rtol=0, atol=1e-12)


def test_closed_forms_and_invariants():
    V = 64
    loss, grad = orc.cross_entropy(np.zeros((1, V)), [5])           # uniform logits: loss = ln V, grad = 1/V - onehot
    assert abs(loss[0] - np.log(V)) < 1e-14
    want = np.full(V, 1.0 / V); want[5] -= 1
    assert np.allclose(grad[0], want, atol=1e-15)
    rng = np.random.default_rng(1)
    z = rng.normal(size=(3, V)) * 5
    y = [0, V - 1, 17]
    l1, g1 = orc.cross_entropy(z, y)
    l2, g2 = orc.cross_entropy(z + 123.0, y)                        # shift invariance of the softmax
    assert np.allclose(l1, l2, atol=1e-10) and np.allclose(g1, g2, atol=1e-12)
    assert np.allclose(g1.sum(axis=1), 0, atol=1e-14)               # rows of the gradient sum to zero
    zz = np.full((1, V), -50.0); zz[0, 9] = 50.0                    # a row dominated by its target: loss -> 0, grad -> 0
    l3, g3 = orc.cross_entropy(zz, [9])
    assert l3[0] < 1e-30 or l3[0] < 1e-12
    assert np.abs(g3).max() < 1e-12


def test_finite_differences():
    rng = np.random.default_rng(2)
    z = rng.normal(size=(2, 9))
    y = [4, 0]
    _, g = orc.cross_entropy(z, y)
    h = 1e-6
    for i in range(2):
        for j in range(9):
            zp, zm = z.copy(), z.copy()
            zp[i, j] += h; zm[i, j] -= h
            d = (orc.cross_entropy(zp, y)[0].sum() - orc.cross_entropy(zm, y)[0].sum()) / (2 * h)
            assert abs(d - g[i, j]) < 1e-8
