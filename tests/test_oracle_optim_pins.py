"""Pins for the optimizer oracle: torch.optim on CPU float64 (a library routine the oracle does not
call), closed forms of the first step, and special cases."""
import numpy as np
import pytest

from oracle import optim as oo


def _data(seed=0, n=257):
    rng = np.random.default_rng(seed)
    return rng.standard_normal(n), [rng.standard_normal(n) for _ in range(4)]


@pytest.mark.parametrize("momentum,wd", [(0.0, 0.0), (0.9, 0.0), (0.9, 0.01), (0.0, 0.1)])
def test_sgd_matches_torch(momentum, wd):
    torch = pytest.importorskip("torch")
    p0, grads = _data(1)
    tp = torch.tensor(p0.copy(), dtype=torch.float64, requires_grad=True)
    opt = torch.optim.SGD([tp], lr=0.05, momentum=momentum, weight_decay=wd)
    p, buf = p0.copy(), np.zeros_like(p0)
    for g in grads:
        tp.grad = torch.tensor(g)
        opt.step()
        p, buf = oo.sgd_step(p, g, buf, lr=0.05, momentum=momentum, weight_decay=wd)
        assert np.allclose(p, tp.detach().numpy(), atol=1e-13)


@pytest.mark.parametrize("wd", [0.0, 0.01])
def test_adam_matches_torch(wd):
    torch = pytest.importorskip("torch")
    p0, grads = _data(2)
    tp = torch.tensor(p0.copy(), dtype=torch.float64, requires_grad=True)
    opt = torch.optim.Adam([tp], lr=1e-2, betas=(0.9, 0.98), eps=1e-6, weight_decay=wd)
    p, m, v = p0.copy(), np.zeros_like(p0), np.zeros_like(p0)
    for t, g in enumerate(grads, start=1):
        tp.grad = torch.tensor(g)
        opt.step()
        p, m, v = oo.adam_step(p, g, m, v, lr=1e-2, step=t, beta1=0.9, beta2=0.98, eps=1e-6, weight_decay=wd)
        assert np.allclose(p, tp.detach().numpy(), atol=1e-12)


def test_closed_forms_of_the_first_step():
    p, g = np.array([1.0, -2.0, 0.5]), np.array([0.3, -0.1, 2.0])
    # Adam, step 1, no decay: m_hat = g, v_hat = g^2  =>  p - lr * g / (|g| + eps) = p - lr * sign(g) (eps -> 0)
    pn, m, v = oo.adam_step(p, g, np.zeros(3), np.zeros(3), lr=0.1, step=1, eps=0.0)
    assert np.allclose(pn, p - 0.1 * np.sign(g), atol=1e-15)
    assert np.allclose(m, 0.1 * g) and np.allclose(v, 0.001 * g * g)
    # SGD: plain, and two momentum steps with a constant gradient: buf2 = (1 + mu) g
    pn, buf = oo.sgd_step(p, g, np.zeros(3), lr=0.5)
    assert np.allclose(pn, p - 0.5 * g) and np.allclose(buf, g)
    p1, b1 = oo.sgd_step(p, g, np.zeros(3), lr=0.5, momentum=0.9)
    p2, b2 = oo.sgd_step(p1, g, b1, lr=0.5, momentum=0.9)
    assert np.allclose(b2, 1.9 * g) and np.allclose(p2, p - 0.5 * g - 0.5 * 1.9 * g)
    # weight decay alone shrinks the parameter geometrically
    pn, _ = oo.sgd_step(p, np.zeros(3), np.zeros(3), lr=0.1, weight_decay=0.5)
    assert np.allclose(pn, p * (1 - 0.05))
    assert np.allclose(oo.accumulate(p, g), p + g)


def test_zero_gradient_leaves_adam_parameters_unchanged():
    p = np.array([1.0, 2.0])
    pn, m, v = oo.adam_step(p, np.zeros(2), np.zeros(2), np.zeros(2), lr=0.1, step=1)
    assert np.array_equal(pn, p) and not m.any() and not v.any()
