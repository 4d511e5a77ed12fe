"""Pins of the oracle's parameter-update functions (decode + optimizer step, Sections 4.1 and 4.3):
closed forms for a constant gradient, the zero-gradient case (unsent elements), and torch's CPU
optimizers as an independent library implementation of the same methods."""
import numpy as np
import pytest

from oracle import vgc_oracle as O

F32 = np.float32


def test_momentum_constant_gradient_closed_form():
    # m_T = -lr g (1 - mu^T) / (1 - mu);  w_T = w_0 + sum_t m_t
    lr, mu, T = 0.05, 0.9, 40
    g = np.array([0.5, -2.0, 1e-3, 0.0], F32)
    w = np.array([1.0, -1.0, 0.25, 3.0], F32)
    m = np.zeros(4, F32)
    w0 = w.astype(np.float64)
    for _ in range(T):
        w, m = O.momentum_sgd_step(g, w, m, lr, mu)
    g64 = g.astype(np.float64)
    m_T = -lr * g64 * (1 - mu ** T) / (1 - mu)
    # sum_{t=1..T} m_t = -lr g / (1 - mu) * (T - mu (1 - mu^T) / (1 - mu))
    w_T = w0 - lr * g64 / (1 - mu) * (T - mu * (1 - mu ** T) / (1 - mu))
    assert np.allclose(m, m_T, rtol=1e-5, atol=1e-9)
    assert np.allclose(w, w_T, rtol=1e-5, atol=1e-7)
    assert w[3] == F32(3.0) and m[3] == 0.0                     # zero gradient, zero momentum: untouched


def test_momentum_unsent_elements_only_decay():
    # an element nobody sent has ghat = 0: m shrinks by mu per step and w moves by the remaining momentum
    w, m = np.array([2.0], F32), np.array([0.5], F32)
    z = np.zeros(1, F32)
    w1, m1 = O.momentum_sgd_step(z, w, m, 0.1, 0.5)
    assert m1[0] == F32(0.25) and w1[0] == F32(2.25)
    w2, m2 = O.momentum_sgd_step(z, w1, m1, 0.1, 0.5)
    assert m2[0] == F32(0.125) and w2[0] == F32(2.375)


def test_momentum_hand_computed_step():
    # mu m - lr g = 0.9*1.0 - 0.5*0.25 = 0.775;  w + m = -1 + 0.775 = -0.225 (all exact or one rounding in float32)
    w, m = O.momentum_sgd_step(np.array([0.25], F32), np.array([-1.0], F32), np.array([1.0], F32), 0.5, 0.9)
    assert m[0] == F32(F32(0.9) * F32(1.0) - F32(0.125)) and abs(float(m[0]) - 0.775) < 1e-7
    assert abs(float(w[0]) + 0.225) < 1e-7
    # the sign convention: a positive gradient lowers the parameter
    assert w[0] > -1.0 and O.momentum_sgd_step(np.array([4.0], F32), np.array([-1.0], F32), np.zeros(1, F32), 0.5, 0.9)[0][0] == F32(-3.0)


def test_adam_constant_gradient_moves_by_lr_per_step():
    # with a constant gradient the bias-corrected moments are g and g^2 at every step, so every step is
    # lr g / (|g| + eps): the property the bias correction exists for (a wrong or swapped beta breaks it)
    lr, b1, b2, eps, T = 1e-3, 0.9, 0.999, 1e-8, 25
    g = np.array([3.0, -0.02, 1e-4], F32)
    w = np.zeros(3, F32); m = np.zeros(3, F32); v = np.zeros(3, F32)
    for t in range(1, T + 1):
        w, m, v = O.adam_step(g, w, m, v, lr, b1, b2, eps, t)
    g64 = g.astype(np.float64)
    assert np.allclose(w, -T * lr * g64 / (np.abs(g64) + eps), rtol=2e-5)
    assert np.allclose(m, g64 * (1 - b1 ** T), rtol=1e-5) and np.allclose(v, g64 ** 2 * (1 - b2 ** T), rtol=1e-4)


def test_adam_zero_gradient_after_history():
    # unsent element: moments decay by beta1 / beta2, the step is lr mhat / (sqrt(vhat) + eps)
    w, m, v = np.array([1.0], F32), np.array([0.5], F32), np.array([0.25], F32)
    w1, m1, v1 = O.adam_step(np.zeros(1, F32), w, m, v, 0.1, 0.5, 0.75, 0.0, 3)
    assert m1[0] == F32(0.25) and v1[0] == F32(0.1875)
    mhat, vhat = 0.25 / (1 - 0.5 ** 3), 0.1875 / (1 - 0.75 ** 3)
    assert abs(float(w1[0]) - (1.0 - 0.1 * mhat / np.sqrt(vhat))) < 1e-6


@pytest.mark.parametrize("opt", ["momentum_sgd", "adam"])
def test_against_torch_cpu_optimizers(opt):
    import torch
    rng = np.random.default_rng(7)
    n, T = 257, 12
    w0 = rng.standard_normal(n).astype(F32)
    grads = [(rng.standard_normal(n) * (rng.random(n) < 0.3)).astype(F32) for _ in range(T)]   # 70 % unsent = zero
    p = torch.nn.Parameter(torch.from_numpy(w0.astype(np.float64)))
    if opt == "momentum_sgd":
        # torch: buf <- mu buf + g; p <- p - lr buf.  With a constant lr, -lr buf is the m of the classical form.
        tor = torch.optim.SGD([p], lr=0.05, momentum=0.9)
    else:
        tor = torch.optim.Adam([p], lr=1e-3, betas=(0.9, 0.999), eps=1e-8)
    w, s1, s2 = w0.copy(), np.zeros(n, F32), np.zeros(n, F32)
    for t, g in enumerate(grads, 1):
        p.grad = torch.from_numpy(g.astype(np.float64))
        tor.step()
        if opt == "momentum_sgd":
            w, s1 = O.momentum_sgd_step(g, w, s1, 0.05, 0.9)
        else:
            w, s1, s2 = O.adam_step(g, w, s1, s2, 1e-3, 0.9, 0.999, 1e-8, t)
    assert np.allclose(w, p.detach().numpy(), rtol=2e-5, atol=2e-6)


def test_unpack_apply_is_decode_then_step():
    # two workers' messages built by hand: worker 0 sends +2^-1 at index 1, worker 1 sends -2^-2 at index 1 and +2^0 at 3
    groups = [(0, 4)]
    m0 = (np.array([(0 << 31) | (0 << 28) | 1], np.uint32), [(126, 1, 0)])
    m1 = (np.array([(1 << 31) | (2 << 28) | 1, (0 << 31) | (0 << 28) | 3], np.uint32), [(127, 2, 0)])
    w = np.array([1.0, 1.0, 1.0, 1.0], F32)
    m = np.zeros(4, F32)
    w1, m1_ = O.unpack_apply([m0, m1], groups, 0.5, 4, "momentum_sgd", w, m, lr=1.0, mu=0.0)
    # ghat = 0.5 * [0, 0.5 - 0.25, 0, 1.0] = [0, 0.125, 0, 0.5]
    assert np.array_equal(m1_, np.array([0.0, -0.125, 0.0, -0.5], F32))
    assert np.array_equal(w1, np.array([1.0, 0.875, 1.0, 0.5], F32))
