"""Pins for the oracle's accumulate / test / reset-or-decay step (Alg. 1, Eq. 2)."""
import numpy as np
import pytest

from oracle import vgc_oracle as O
from conftest import read_golden

F32 = np.float32


def _raw_stats(y):
    """g and s of Alg. 1 from raw per-sample gradients y [B, N] (float64)."""
    B = y.shape[0]
    return (y / B).sum(0), ((y / B) ** 2).sum(0)


def test_hand_computed_step():
    G = read_golden("hand_computed_statistic.txt")
    r_acc, r_out, v_out, send = O.accumulate_select(
        [1, 0, 1, 0.5], [0.5, 1, 0.5, 0], [0, 1, -2, 0.5], [0, 1, 0.5, 1], alpha=1.0, zeta=0.5)
    assert send.astype(int).tolist() == G["step_send"]
    assert r_out.tolist() == G["step_r_out"] and v_out.tolist() == G["step_v_out"]
    assert r_acc.tolist() == [1, 1, -1, 1]
    assert r_out.dtype == F32 and v_out.dtype == F32


@pytest.mark.parametrize("B,alpha", [(8, 1.0), (32, 1.5), (16, 2.0), (4, 0.5)])
def test_appendix_a_identity(B, alpha):
    """Eq. 2 on (g, s) selects exactly the elements whose squared mean exceeds
    alpha (B-1)/(B-alpha) V_B / B, V_B the unbiased sample variance (Appendix A, last line)."""
    rng = np.random.default_rng(B)
    N = 20000
    y = rng.standard_normal((B, N)) + 0.3 * rng.standard_normal(N)
    g, s = _raw_stats(y)
    z = np.zeros(N, F32)
    _, _, _, send = O.accumulate_select(g.astype(F32), s.astype(F32), z, z, alpha, 0.999)
    mean = y.mean(0)
    var = y.var(0, ddof=1)
    lhs, rhs = mean ** 2, alpha * (B - 1) / (B - alpha) * var / B
    expect = lhs > rhs
    away = np.abs(lhs - rhs) > 1e-5 * np.maximum(lhs, rhs)       # float32 rounding of g, s
    assert away.mean() > 0.99
    assert np.array_equal(send[away], expect[away])
    assert 0.05 < send.mean() < 0.8


def test_postponed_steps_equal_one_large_batch():
    """Section 4.1: an element postponed k-1 times is tested at step k as if the batch
    were k times larger, and what is sent is the sum over the steps (zeta = 1)."""
    rng = np.random.default_rng(3)
    B, N, k, alpha = 8, 5000, 4, 1.5
    ys = [rng.standard_normal((B, N)) + 0.2 for _ in range(k)]
    r = np.zeros(N, F32)
    v = np.zeros(N, F32)
    never_sent = np.ones(N, bool)
    for t in range(k):
        g, s = _raw_stats(ys[t])
        r_acc, r, v, send = O.accumulate_select(g.astype(F32), s.astype(F32), r, v, alpha, 1.0)
        if t < k - 1:
            never_sent &= ~send
    big = np.concatenate(ys, axis=0)                              # [k*B, N]
    kb = k * B
    lhs = ((big / kb).sum(0)) ** 2
    rhs = alpha * ((big / kb) ** 2).sum(0)
    expect = lhs > rhs
    away = np.abs(lhs - rhs) > 1e-5 * np.maximum(lhs, rhs)
    sel = never_sent & away
    assert sel.sum() > 100
    assert np.array_equal(send[sel], expect[sel])
    np.testing.assert_allclose(r_acc[sel], (big / B).sum(0)[sel], rtol=1e-5, atol=1e-6)   # the sum, not the mean


def test_special_cases_and_postconditions():
    rng = np.random.default_rng(4)
    N, B = 4096, 8
    y = rng.standard_normal((B, N))
    g, s = _raw_stats(y)
    g, s = g.astype(F32), s.astype(F32)
    z = np.zeros(N, F32)
    # alpha = 0: every non-zero accumulated value is sent
    g0 = g.copy(); g0[:7] = 0
    r_acc, r_out, v_out, send = O.accumulate_select(g0, s, z, z, 0.0, 0.999)
    assert np.array_equal(send, r_acc != 0)
    # alpha >= B on a fresh state: nothing can be sent (Cauchy-Schwarz: g^2 <= B s)
    _, _, _, send = O.accumulate_select(g, s, z, z, float(B), 0.999)
    assert not send.any()
    # B = 1, alpha = 1, s fed as fl(g*g): r^2 == v bit for bit, strict test sends nothing
    _, _, _, send = O.accumulate_select(g, g * g, z, z, 1.0, 0.999)
    assert not send.any()
    # post-conditions
    r0 = rng.standard_normal(N).astype(F32) * F32(0.1)
    v0 = (rng.random(N) * 0.05).astype(F32)
    r_acc, r_out, v_out, send = O.accumulate_select(g, s, r0, v0, 1.0, 0.999)
    assert 0 < send.sum() < N
    assert np.array_equal(r_acc, r0 + g)
    assert not r_out[send].any() and not v_out[send].any()
    assert np.array_equal(r_out[~send], r_acc[~send])
    assert np.array_equal(v_out[~send], (F32(0.999) * (v0 + s))[~send])
    # mask is invariant under a power-of-two rescaling of the per-sample gradients
    _, _, _, send2 = O.accumulate_select(g * F32(4), s * F32(16), r0 * F32(4), v0 * F32(16), 1.0, 0.999)
    assert np.array_equal(send, send2)


def test_float32_single_rounding():
    """The test is evaluated in float32: an element that passes in exact arithmetic by
    less than a float32 ulp of r^2 is not sent."""
    r = F32(1.0) + F32(2.0 ** -23)                 # r^2 = 1 + 2^-22 + 2^-46 -> rounds to 1 + 2^-22
    v = F32(1.0) + F32(2.0 ** -22)
    _, _, _, send = O.accumulate_select([r], [v], [0], [0], 1.0, 0.999)
    assert float(r) ** 2 > float(v) and not send[0]
    z32 = F32(0.999)
    _, _, v_out, _ = O.accumulate_select([0.0], [3.0], [0], [0], 1.0, 0.999)
    assert v_out[0] == z32 * F32(3.0) and float(v_out[0]) != 0.999 * 3.0
