"""Pins for the oracle's per-parameter sums (Alg. 1: g = sum grad/B, s = sum (grad/B)^2).

None of these goes through the oracle's own formula: hand-computed values, closed forms,
brute force over materialised per-sample gradients, and a library einsum.
"""
import numpy as np
import pytest

from oracle import vgc_oracle as O
from conftest import read_golden


def test_hand_computed_fc_and_conv():
    G = read_golden("hand_computed_statistic.txt")
    for fn in (O.sqgrad_bruteforce_fc, O.sqgrad_fc):
        g, s = fn([[1.0], [2.0]], [[3.0], [4.0]], 0.5)
        assert g.ravel().tolist() == G["fc1_g"] and s.ravel().tolist() == G["fc1_s"]
        g, s = fn([[1.0, 2.0]], [[3.0, 5.0, 7.0]], 1.0)
        assert g.shape == (2, 3)
        assert g.ravel().tolist() == G["fc2_g"] and s.ravel().tolist() == G["fc2_s"]
    U = np.array([[[1.0], [2.0]], [[3.0], [4.0]]])
    D = np.array([[[1.0], [1.0]], [[2.0], [-1.0]]])
    for fn in (O.sqgrad_bruteforce_conv, O.sqgrad_conv):
        g, s = fn(U, D, 0.5)
        assert g.ravel().tolist() == G["conv1_g"] and s.ravel().tolist() == G["conv1_s"]


def test_closed_form_all_ones():
    B, P, J, C, c = 3, 5, 4, 2, 0.25
    g, s = O.sqgrad_fc(np.ones((B, J)), np.ones((B, C)), c)
    assert np.all(g == c * B) and np.all(s == c * c * B)
    g, s = O.sqgrad_conv(np.ones((B, P, J)), np.ones((B, P, C)), c)
    assert np.all(g == c * B * P) and np.all(s == c * c * B * P * P)


@pytest.mark.parametrize("B,J,C", [(1, 3, 2), (4, 8, 5), (3, 1, 7)])
def test_fc_matches_bruteforce(B, J, C):
    rng = np.random.default_rng(B * 100 + J * 10 + C)
    X, D = rng.standard_normal((B, J)), rng.standard_normal((B, C))
    gb, sb = O.sqgrad_bruteforce_fc(X, D, 1.0 / B)
    g, s = O.sqgrad_fc(X, D, 1.0 / B)
    np.testing.assert_allclose(g, gb, rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(s, sb, rtol=1e-13, atol=1e-15)


@pytest.mark.parametrize("B,P,J,C", [(1, 1, 2, 3), (4, 5, 8, 3), (2, 3, 1, 6)])
def test_conv_matches_bruteforce_and_einsum(B, P, J, C):
    rng = np.random.default_rng(B * 1000 + P * 100 + J * 10 + C)
    U, D = rng.standard_normal((B, P, J)), rng.standard_normal((B, P, C))
    c = 1.0 / B
    gb, sb = O.sqgrad_bruteforce_conv(U, D, c)
    g, s = O.sqgrad_conv(U, D, c)
    np.testing.assert_allclose(g, gb, rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(s, sb, rtol=1e-13, atol=1e-15)
    per_sample = np.einsum("zpj,zpc->zjc", U, D) * c          # library routine, then square-sum
    np.testing.assert_allclose(g, per_sample.sum(0), rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(s, (per_sample ** 2).sum(0), rtol=1e-13, atol=1e-15)


def test_conv_with_one_position_is_fc():
    rng = np.random.default_rng(5)
    X, D = rng.standard_normal((6, 7)), rng.standard_normal((6, 4))
    g1, s1 = O.sqgrad_fc(X, D, 1 / 6)
    g2, s2 = O.sqgrad_conv(X[:, None, :], D[:, None, :], 1 / 6)
    np.testing.assert_allclose(g1, g2, rtol=1e-14)
    np.testing.assert_allclose(s1, s2, rtol=1e-14)


def test_conv_cross_terms_are_kept():
    """The square is of the per-sample gradient (sum over positions first), so treating
    every position as a sample must NOT give the same answer."""
    rng = np.random.default_rng(7)
    U, D = rng.standard_normal((3, 4, 5)), rng.standard_normal((3, 4, 2))
    _, s = O.sqgrad_conv(U, D, 1.0)
    wrong = (U.reshape(12, 5) ** 2).T @ (D.reshape(12, 2) ** 2)
    assert np.abs(s - wrong).max() > 1e-3


def test_single_sample_square_and_cauchy_schwarz_and_scaling():
    rng = np.random.default_rng(11)
    X, D = rng.standard_normal((1, 9)), rng.standard_normal((1, 4))
    g, s = O.sqgrad_fc(X, D, 1.0)
    np.testing.assert_allclose(s, g * g, rtol=1e-14)
    B = 8
    U, D = rng.standard_normal((B, 3, 6)), rng.standard_normal((B, 3, 5))
    g, s = O.sqgrad_conv(U, D, 1.0 / B)
    assert np.all(s >= 0) and np.all(g * g <= B * s * (1 + 1e-12))
    g2, s2 = O.sqgrad_conv(U, 2.0 * D, 1.0 / B)                 # power-of-two scaling is exact
    assert np.array_equal(g2, 2.0 * g) and np.array_equal(s2, 4.0 * s)
    gz, sz = O.sqgrad_conv(U, 0.0 * D, 1.0 / B)
    assert not gz.any() and not sz.any()


def test_bf16_inputs_widen_exactly():
    from paper_1802_06058_amd import workloads as W
    x = np.array([1.0, 1.00390625, -3.140625, 1e-3], np.float32)
    b = W.f32_to_bf16_bits(x)
    back = W.bf16_bits_to_f32(b)
    assert back[0] == 1.0 and back[2] == -3.140625
    assert back[1] == 1.0                       # 1 + 2^-8 is a tie between 1 and 1+2^-7: to even
    assert abs(back[3] - 1e-3) <= 1e-3 * 2.0 ** -8
