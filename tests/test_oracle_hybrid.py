"""Pins for the oracle's hybrid step (Alg. 2, Section 4.5)."""
import numpy as np

from oracle import vgc_oracle as O
from conftest import read_golden

F32 = np.float32


def test_hand_computed_hybrid_step():
    G = read_golden("hand_computed_statistic.txt")
    r_out, v_out, send, sign = O.accumulate_select_hybrid(
        [2, 0.25, -1, 0.25], [1, 0.01, 0.5, 0.0625], [0, 0, -1, 0.25], [0, 0, 1, 0], alpha=1.0, zeta=0.5, tau=0.5)
    assert send.astype(int).tolist() == G["hybrid_send"] and sign.tolist() == G["hybrid_sign"]
    assert r_out.tolist() == G["hybrid_r_out"]
    np.testing.assert_allclose(v_out, np.array(G["hybrid_v_out"], F32), rtol=1e-7)


def test_square_completion_identity():
    """Section 4.5: the correction turns a^2 into (a - b)^2.  With a single sample (v = r^2 exactly,
    powers of two so every operation is exact) the corrected v equals the square of what is left in r."""
    r0 = np.array([4.0, -8.0, 2.0, -0.5, 16.0], F32)
    tau = 1.0
    z = np.zeros(5, F32)
    r_out, v_out, send, sign = O.accumulate_select_hybrid(r0, r0 * r0, z, z, alpha=0.5, zeta=1.0, tau=tau)
    assert send.tolist() == [True, True, True, False, True]
    assert np.array_equal(r_out[send], (r0 - np.sign(r0) * F32(tau))[send])
    assert np.array_equal(v_out[send], (r_out * r_out)[send])
    assert r_out[3] == r0[3] and v_out[3] == r0[3] * r0[3]
    # the other reading of |r| (after the subtraction) is different: v - 2(|a|-tau)tau + tau^2
    _, v_alt, _, _ = O.accumulate_select_hybrid(r0, r0 * r0, z, z, alpha=0.5, zeta=1.0, tau=tau, abs_r="after")
    assert not np.array_equal(v_alt[send], v_out[send])


def test_reduces_to_threshold_method_and_is_stricter_than_basic():
    rng = np.random.default_rng(0)
    n = 20000
    g = (rng.standard_normal(n) * 0.02).astype(F32)
    s = (rng.random(n) * 1e-4).astype(F32)
    r = (rng.standard_normal(n) * 0.02).astype(F32)
    v = (rng.random(n) * 1e-4).astype(F32)
    tau = 0.03
    # alpha = 0: the variance test always passes for non-zero r, leaving the threshold method of
    # Section 3: send when the accumulated value exceeds the threshold, keep the remainder
    r_out, v_out, send, sign = O.accumulate_select_hybrid(g, s, r, v, 0.0, 0.999, tau)
    acc = r + g
    assert np.array_equal(send, np.abs(acc) > F32(tau))
    assert np.array_equal(r_out[send], (acc - np.sign(acc) * F32(tau))[send]) and np.array_equal(r_out[~send], acc[~send])
    assert np.all(np.abs(r_out[send]) < np.abs(acc[send]))
    # alpha = 1: the hybrid mask is the basic mask restricted to |r| > tau; unsent state decays as in Alg. 1
    r_out, v_out, send_h, _ = O.accumulate_select_hybrid(g, s, r, v, 1.0, 0.999, tau)
    _, r_b, v_b, send_b = O.accumulate_select(g, s, r, v, 1.0, 0.999)
    assert np.array_equal(send_h, send_b & (np.abs(acc) > F32(tau)))
    both_unsent = ~send_h & ~send_b
    assert np.array_equal(r_out[both_unsent], r_b[both_unsent]) and np.array_equal(v_out[both_unsent], v_b[both_unsent])
    assert np.all(v_out >= 0)
    # tau huge: nothing is sent, and v still decays every step
    _, v_none, send_none, _ = O.accumulate_select_hybrid(g, s, r, v, 1.0, 0.999, 1e9)
    assert not send_none.any() and np.array_equal(v_none, F32(0.999) * (v + s))


def test_pack_hybrid_words_decode_to_tau_signs():
    rng = np.random.default_rng(1)
    sizes = [300, 1, 700]
    groups, off = [], 0
    for sz in sizes:
        groups.append((off, sz)); off += sz
    n = off
    sign = np.zeros(n, F32)
    send = rng.random(n) < 0.3
    send[300] = False
    sign[send] = np.where(rng.random(send.sum()) < 0.5, -1, 1)
    words, hdrs = O.pack_hybrid(sign, send, groups)
    assert hdrs[1][:2] == (0, 0) and hdrs[0][0] == 127 and sum(h[1] for h in hdrs) == words.size == send.sum()
    assert not (words & np.uint32(0x70000000)).any()            # exponent code 0 everywhere
    tau = 0.125
    dense = np.zeros(n, F32)
    O.unpack_add(words, hdrs, groups, tau, dense)
    assert np.array_equal(dense, sign * F32(tau))
