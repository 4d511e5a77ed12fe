"""Pins for the oracle's quantiser and word packing (Section 4.2, Section 4.4, Appendix B)."""
import math

import numpy as np
import pytest

from oracle import vgc_oracle as O
from conftest import read_golden

F32 = np.float32
U32 = np.uint32


def test_appendix_b_worked_example():
    G = read_golden("appendix_b_quantisation.txt")
    x = np.array(G["inputs"], F32)
    assert float(np.abs(x).max()) == G["M_k"][0]
    E = O.floor_log2(np.abs(x).max())
    assert E == G["floor_log2_M_k"][0] and 2.0 ** E == G["pow2_floor_log2_M_k"][0]
    lq, keep = O.quantise_prose(np.abs(x), E)
    assert (2.0 ** lq).tolist() == G["rounded_magnitudes"]
    assert (E - lq).tolist() == G["d"]
    assert keep.astype(int).tolist() == G["sent_flags"]
    # the integer recipe gives the same codes
    ab = x.view(U32) & U32(0x7FFFFFFF)
    e_field, d, keep_b = O.quantise_bits(ab, E + 127)
    assert d.tolist() == G["d"] and keep_b.astype(int).tolist() == G["sent_flags"]
    # and the packed message is the paper's tuple
    words, hdrs, encoded = O.pack(x, np.ones(5, bool), [(0, 5)])
    assert hdrs == [(E + 127, 4, 0)]
    assert ((words >> U32(28)) & U32(7)).tolist() == G["sent_codes_d"]
    assert [(-1.0 if w >> 31 else 1.0) for w in words.tolist()] == G["sent_signed_codes_sign"]
    assert (words & U32(O.INDEX_MASK)).tolist() == G["sent_indices"]
    assert encoded.tolist() == [False, True, True, True, True]


def test_prose_equals_bit_recipe_exhaustive_binade():
    """Every float32 of one binade, against several group exponents."""
    mant = np.arange(1 << 23, dtype=np.uint32)
    for e_field, E_field in [(127, 127), (127, 128), (120, 127), (100, 108), (1, 5), (253, 254)]:
        ab = (U32(e_field) << U32(23)) | mant
        a = ab.view(F32).astype(np.float64)
        if e_field == E_field:                       # M_k itself lives in this binade
            pass
        lq, keep_p = O.quantise_prose(a, E_field - 127)
        ef, d, keep_b = O.quantise_bits(ab, E_field)
        assert np.array_equal(lq + 127, ef)
        assert np.array_equal(keep_p, keep_b)
        # rounding boundary is the linear midpoint 1.5 * 2^e, tie up
        up = ef > e_field
        if E_field > e_field:
            assert np.array_equal(up, mant >= (1 << 22))


def test_prose_equals_bit_recipe_random_exponents():
    rng = np.random.default_rng(0)
    ab = rng.integers(1 << 23, 255 << 23, size=200000, dtype=np.uint32)   # normal, finite
    a = ab.view(F32).astype(np.float64)
    E_field = int(ab.max() >> 23)
    lq, keep_p = O.quantise_prose(a, E_field - 127)
    ef, d, keep_b = O.quantise_bits(ab, E_field)
    assert np.array_equal(lq + 127, ef) and np.array_equal(keep_p, keep_b)


def _scalar_prose(a, E):
    """Independent scalar reading of Section 4.2 with math.log2-free arithmetic."""
    if a > 2.0 ** E:
        q = 2.0 ** E
    else:
        lo = 2.0 ** O.floor_log2(a)
        q = lo if (a - lo) < (2 * lo - a) else 2 * lo          # closer of the two; tie up
    d = E - int(round(math.log2(q)))
    return q, d


def test_scalar_prose_agrees_and_error_bounds():
    rng = np.random.default_rng(1)
    x = (rng.standard_normal(3000) * np.exp(rng.uniform(-6, 6, 3000))).astype(F32)
    x = x[x != 0]
    E = O.floor_log2(np.abs(x).max())
    lq, keep = O.quantise_prose(np.abs(x), E)
    for a, l, k in zip(np.abs(x).astype(np.float64), lq, keep):
        q, d = _scalar_prose(a, E)
        assert q == 2.0 ** l and (d <= 7) == bool(k)
        if a > 2.0 ** E:
            assert abs(q - a) < a / 2                               # truncated to 2^E
        else:
            assert abs(q - a) <= a / 3 * (1 + 1e-15)                # rounded to a neighbour
        if not k:
            assert a < 1.5 * 2.0 ** (E - 8)                         # what is rounded to zero is tiny
    assert lq[np.argmax(np.abs(x))] == E                            # the maximum always gets d = 0


def test_pack_structure_multi_group():
    rng = np.random.default_rng(2)
    sizes = [1000, 1, 37, 5000, 64]
    groups, off = [], 0
    for s in sizes:
        groups.append((off, s)); off += s
    N = off
    r_acc = (rng.standard_normal(N) * np.exp(rng.uniform(-8, 2, N))).astype(F32)
    send = rng.random(N) < 0.4
    send[1000] = False                                              # the 1-element group sends nothing
    send[1001:1038] = False                                         # and so does the next
    words, hdrs, encoded = O.pack(r_acc, send, groups)
    assert hdrs[1] == (0, 0, hdrs[0][1]) and hdrs[2][:2] == (0, 0)
    assert sum(h[1] for h in hdrs) == words.size == encoded.sum()
    assert not encoded[~send].any()
    pos = 0
    for (o, s), (E_field, cnt, woff) in zip(groups, hdrs):
        assert woff == pos
        w = words[pos:pos + cnt]; pos += cnt
        if cnt == 0:
            continue
        idx = (w & U32(O.INDEX_MASK)).astype(np.int64)
        assert np.all(np.diff(idx) > 0) and idx.max() < s            # ascending, local, in range
        assert np.array_equal(np.flatnonzero(encoded[o:o + s]), idx)
        sent_abs = np.abs(r_acc[o:o + s][send[o:o + s]])
        M = float(sent_abs.max())
        assert E_field - 127 == O.floor_log2(M)
        d = ((w >> U32(28)) & U32(7)).astype(np.int64)
        assert d.min() == 0                                          # the maximum is in the message
        sign = (w >> U32(31)).astype(bool)
        assert np.array_equal(sign, r_acc[o:o + s][idx] < 0)
        # kept <=> rounded magnitude >= 2^(E-7)
        lq, _ = O.quantise_prose(sent_abs, E_field - 127)
        assert (lq >= E_field - 127 - 7).sum() == cnt
    # deterministic
    words2, hdrs2, _ = O.pack(r_acc, send, groups)
    assert np.array_equal(words, words2) and hdrs == hdrs2


def test_max_over_reading_flag():
    """M_k over the sent elements (shipped reading) vs over the whole group."""
    r_acc = np.array([100.0, 1.0, 0.5, 0.004], F32)
    send = np.array([False, True, True, True])
    w_sent, h_sent, _ = O.pack(r_acc, send, [(0, 4)], max_over="sent")
    w_all, h_all, _ = O.pack(r_acc, send, [(0, 4)], max_over="all")
    assert h_sent[0][0] == 127 and h_sent[0][1] == 2                # 0.004 -> 2^-8: d = 8, rounded to zero
    assert h_all[0][0] == 133 and h_all[0][1] == 2                  # 2^6: 1.0 has d=6, 0.5 d=7, 0.004 dropped
    assert ((w_all >> U32(28)) & U32(7)).tolist() == [6, 7]


def test_subnormals_and_empty():
    tiny = np.array([1e-45, 3e-39, -5e-39], F32)                   # all subnormal
    words, hdrs, enc = O.pack(tiny, np.ones(3, bool), [(0, 3)])
    assert words.size == 0 and hdrs == [(0, 0, 0)] and not enc.any()
    mixed = np.array([2.0 ** -120, 2.0 ** -126, 1.2e-38, 1e-40], F32)   # E field 7; 2^-126 has field 1: d=6
    words, hdrs, enc = O.pack(mixed, np.ones(4, bool), [(0, 4)])
    assert hdrs[0][0] == 7
    assert ((words >> U32(28)) & U32(7)).tolist() == [0, 6, 6]     # 1.2e-38 (> 2^-126.5..) rounds to 2^-126
    assert enc.tolist() == [True, True, True, False]
    words, hdrs, enc = O.pack(np.ones(4, F32), np.zeros(4, bool), [(0, 4)])
    assert words.size == 0 and hdrs == [(0, 0, 0)]
