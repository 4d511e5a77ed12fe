"""Pins for the oracle's decode + sum (Section 4.3) and the whole-step invariants."""
import numpy as np

from oracle import vgc_oracle as O

F32 = np.float32
U32 = np.uint32


def _state(rng, N):
    g = (rng.standard_normal(N) * 0.1).astype(F32)
    s = ((rng.random(N) * 0.02) + g.astype(np.float64) ** 2 / 8).astype(F32)
    r = (rng.standard_normal(N) * 0.05).astype(F32)
    v = (rng.random(N) * 0.01).astype(F32)
    return g, s, r, v


def test_decode_hand_built_words():
    # exp_field 130 (2^3): d=0 -> 8, d=2 -> 2 ; negative sign bit
    w = np.array([(0 << 31) | (0 << 28) | 5, (1 << 31) | (2 << 28) | 9], dtype=np.uint64).astype(U32)
    idx, val = O.decode_words(w, 130)
    assert idx.tolist() == [5, 9] and val.tolist() == [8.0, -2.0]
    out = np.zeros(12, F32); out[5] = 1.0
    O.unpack_add(w, [(130, 2, 0)], [(0, 12)], 0.5, out)
    assert out[5] == 5.0 and out[9] == -1.0 and np.count_nonzero(out) == 2


def test_round_trip_and_conservation():
    rng = np.random.default_rng(0)
    sizes = [3000, 17, 4096, 1]
    groups, off = [], 0
    for sz in sizes:
        groups.append((off, sz)); off += sz
    N = off
    g, s, r, v = _state(rng, N)
    r_acc, r_out, v_out, send = O.accumulate_select(g, s, r, v, 1.0, 0.999)
    assert 0.1 < send.mean() < 0.9
    words, hdrs, encoded = O.pack(r_acc, send, groups)
    dense = np.zeros(N, F32)
    O.unpack_add(words, hdrs, groups, 1.0, dense)
    # (ii) equals the dense quantised vector of the prose quantiser
    expect = np.zeros(N, np.float64)
    for (o, sz), (Ef, cnt, _) in zip(groups, hdrs):
        m = send[o:o + sz]
        if not m.any() or cnt == 0:
            continue
        a = np.abs(r_acc[o:o + sz][m].astype(np.float64))
        lq, keep = O.quantise_prose(a, O.floor_log2(a.max()))
        q = np.where(keep, np.sign(r_acc[o:o + sz][m]) * 2.0 ** lq, 0.0)
        expect[o:o + sz][m] = q
    assert np.array_equal(dense.astype(np.float64), expect)
    # (iii) per-element conservation: decoded + retained residual vs accumulated value
    ra = r_acc.astype(np.float64)
    dd = dense.astype(np.float64)
    unsent = ~send
    assert not dd[unsent].any() and np.array_equal(r_out[unsent], r_acc[unsent])
    kept = encoded
    assert not r_out[send].any() and not v_out[send].any()
    for (o, sz), (Ef, cnt, _) in zip(groups, hdrs):
        if cnt == 0:
            continue
        top = 2.0 ** (Ef - 127)
        k = kept[o:o + sz]
        x, y = ra[o:o + sz][k], dd[o:o + sz][k]
        clipped = np.abs(x) > top
        assert np.all(np.abs(y - x)[~clipped] <= np.abs(x)[~clipped] / 3 * (1 + 1e-12))
        assert np.all(np.abs(y - x)[clipped] < np.abs(x)[clipped] / 2)
        dropped = send[o:o + sz] & ~k
        assert np.all(np.abs(ra[o:o + sz][dropped]) < 1.5 * top / 256)
        assert not dd[o:o + sz][dropped].any()


def test_messages_apply_in_order_and_mean_of_identical_messages():
    rng = np.random.default_rng(1)
    N = 5000
    groups = [(0, 2000), (2000, 3000)]
    msgs = []
    for w in range(4):
        g, s, r, v = _state(rng, N)
        r_acc, _, _, send = O.accumulate_select(g, s, r, v, 1.0, 0.999)
        words, hdrs, _ = O.pack(r_acc, send, groups)
        msgs.append((words, hdrs))
    out = (rng.standard_normal(N)).astype(F32)
    expect = out.copy()
    for words, hdrs in msgs:
        O.unpack_add(words, hdrs, groups, 0.25, out)
    # literal per-word loop, in message order then word order
    for words, hdrs in msgs:
        for (o, sz), (Ef, cnt, woff) in zip(groups, hdrs):
            for w in words[woff:woff + cnt].tolist():
                i = w & 0x0FFFFFFF
                val = (-1.0 if w >> 31 else 1.0) * 2.0 ** (Ef - ((w >> 28) & 7) - 127)
                expect[o + i] = F32(expect[o + i] + F32(F32(0.25) * F32(val)))
    assert np.array_equal(out, expect)
    # p identical messages at scale 1/p == one message at scale 1 (p a power of two)
    a = np.zeros(N, F32); b = np.zeros(N, F32)
    for _ in range(8):
        O.unpack_add(msgs[0][0], msgs[0][1], groups, 1 / 8, a)
    O.unpack_add(msgs[0][0], msgs[0][1], groups, 1.0, b)
    assert np.array_equal(a, b)
