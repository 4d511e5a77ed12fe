"""Pins of the oracle's compressed index encoding (pack_compact / unpack_compact).  The paper only names the idea
(Section 4.2, last paragraph), so the format is this build's own; what pins the oracle is a hand-encoded example,
the round trip, the size bound against 32 bits per element, and the byte-level boundary cases of the code."""
import numpy as np
import pytest

from oracle import vgc_oracle as O
from paper_1802_06058_amd import workloads as W

U32 = np.uint32


def _words(idx, sign, d):
    return ((np.asarray(sign, np.uint64) << 31) | (np.asarray(d, np.uint64) << 28) | np.asarray(idx, np.uint64)).astype(U32)


def test_hand_encoded_example(golden):
    ex = golden("compact_index_example.txt")
    w = _words([int(x) for x in ex["indices"]], [int(x) for x in ex["signs"]], [int(x) for x in ex["d"]])
    stream, tile_bytes, run_offsets, hdrs = O.pack_compact(w, [(130, w.size, 0)], [(0, 5000)])
    assert stream.tolist() == [int(x) for x in ex["stream"]]
    assert tile_bytes.tolist() == [int(x) for x in ex["tile_bytes"]]
    assert run_offsets.tolist() == [int(x) for x in ex["run_offsets"]]
    assert hdrs == [(130, 7, 0)]
    w2, h2 = O.unpack_compact(stream, tile_bytes, run_offsets, hdrs, [(0, 5000)])
    assert np.array_equal(w2, w) and h2 == [(130, 7, 0)]


def test_one_or_two_bytes_at_the_gap_boundary():
    """gap 7 is the last one-byte gap, gap 8 the first two-byte one, gap 2047 the largest possible."""
    for gap, nbytes in [(0, 1), (7, 1), (8, 2), (255, 2), (2046, 2)]:
        w = _words([0, gap + 1], [0, 1], [2, 5])
        stream, tb, ro, h = O.pack_compact(w, [(127, 2, 0)], [(0, 2048)])
        assert stream.size == 1 + nbytes and tb.tolist() == [1 + nbytes]
        assert stream[0] == 0x02                                       # first element: gap 0, code 2
        if nbytes == 1:
            assert stream[1] == (gap << 4) | 13
        else:
            assert stream[1] == 0x80 | ((gap & 7) << 4) | 13 and stream[2] == gap >> 3
    w = _words([2047], [1], [7])                                       # a lone element at the tile's end: gap 2047
    stream, tb, ro, h = O.pack_compact(w, [(127, 1, 0)], [(0, 2048)])
    assert stream.tolist() == [0x80 | (7 << 4) | 15, 255]


@pytest.mark.parametrize("density", [0.0, 1e-4, 0.01, 0.2, 0.6, 1.0])
def test_round_trip_and_size_bound(density):
    rng = np.random.default_rng(int(density * 1e4) + 1)
    sizes = [2048 * 70 + 5, 3, 5000, 2048 * 130, 1, 2048]
    groups = W.groups_from_sizes(sizes)
    words, hdrs, off = [], [], 0
    for size in sizes:
        idx = np.flatnonzero(rng.random(size) < density)
        w = _words(idx, rng.integers(0, 2, idx.size), rng.integers(0, 8, idx.size))
        hdrs.append((int(rng.integers(1, 255)) if idx.size else 0, int(idx.size), off))
        words.append(w); off += idx.size
    words = np.concatenate(words)
    stream, tile_bytes, run_offsets, ch = O.pack_compact(words, hdrs, groups)
    tiles, run_first = O.compact_layout(groups)
    assert tile_bytes.size == len(tiles) and run_offsets.size == len(run_first)
    assert int(tile_bytes.astype(np.int64).sum()) == stream.size
    # never more than two bytes per element, never fewer than one; each tile's bytes fit 16 bits
    assert words.size <= stream.size <= 2 * words.size and int(tile_bytes.max(initial=0)) <= 2 * O.COMPACT_TILE
    # against 32 bits per element: smaller as soon as there is one element per tile on average
    if words.size >= len(tiles):
        assert stream.size + 2 * len(tiles) + 8 * len(run_first) <= 4 * words.size
    # group headers: same exponent and count, byte offsets chain
    assert [(e, c) for e, c, _ in ch] == [(e, c) for e, c, _ in hdrs]
    assert ch[0][2] == 0 and all(a[2] <= b[2] for a, b in zip(ch, ch[1:]))
    w2, h2 = O.unpack_compact(stream, tile_bytes, run_offsets, ch, groups)
    assert np.array_equal(w2, words) and h2 == hdrs
    # geometric gaps: the expected bytes per element are 2 - P(gap < 8) = 1 + (1 - density)^8
    if density in (0.2, 0.6) :
        assert abs(stream.size / words.size - (1 + (1 - density) ** 8)) < 0.02


def test_compact_message_decodes_to_the_same_dense_sum():
    """End to end on the oracle's own pipeline: select, pack, re-encode, decode the re-decoded words."""
    sizes = [2048 * 3 + 17, 4000]
    groups = W.groups_from_sizes(sizes)
    n = sum(sizes)
    rng = np.random.default_rng(3)
    g = (rng.standard_normal(n) * 0.01).astype(np.float32)
    s = (g.astype(np.float64) ** 2 * rng.uniform(0.2, 3, n)).astype(np.float32)
    z = np.zeros(n, np.float32)
    r_acc, _, _, send = O.accumulate_select(g, s, z, z, 1.0, 0.999)
    words, hdrs, _ = O.pack(r_acc, send, groups)
    w2, h2 = O.unpack_compact(*O.pack_compact(words, hdrs, groups), groups)
    a, b = np.zeros(n, np.float32), np.zeros(n, np.float32)
    O.unpack_add(words, hdrs, groups, 0.5, a)
    O.unpack_add(w2, h2, groups, 0.5, b)
    assert np.array_equal(a.view(U32), b.view(U32)) and a.any()
