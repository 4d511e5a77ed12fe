"""The compressed index format on the GPU (vgc_pack_compact, vgc_unpack_compact_add_batch) against the oracle:
stream bytes, per-tile byte counts, run offsets and headers bit for bit; decoded dense sums bit for bit equal to the
oracle's decode of the plain message, messages in order."""
import numpy as np
import pytest

from oracle import vgc_oracle as O
from paper_1802_06058_amd import workloads as W
from streams import sample_stream

pytestmark = pytest.mark.gpu

F32 = np.float32
U32 = np.uint32


@pytest.fixture(scope="module")
def dev():
    import torch
    from paper_1802_06058_amd import vgc
    assert torch.cuda.is_available()
    vgc.load()
    return torch.device("cuda:0")


def _dev(a, dev):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).to(dev)


def _bits(a):
    return np.ascontiguousarray(a).view(U32)


class CompactMessage:
    def __init__(self, plan, dev, cap):
        import torch
        self.stream = torch.full((cap + 64,), 0xEE, dtype=torch.uint8, device=dev)         # 64 canary bytes
        self.cap = cap
        self.tile_bytes = torch.full((plan.n_tiles,), -1, dtype=torch.int16, device=dev)
        self.run_offsets = torch.full((plan.n_runs,), -1, dtype=torch.int64, device=dev)
        self.hdrs, self.status = plan.new_headers(), plan.new_status()


def _select(plan, g, s, alpha, dev):
    import torch
    from paper_1802_06058_amd import vgc
    n = plan.n
    r = torch.zeros(n, dtype=torch.float32, device=dev); v = torch.zeros(n, dtype=torch.float32, device=dev)
    scratch = plan.new_scratch()
    vgc.accumulate_select(_dev(g, dev), _dev(s, dev), r, v, plan, alpha, 0.999, scratch)
    return scratch


def _oracle_message(g, s, groups, alpha):
    z = np.zeros(g.size, F32)
    r_acc, _, _, send = O.accumulate_select(g, s, z, z, alpha, 0.999)
    words, hdrs, _ = O.pack(r_acc, send, groups)
    return words, hdrs


GROUP_SETS = {
    "mixed": [1000, 1, 37, 5000, 64, 2048, 4099, 3, 6144, 10],
    "runs": [2048 * 70 + 5, 3, 5000, 2048 * 130, 1],
    "one_partial": [777],
}


@pytest.mark.parametrize("name", list(GROUP_SETS))
@pytest.mark.parametrize("alpha", [0.0, 1.0, 4.0, 12.0])
def test_pack_compact_matches_oracle(dev, name, alpha):
    import torch
    from paper_1802_06058_amd import vgc
    sizes = GROUP_SETS[name]
    groups = W.groups_from_sizes(sizes)
    plan = vgc.Plan(groups, dev)
    n = plan.n
    g, s = sample_stream(71, (len(name), int(alpha)), n, 16, "student", sigma=0.01)
    if name == "runs":
        g[: 2048 * 3] = 0                                      # leading tiles without any element
    scratch = _select(plan, g, s, alpha, dev)
    words, hdrs = _oracle_message(g, s, groups, alpha)
    stream, tile_bytes, run_offsets, chdrs = O.pack_compact(words, hdrs, groups)
    msg = CompactMessage(plan, dev, 2 * n)
    vgc.pack_compact(plan, scratch, msg.stream[:msg.cap], msg.tile_bytes, msg.run_offsets, msg.hdrs, msg.status)
    # the plain encoder reads the same staged result, before or after
    plain = torch.empty(n, dtype=torch.int32, device=dev)
    ph, ps = plan.new_headers(), plan.new_status()
    vgc.pack(plan, scratch, plain, ph, ps)
    torch.cuda.synchronize()
    total, overflow = vgc.read_status(msg.status)
    assert overflow == 0 and total == stream.size
    got = msg.stream.cpu().numpy()
    assert np.array_equal(got[:total], stream)
    assert np.all(got[msg.cap:] == 0xEE)
    assert np.array_equal(msg.tile_bytes.cpu().numpy().view(np.uint16), tile_bytes)
    assert np.array_equal(msg.run_offsets.cpu().numpy().view(np.uint64), run_offsets)
    assert vgc.read_headers(msg.hdrs) == chdrs
    assert vgc.read_status(ps) == (words.size, 0) and np.array_equal(plain[:words.size].cpu().numpy().view(U32), words)
    if words.size >= plan.n_tiles:
        assert total + 2 * plan.n_tiles + 8 * plan.n_runs <= 4 * words.size


def test_pack_compact_capacity_overflow_is_reported_not_written(dev):
    from paper_1802_06058_amd import vgc
    import torch
    groups = W.groups_from_sizes([2048 * 5 + 9, 3000])
    plan = vgc.Plan(groups, dev)
    g, s = sample_stream(72, (0,), plan.n, 16, "normal", sigma=0.1)
    scratch = _select(plan, g, s, 1.0, dev)
    stream = O.pack_compact(*_oracle_message(g, s, groups, 1.0), groups)[0]
    cap = stream.size // 2
    msg = CompactMessage(plan, dev, cap)
    vgc.pack_compact(plan, scratch, msg.stream[:cap], msg.tile_bytes, msg.run_offsets, msg.hdrs, msg.status)
    torch.cuda.synchronize()
    assert vgc.read_status(msg.status) == (stream.size, 1)
    got = msg.stream.cpu().numpy()
    assert np.array_equal(got[:cap], stream[:cap]) and np.all(got[cap:] == 0xEE)


@pytest.mark.parametrize("p,overwrite", [(0, True), (1, False), (3, True), (8, False), (11, True)])
def test_unpack_compact_batch_equals_plain_decode_in_order(dev, p, overwrite):
    import torch
    from paper_1802_06058_amd import vgc
    sizes = [2048 * 70 + 5, 3, 5000, 2048 * 130, 1]
    groups = W.groups_from_sizes(sizes)
    plan = vgc.Plan(groups, dev)
    n = plan.n
    rng = np.random.default_rng(p)
    dense0 = rng.standard_normal(n).astype(F32)
    expect = np.zeros(n, F32) if overwrite else dense0.copy()
    dense = _dev(dense0, dev)
    scale = 1.0 / 3.0
    msgs, nbytes = [], []
    for w in range(p):
        g, s = sample_stream(73, (p, w), n, 16, "student", sigma=10.0 ** rng.uniform(-3, 0))
        alpha = [0.0, 1.0, 4.0, 12.0][w % 4]
        if w == 2:
            g[: 2048 * 70 + 5] = 0                             # a whole group absent from this message
        words, hdrs = _oracle_message(g, s, groups, alpha)
        O.unpack_add(words, hdrs, groups, scale, expect)
        # the GPU's own encoder makes the message (checked against the oracle's bytes above)
        scratch = _select(plan, g, s, alpha, dev)
        msg = CompactMessage(plan, dev, 2 * n)
        vgc.pack_compact(plan, scratch, msg.stream[:msg.cap], msg.tile_bytes, msg.run_offsets, msg.hdrs, msg.status)
        torch.cuda.synchronize()
        total, _ = vgc.read_status(msg.status)
        assert total == O.pack_compact(words, hdrs, groups)[0].size
        msgs.append(msg); nbytes.append(total)
    vgc.unpack_compact_add_batch([m.stream for m in msgs], nbytes, [m.tile_bytes for m in msgs], [m.run_offsets for m in msgs],
                                 [m.hdrs for m in msgs], plan, scale, dense, overwrite=overwrite)
    torch.cuda.synchronize()
    got = dense.cpu().numpy()
    assert np.array_equal(_bits(got), _bits(expect)), f"{np.flatnonzero(_bits(got) != _bits(expect))[:10]}"


def test_unpack_compact_from_oracle_bytes_with_long_gaps(dev):
    """A hand-made sparse message straight from the oracle's encoder: two-byte elements across the 64-byte rounds of
    the decoder (an element's first byte in lane 63), an element at the last position of a partial tile."""
    import torch
    from paper_1802_06058_amd import vgc
    sizes = [2048 * 2 + 100, 2048]
    groups = W.groups_from_sizes(sizes)
    plan = vgc.Plan(groups, dev)
    n = plan.n
    idx0 = np.concatenate([np.arange(0, 2048, 9), 2048 + np.arange(0, 2048, 31), [4096 + 99]])   # gaps of 8 and 30: two bytes each
    idx1 = np.array([0, 1, 2, 2047])
    mk = lambda idx, seed: ((np.random.default_rng(seed).integers(0, 16, idx.size).astype(np.uint64) << 28) | idx.astype(np.uint64)).astype(U32)
    words = np.concatenate([mk(idx0, 1), mk(idx1, 2)])
    hdrs = [(140, idx0.size, 0), (100, idx1.size, idx0.size)]
    stream, tile_bytes, run_offsets, chdrs = O.pack_compact(words, hdrs, groups)
    assert stream.size > 2 * 64 and tile_bytes[0] == 2 * 228 - 1
    expect = np.zeros(n, F32)
    O.unpack_add(words, hdrs, groups, 0.25, expect)
    dense = torch.zeros(n, dtype=torch.float32, device=dev)
    vgc.unpack_compact_add_batch([_dev(stream, dev)], [stream.size], [_dev(tile_bytes.view(np.int16), dev)],
                                 [_dev(run_offsets.view(np.int64), dev)],
                                 [_dev(np.array(chdrs, dtype=vgc.HDR_DTYPE).view(np.uint8), dev)], plan, 0.25, dense, overwrite=True)
    torch.cuda.synchronize()
    assert np.array_equal(_bits(dense.cpu().numpy()), _bits(expect))
