"""Parity of the HIP accumulate/select, pack and unpack-add path against the CPU oracle,
through the C ABI.  Bit-exact: mask, state, headers, words, decoded sums."""
import numpy as np
import pytest

from oracle import vgc_oracle as O
from paper_1802_06058_amd import workloads as W
from streams import device_student_stream, sample_stream

pytestmark = pytest.mark.gpu

F32 = np.float32
U32 = np.uint32


@pytest.fixture(scope="module")
def dev():
    import torch
    from paper_1802_06058_amd import vgc
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    vgc.load()
    return torch.device("cuda:0")


def _dev(a, dev):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).to(dev)


def _bits(a):
    return np.ascontiguousarray(a).view(U32)


class GpuWorker:
    """r, v state + scratch + message buffers of one simulated worker on the GPU."""

    def __init__(self, groups, dev, words_cap=None, r0=None, v0=None):
        import torch
        from paper_1802_06058_amd import vgc
        self.vgc = vgc
        self.plan = vgc.Plan(groups, dev)
        n = self.plan.n
        self.r = torch.zeros(n, dtype=torch.float32, device=dev) if r0 is None else _dev(r0, dev)
        self.v = torch.zeros(n, dtype=torch.float32, device=dev) if v0 is None else _dev(v0, dev)
        self.scratch = self.plan.new_scratch()
        self.scratch.fill_(0xAB)                               # stale garbage must not matter
        self.cap = n if words_cap is None else words_cap
        self.words = torch.full((self.cap + 64,), -1, dtype=torch.int32, device=dev)   # 64 canary words
        self.hdrs = self.plan.new_headers()
        self.status = self.plan.new_status()

    def step(self, g, s, alpha, zeta):
        import torch
        vgc = self.vgc
        vgc.accumulate_select(g, s, self.r, self.v, self.plan, alpha, zeta, self.scratch)
        mask = self.plan.send_mask(self.scratch)
        vgc.pack(self.plan, self.scratch, self.words[:self.cap], self.hdrs, self.status)
        torch.cuda.synchronize()
        total, overflow = vgc.read_status(self.status)
        hdrs = vgc.read_headers(self.hdrs)
        words = self.words.cpu().numpy().view(U32)
        assert np.all(words[self.cap:] == 0xFFFFFFFF), "wrote past words_cap"
        return mask, hdrs, words[:min(total, self.cap)].copy(), total, overflow


def _compare_step(gw, g, s, r, v, groups, alpha, zeta, dev):
    r_acc, r_out, v_out, send = O.accumulate_select(g, s, r, v, alpha, zeta)
    words, hdrs, _ = O.pack(r_acc, send, groups)
    mask, ghdrs, gwords, total, overflow = gw.step(_dev(g, dev), _dev(s, dev), alpha, zeta)
    assert np.array_equal(mask, send), f"mask differs at {np.flatnonzero(mask != send)[:10]}"
    assert np.array_equal(_bits(gw.r.cpu().numpy()), _bits(r_out))
    assert np.array_equal(_bits(gw.v.cpu().numpy()), _bits(v_out))
    assert ghdrs == hdrs
    assert total == words.size and overflow == 0
    assert np.array_equal(gwords, words)
    return r_out, v_out, send, words, hdrs


GROUP_SETS = {
    "one_aligned": [4 * 2048],
    "one_ragged": [5 * 2048 + 777],
    "tiny": [1],
    "mixed": [1000, 1, 37, 5000, 64, 2048, 4099, 3, 6144, 10],
    "odd_offsets": [3, 2048 * 3, 5, 2048 * 2 + 1, 8192],
}


@pytest.mark.parametrize("name", list(GROUP_SETS))
@pytest.mark.parametrize("alpha", [1.0, 2.0])
def test_step_matches_oracle(dev, name, alpha):
    groups = W.groups_from_sizes(GROUP_SETS[name])
    n = sum(GROUP_SETS[name])
    rng = np.random.default_rng(len(name) * 7 + int(alpha))
    g, s = sample_stream(11, (len(name), int(alpha)), n, 16, "student", sigma=0.01)
    r = (rng.standard_normal(n) * 0.003).astype(F32)
    v = (rng.random(n) * 1e-5).astype(F32)
    gw = GpuWorker(groups, dev, r0=r, v0=v)
    _compare_step(gw, g, s, r, v, groups, alpha, 0.999, dev)


def test_wide_dynamic_range_exercises_shift_and_drop(dev):
    """Magnitudes spread over 2^24 inside one group: tile exponents differ from the group's,
    many sent elements fall below 2^(E-7) and are rounded to zero, some are subnormal."""
    sizes = [2048 * 6 + 5, 2048 * 3, 100]
    groups = W.groups_from_sizes(sizes)
    n = sum(sizes)
    rng = np.random.default_rng(5)
    mag = np.exp2(rng.uniform(-24, 0, n))
    mag[: 2048 * 2] *= 2.0 ** -12                              # whole tiles far below the group's maximum
    g = (rng.standard_normal(n) * mag).astype(F32)
    g[2048 * 6 + 5: 2048 * 6 + 5 + 300] = (rng.standard_normal(300) * 1e-39).astype(F32)   # subnormal accumulations
    s = (g.astype(np.float64) ** 2 * rng.uniform(0.2, 3.0, n)).astype(F32)
    z = np.zeros(n, F32)
    gw = GpuWorker(groups, dev)
    r_out, v_out, send, words, hdrs = _compare_step(gw, g, s, z, z, groups, 1.0, 0.999, dev)
    assert 0.2 < send.mean() < 0.9
    assert words.size < send.sum()                             # something was rounded to zero
    d = (words >> U32(28)) & U32(7)
    assert set(np.unique(d).tolist()) == set(range(8))


def test_group_of_several_scan_segments(dev):
    """A group larger than one scan segment (8192 tiles): E_k comes from the last segment, the first
    segment lies partly below 2^(E_k-7) and the middle one wholly, so segment totals of zero, the
    segment bases and the shift all matter; a one-tile group before and after."""
    S = 8192 * 2048
    sizes = [700, 2 * S + 3 * 2048 + 5, 2048]
    groups = W.groups_from_sizes(sizes)
    n = sum(sizes)
    rng = np.random.default_rng(21)
    g = rng.standard_normal(n, dtype=F32)
    scale = np.ones(n, F32)
    scale[700:700 + S] = 2.0 ** -6
    scale[700 + S:700 + 2 * S] = 2.0 ** -14
    g *= scale
    g[700 + 2 * S + 4000] = 3.0                                # group maximum in the short last segment
    s = (g.astype(np.float64) ** 2 * rng.uniform(0.2, 3.0, n)).astype(F32)
    del scale
    z = np.zeros(n, F32)
    gw = GpuWorker(groups, dev)
    r_out, v_out, send, words, hdrs = _compare_step(gw, g, s, z, z, groups, 1.0, 0.999, dev)
    idx = (words[hdrs[1][2]:hdrs[1][2] + hdrs[1][1]] & U32(0x0FFFFFFF)).astype(np.int64)
    assert hdrs[1][1] > 0 and (idx < S).any() and not ((idx >= S) & (idx < 2 * S)).any() and (idx >= 2 * S).any()


def test_alpha_extremes_and_ties(dev):
    sizes = [3000, 5000]
    groups = W.groups_from_sizes(sizes)
    n = sum(sizes)
    rng = np.random.default_rng(9)
    g = rng.standard_normal(n).astype(F32)
    g[::17] = 0
    s = (g * g).astype(F32)                                   # single-sample batch: r^2 == v exactly
    z = np.zeros(n, F32)
    gw = GpuWorker(groups, dev)
    _, _, send, _, _ = _compare_step(gw, g, s, z, z, groups, 1.0, 0.999, dev)
    assert not send.any()                                     # ties are not sent (strict test)
    gw = GpuWorker(groups, dev)
    _, _, send, words, _ = _compare_step(gw, g, s, z, z, groups, 0.0, 0.999, dev)
    assert np.array_equal(send, g != 0)
    gw = GpuWorker(groups, dev)
    _, _, send, _, hdrs = _compare_step(gw, g, s, z, z, groups, 1e30, 0.999, dev)
    assert not send.any() and all(h[:2] == (0, 0) for h in hdrs)


def test_config1_ten_iterations_state_carry(dev):
    """Config 1: 1024x1024 weight, batch 32, 10 iterations, alpha 1, zeta 0.999.  The GPU keeps its
    own state across iterations; it must stay bit-identical to the oracle's."""
    cfg = W.CONFIGS["C1"]
    groups = W.groups_from_sizes([1024 * 1024])
    n = 1024 * 1024
    r = np.zeros(n, F32)
    v = np.zeros(n, F32)
    gw = GpuWorker(groups, dev)
    sent_frac = []
    for it in range(cfg["iterations"]):
        X, D = W.c1_inputs(it)
        g64, s64 = O.sqgrad_fc(X, D, 1.0 / cfg["batch"])
        g, s = g64.astype(F32).ravel(), s64.astype(F32).ravel()
        r, v, send, words, _ = _compare_step(gw, g, s, r, v, groups, cfg["alpha"], cfg["zeta"], dev)
        sent_frac.append(send.mean())
    assert 0.2 < sent_frac[0] < 0.45                          # fresh state, alpha = 1: about 0.3 for i.i.d. samples


def test_config1_whole_chain_from_the_gpu_statistic(dev):
    """Config 1 with every stage on the GPU: vgc_sqgrad (FC form, float32) feeds vgc_accumulate_select, vgc_pack and
    vgc_unpack_add directly, five iterations with the state carried.  The statistic is checked against the float64
    oracle at its tolerance; the stages after it are checked bit for bit against the oracle run on the very g, s the
    GPU produced (a last-bit difference in s may flip an element that sits on the test's boundary, so the comparison
    downstream takes the GPU's own statistic as its input)."""
    import torch
    from paper_1802_06058_amd import vgc
    cfg = W.CONFIGS["C1"]
    n, B = 1024 * 1024, cfg["batch"]
    groups = W.groups_from_sizes([n])
    plan = vgc.Plan(groups, dev)
    r = torch.zeros(n, dtype=torch.float32, device=dev); v = torch.zeros(n, dtype=torch.float32, device=dev)
    g = torch.empty(1024, 1024, dtype=torch.float32, device=dev); s = torch.empty(1024, 1024, dtype=torch.float32, device=dev)
    scratch, hdrs, status = plan.new_scratch(), plan.new_headers(), plan.new_status()
    words = torch.empty(n, dtype=torch.int32, device=dev)
    dense = torch.zeros(n, dtype=torch.float32, device=dev)
    r_ref, v_ref, d_ref = np.zeros(n, F32), np.zeros(n, F32), np.zeros(n, F32)
    for it in range(5):
        X, D = W.c1_inputs(it)
        vgc.sqgrad(vgc.FC, _dev(X, dev), _dev(D, dev), 1.0 / B, s, g)
        vgc.accumulate_select(g.view(-1), s.view(-1), r, v, plan, cfg["alpha"], cfg["zeta"], scratch)
        vgc.pack(plan, scratch, words, hdrs, status)
        torch.cuda.synchronize()
        total, overflow = vgc.read_status(status)
        vgc.unpack_add(words, total, hdrs, plan, 1.0, dense)
        gh, sh = g.cpu().numpy().ravel(), s.cpu().numpy().ravel()
        g64, s64 = O.sqgrad_fc(X, D, 1.0 / B)
        assert (np.abs(sh - s64.ravel()) <= 1e-5 * s64.ravel()).all()
        absG = (np.abs(X.astype(np.float64)).T @ np.abs(D.astype(np.float64))).ravel() / B
        assert (np.abs(gh - g64.ravel()) <= 1e-5 * absG).all()
        r_acc, r_ref, v_ref, send = O.accumulate_select(gh, sh, r_ref, v_ref, cfg["alpha"], cfg["zeta"])
        w_ref, h_ref, _ = O.pack(r_acc, send, groups)
        O.unpack_add(w_ref, h_ref, groups, 1.0, d_ref)
        assert np.array_equal(plan.send_mask(scratch), send)
        assert overflow == 0 and total == w_ref.size and vgc.read_headers(hdrs) == h_ref
        assert np.array_equal(words[:total].cpu().numpy().view(U32), w_ref)
        assert np.array_equal(_bits(r.cpu().numpy()), _bits(r_ref)) and np.array_equal(_bits(v.cpu().numpy()), _bits(v_ref))
        torch.cuda.synchronize()
        assert np.array_equal(_bits(dense.cpu().numpy()), _bits(d_ref))


def test_config2_mlp_sparse_inputs(dev):
    """Config 2, all 50 iterations with the state carried: three groups, ReLU-sparse inputs give exact ties."""
    cfg = W.CONFIGS["C2"]
    layers = cfg["layers"]
    groups = W.groups_from_sizes([L["size"] for L in layers])
    n = sum(L["size"] for L in layers)
    r = np.zeros(n, F32)
    v = np.zeros(n, F32)
    gw = GpuWorker(groups, dev)
    for it in range(cfg["iterations"]):
        gs, ss = [], []
        for li in range(3):
            X, D = W.c2_inputs(it, li)
            g64, s64 = O.sqgrad_fc(X, D, 1.0 / cfg["batch"])
            gs.append(g64.astype(F32).ravel()); ss.append(s64.astype(F32).ravel())
        r, v, send, _, _ = _compare_step(gw, np.concatenate(gs), np.concatenate(ss), r, v, groups,
                                         cfg["alpha"], cfg["zeta"], dev)


def test_capacity_overflow_is_reported_not_written(dev):
    sizes = [2048 * 4, 3000]
    groups = W.groups_from_sizes(sizes)
    n = sum(sizes)
    g, s = sample_stream(3, (0,), n, 16, "normal", sigma=0.1)
    z = np.zeros(n, F32)
    r_acc, _, _, send = O.accumulate_select(g, s, z, z, 1.0, 0.999)
    words, hdrs, _ = O.pack(r_acc, send, groups)
    cap = words.size // 2
    gw = GpuWorker(groups, dev, words_cap=cap)
    mask, ghdrs, gwords, total, overflow = gw.step(_dev(g, dev), _dev(s, dev), 1.0, 0.999)
    assert overflow == 1 and total == words.size and ghdrs == hdrs
    assert np.array_equal(gwords, words[:cap])                # what fits is right; the canary check ran in step()


def test_deterministic_and_independent_of_stale_scratch(dev):
    sizes = [2048 * 9 + 100, 777]
    groups = W.groups_from_sizes(sizes)
    n = sum(sizes)
    g, s = sample_stream(4, (0,), n, 16, "student", sigma=1.0)
    outs = []
    for fill in (0x00, 0xFF):
        gw = GpuWorker(groups, dev)
        gw.scratch.fill_(fill)
        mask, hdrs, words, total, _ = gw.step(_dev(g, dev), _dev(s, dev), 1.0, 0.999)
        outs.append((mask, hdrs, words, gw.r.cpu().numpy(), gw.v.cpu().numpy()))
    assert np.array_equal(outs[0][0], outs[1][0]) and outs[0][1] == outs[1][1]
    assert np.array_equal(outs[0][2], outs[1][2])
    assert np.array_equal(_bits(outs[0][3]), _bits(outs[1][3])) and np.array_equal(_bits(outs[0][4]), _bits(outs[1][4]))


@pytest.mark.parametrize("scale", [0.125, 1.0 / 3.0])
def test_unpack_add_messages_in_order(dev, scale):
    import torch
    from paper_1802_06058_amd import vgc
    sizes = [5000, 1, 2048 * 3, 77]
    groups = W.groups_from_sizes(sizes)
    n = sum(sizes)
    plan = vgc.Plan(groups, dev)
    rng = np.random.default_rng(2)
    dense0 = rng.standard_normal(n).astype(F32)
    expect = dense0.copy()
    dense = _dev(dense0, dev)
    for w in range(8):
        g, s = sample_stream(6, (w,), n, 16, "student", sigma=10.0 ** rng.uniform(-3, 0))
        z = np.zeros(n, F32)
        r_acc, _, _, send = O.accumulate_select(g, s, z, z, 1.0, 0.999)
        words, hdrs, _ = O.pack(r_acc, send, groups)
        O.unpack_add(words, hdrs, groups, scale, expect)
        h = np.array(hdrs, dtype=vgc.HDR_DTYPE)
        d_words = _dev(words.view(np.int32) if words.size else np.zeros(1, np.int32), dev)
        d_hdrs = _dev(h.view(np.uint8), dev)
        vgc.unpack_add(d_words, words.size, d_hdrs, plan, scale, dense)
    torch.cuda.synchronize()
    assert np.array_equal(_bits(dense.cpu().numpy()), _bits(expect))


@pytest.mark.parametrize("alpha", [0.0, 1.0, 6.0])
def test_unpack_add_both_kernels_decode_the_same_message(dev, alpha):
    """vgc_unpack_add picks its kernel from n_words (one thread per word below n / 8, tile by tile from there on) and
    accepts an upper bound for it: the same message given with its exact count and with a bound on the other side of
    n / 8 (where the count allows) must decode to the oracle's bits both times."""
    import torch
    from paper_1802_06058_amd import vgc
    sizes = [2048 * 9 + 77, 3, 2048 * 4, 5000]
    groups = W.groups_from_sizes(sizes)
    n = sum(sizes)
    plan = vgc.Plan(groups, dev)
    g, s = sample_stream(31, (int(alpha),), n, 16, "student", sigma=0.05)
    z = np.zeros(n, F32)
    r_acc, _, _, send = O.accumulate_select(g, s, z, z, alpha, 0.999)
    words, hdrs, _ = O.pack(r_acc, send, groups)
    rng = np.random.default_rng(5)
    dense0 = rng.standard_normal(n).astype(F32)
    expect = dense0.copy()
    O.unpack_add(words, hdrs, groups, 0.25, expect)
    pad = np.full(n + 8, 0x0BADC0DE, np.uint32)                 # junk past the message
    pad[:words.size] = words
    d_words = _dev(pad.view(np.int32), dev)
    d_hdrs = _dev(np.array(hdrs, dtype=vgc.HDR_DTYPE).view(np.uint8), dev)
    counts = {words.size, max(words.size, n // 8), max(words.size, n // 8 - 1), n}
    assert any(c >= n // 8 for c in counts) and (words.size >= n // 8 or any(c < n // 8 for c in counts))
    for c in sorted(counts):
        dense = _dev(dense0, dev)
        vgc.unpack_add(d_words, c, d_hdrs, plan, 0.25, dense)
        torch.cuda.synchronize()
        assert np.array_equal(_bits(dense.cpu().numpy()), _bits(expect)), f"n_words = {c} of n = {n}, message of {words.size}"


def test_full_round_trip_gpu_pack_to_gpu_unpack(dev):
    """GPU-packed message decoded by the GPU equals the oracle's decode of the oracle's message,
    and the conservation invariant holds on the GPU results."""
    import torch
    from paper_1802_06058_amd import vgc
    sizes = [2048 * 5 + 9, 4000]
    groups = W.groups_from_sizes(sizes)
    n = sum(sizes)
    g, s = sample_stream(8, (0,), n, 16, "student", sigma=0.02)
    z = np.zeros(n, F32)
    gw = GpuWorker(groups, dev)
    r_out, v_out, send, words, hdrs = _compare_step(gw, g, s, z, z, groups, 1.0, 0.999, dev)
    dense = torch.zeros(n, dtype=torch.float32, device=dev)
    vgc.unpack_add(gw.words, gw.cap, gw.hdrs, gw.plan, 1.0, dense)     # n_words given as an upper bound
    torch.cuda.synchronize()
    expect = np.zeros(n, F32)
    O.unpack_add(words, hdrs, groups, 1.0, expect)
    got = dense.cpu().numpy()
    assert np.array_equal(_bits(got), _bits(expect))
    r_acc = (z + g)
    kept = got != 0
    assert np.all(np.abs(got[kept].astype(np.float64) - r_acc[kept]) < np.abs(r_acc[kept]) / 2)
    assert not got[~send].any()


def test_abi_rejects_bad_arguments(dev):
    import torch
    from paper_1802_06058_amd import vgc
    lib = vgc.load()
    groups = W.groups_from_sizes([100, 200])
    plan = vgc.Plan(groups, dev)
    t = torch.zeros(300, dtype=torch.float32, device=dev)
    sc = plan.new_scratch()
    with pytest.raises(vgc.VgcError):
        vgc.accumulate_select(t, t, t, t, plan, -1.0, 0.999, sc)
    with pytest.raises(vgc.VgcError):
        vgc.accumulate_select(t, t, t, t, plan, 1.0, 1.5, sc)
    with pytest.raises(vgc.VgcError):
        vgc.accumulate_select(t, t, t, None, plan, 1.0, 0.999, sc)
    assert float(t.abs().sum()) == 0.0


@pytest.mark.parametrize("p,overwrite", [(0, True), (1, False), (3, True), (8, False), (11, True)])
def test_unpack_add_batch_equals_sequential(dev, p, overwrite):
    """One pass over the dense buffer for p messages: bit-identical to the oracle applying the
    messages one after another (and so to p single-message launches).  Groups span several runs
    of 64 tiles, have ragged tails and odd offsets; message densities differ widely."""
    import torch
    from paper_1802_06058_amd import vgc
    sizes = [2048 * 70 + 5, 3, 5000, 2048 * 130, 1]
    groups = W.groups_from_sizes(sizes)
    n = sum(sizes)
    plan = vgc.Plan(groups, dev)
    rng = np.random.default_rng(p)
    dense0 = rng.standard_normal(n).astype(F32)
    expect = np.zeros(n, F32) if overwrite else dense0.copy()
    dense = _dev(dense0, dev)
    dense_seq = torch.zeros(n, dtype=torch.float32, device=dev) if overwrite else _dev(dense0, dev)
    d_words, d_hdrs, counts = [], [], []
    scale = 1.0 / 3.0
    for w in range(p):
        g, s = sample_stream(16, (p, w), n, 16, "student", sigma=10.0 ** rng.uniform(-3, 0))
        z = np.zeros(n, F32)
        alpha = [0.0, 1.0, 4.0, 12.0][w % 4]                   # dense, typical, sparse, very sparse messages
        r_acc, _, _, send = O.accumulate_select(g, s, z, z, alpha, 0.999)
        if w == 2:
            send[: 2048 * 70 + 5] = False                      # a whole group absent from this message
        words, hdrs, _ = O.pack(r_acc, send, groups)
        O.unpack_add(words, hdrs, groups, scale, expect)
        pad = np.full(words.size + 100, 0x12345678, np.uint32)  # junk past the message; counts are upper bounds
        pad[:words.size] = words
        d_words.append(_dev(pad.view(np.int32), dev))
        d_hdrs.append(_dev(np.array(hdrs, dtype=vgc.HDR_DTYPE).view(np.uint8), dev))
        counts.append(words.size + (50 if w % 2 else 0))
        vgc.unpack_add(d_words[-1], counts[-1], d_hdrs[-1], plan, scale, dense_seq)
    vgc.unpack_add_batch(d_words, counts, d_hdrs, plan, scale, dense, overwrite=overwrite)
    torch.cuda.synchronize()
    got = dense.cpu().numpy()
    assert np.array_equal(_bits(got), _bits(expect)), f"{np.flatnonzero(_bits(got) != _bits(expect))[:10]}"
    assert np.array_equal(_bits(dense_seq.cpu().numpy()), _bits(expect))


def test_plan_of_another_group_list_is_refused_on_the_device(dev):
    """A device plan used with a host group list it was not built from (same n, same number of groups and tiles,
    so every table has the same size): the kernels compare the list's hash with the plan's and do nothing; the
    status says so, r, v, the word buffer and the dense buffer stay as they were, the headers describe an empty message."""
    import torch
    from paper_1802_06058_amd import vgc
    a = vgc.Plan(W.groups_from_sizes([4096, 4096]), dev)
    b = vgc.Plan(W.groups_from_sizes([2048, 6144]), dev)
    assert (a.n, a.n_groups, a.n_tiles) == (b.n, b.n_groups, b.n_tiles)
    b.plan = a.plan                                            # host list of b, device tables of a
    n = a.n
    g, s = sample_stream(12, (0,), n, 16, "student", sigma=0.01)
    r = torch.full((n,), 3.0, dtype=torch.float32, device=dev); v = torch.full((n,), 5.0, dtype=torch.float32, device=dev)
    scratch, hdrs, status = b.new_scratch(), b.new_headers(), b.new_status()
    hdrs.fill_(0xEE)
    words = torch.full((n,), -1, dtype=torch.int32, device=dev)
    vgc.accumulate_select(_dev(g, dev), _dev(s, dev), r, v, b, 1.0, 0.999, scratch)
    vgc.pack(b, scratch, words, hdrs, status)
    torch.cuda.synchronize()
    with pytest.raises(vgc.VgcError, match="not built from the group list"):
        vgc.read_status(status)
    assert float(r.min()) == 3.0 == float(r.max()) and float(v.min()) == 5.0 == float(v.max())
    assert int((words != -1).sum()) == 0
    assert vgc.read_headers(hdrs) == [(0, 0, 0), (0, 0, 0)]
    # the decoders refuse the same way: nothing is added
    good = GpuWorker(W.groups_from_sizes([2048, 6144]), dev)
    mask, ghdrs, gwords, total, overflow = good.step(_dev(g, dev), _dev(s, dev), 1.0, 0.999)
    assert total > 0
    dense = torch.full((n,), 7.0, dtype=torch.float32, device=dev)
    vgc.unpack_add(good.words, total, good.hdrs, b, 1.0, dense)
    vgc.unpack_add_batch([good.words], [total], [good.hdrs], b, 1.0, dense, overwrite=True)
    m = torch.zeros(n, dtype=torch.float32, device=dev)
    vgc.unpack_apply([good.words], [total], [good.hdrs], b, 1.0, dense, m, kind=vgc.MOMENTUM_SGD, lr=1.0, momentum=0.5)
    torch.cuda.synchronize()
    assert float(dense.min()) == 7.0 == float(dense.max()) and float(m.abs().max()) == 0.0
