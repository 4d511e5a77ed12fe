"""vgc_sqgrad_accumulate_select (the statistic of a fully-connected layer formed on the matrix cores and consumed
in place by Alg. 1's loop body) and vgc_accumulate_select_range (the pass over the remaining groups).

The statistic is compared with the float64 oracle at its tolerance (s: relative 1e-5 for float32, 1e-2 for bfloat16
inputs; g against the magnitudes summed).  Everything after it is compared bit for bit with the oracle run on the very
g, s the kernel produced (its optional g_out / s_out): a last-bit difference in s may flip an element on the test's
boundary, so the stages downstream take the GPU's own statistic as their input."""
import numpy as np
import pytest

from oracle import vgc_oracle as O
from paper_1802_06058_amd import workloads as W
from streams import sample_stream

pytestmark = pytest.mark.gpu

F32 = np.float32
U32 = np.uint32
RTOL = {"f32": 1e-5, "bf16": 1e-2}


@pytest.fixture(scope="module")
def dev():
    import torch
    from paper_1802_06058_amd import vgc
    assert torch.cuda.is_available()
    vgc.load()
    return torch.device("cuda:0")


def _bits(a):
    return np.ascontiguousarray(a).view(U32)


CASES = [  # B, J, C, precision, size of the group in front of the layer
    (64, 100, 4096, "bf16", 1000),      # a tile is half a row; the last block has 4 live rows of 16
    (32, 48, 2048, "f32", 3000),        # a tile is a row
    (50, 40, 2048, "bf16", 1001),       # batch not a multiple of the MFMA's K; odd offset: 4-byte accesses throughout
    (32, 1024, 1024, "f32", 2048),      # config 1's layer: a tile is two rows
    (7, 20, 1024, "f32", 8),            # tiny batch
    (16, 70, 512, "bf16", 512),         # a tile is four rows; 17.5 tiles: the last tile is partial
    (8, 33, 256, "f32", 4),             # a tile is eight rows; partial last tile
    (128, 64, 6144, "bf16", 100),       # three column blocks, batch of config 2
]


@pytest.mark.parametrize("B,J,C,prec,front", CASES)
def test_fused_layer_inside_a_model(dev, B, J, C, prec, front):
    import torch
    from paper_1802_06058_amd import vgc
    bf16 = prec == "bf16"
    sizes = [front, J * C, 5000]
    groups = W.groups_from_sizes(sizes)
    plan = vgc.Plan(groups, dev)
    n, lo, hi = plan.n, front, front + J * C
    code = vgc.BF16 if bf16 else vgc.F32
    nb = vgc.sqgrad_accumulate_select_workspace_bytes(code, B, J, C)
    assert nb > 0
    ws = torch.full((nb,), 0xFF, dtype=torch.uint8, device=dev)
    rng = np.random.default_rng(B + J)
    r0 = (rng.standard_normal(n) * 1e-4).astype(F32)
    v0 = (rng.random(n) * 1e-8).astype(F32)
    r = torch.from_numpy(r0).to(dev); v = torch.from_numpy(v0).to(dev)
    r_ref, v_ref = r0.copy(), v0.copy()
    scratch = plan.new_scratch(); scratch.fill_(0xC3)
    words = torch.full((n + 64,), -1, dtype=torch.int32, device=dev)
    hdrs, status = plan.new_headers(), plan.new_status()
    g_out = torch.empty(J, C, dtype=torch.float32, device=dev); s_out = torch.empty(J, C, dtype=torch.float32, device=dev)
    c = 1.0 / B
    for step in range(3):
        X, D = W.fc_inputs(61, (B, J, C, step), B, J, C, "normal", relu_sparse=(step == 1), d_sigma=0.01, bf16=bf16)
        g_rest, s_rest = sample_stream(62, (J, C, step), n, 16, "student", sigma=3e-4)
        g_rest[lo:hi] = np.nan; s_rest[lo:hi] = np.nan                       # the layer's part of g, s must never be read
        gd, sd = torch.from_numpy(g_rest).to(dev), torch.from_numpy(s_rest).to(dev)
        Xd, Dd = torch.from_numpy(X).to(dev), torch.from_numpy(D).to(dev)
        if bf16:
            Xd, Dd = Xd.view(torch.bfloat16), Dd.view(torch.bfloat16)
        g_out.fill_(float("nan")); s_out.fill_(float("nan"))
        state = (r.clone(), v.clone())
        vgc.accumulate_select_range(gd, sd, r, v, plan, 0, 1, 1.0, 0.999, scratch)
        vgc.sqgrad_accumulate_select(Xd, Dd, c, r, v, plan, 1, 1.0, 0.999, scratch, ws, g_out, s_out)
        vgc.accumulate_select_range(gd, sd, r, v, plan, 2, 1, 1.0, 0.999, scratch)
        mask = plan.send_mask(scratch)
        vgc.pack(plan, scratch, words[:n], hdrs, status)
        torch.cuda.synchronize()
        total, overflow = vgc.read_status(status)
        gh, sh = g_out.cpu().numpy(), s_out.cpu().numpy()
        # the statistic against the float64 oracle
        Xw = W.bf16_bits_to_f32(X).astype(np.float64) if bf16 else X.astype(np.float64)
        Dw = W.bf16_bits_to_f32(D).astype(np.float64) if bf16 else D.astype(np.float64)
        g64, s64 = O.sqgrad_fc(Xw, Dw, c)
        assert np.isfinite(sh).all() and np.isfinite(gh).all()
        pos = s64 > 0
        assert (np.abs(sh - s64)[pos] <= RTOL[prec] * s64[pos]).all(), f"s relative error {(np.abs(sh - s64)[pos] / s64[pos]).max():.3e}"
        assert np.all(sh[~pos] == 0)
        absG = (np.abs(Xw).T @ np.abs(Dw)) * c
        assert (np.abs(gh - g64) <= RTOL[prec] * absG + 1e-300).all()
        # everything downstream, bit for bit, from the GPU's own g, s
        g_all, s_all = g_rest.copy(), s_rest.copy()
        g_all[lo:hi], s_all[lo:hi] = gh.ravel(), sh.ravel()
        r_acc, r_ref, v_ref, send = O.accumulate_select(g_all, s_all, r_ref, v_ref, 1.0, 0.999)
        w_ref, h_ref, _ = O.pack(r_acc, send, groups)
        assert np.array_equal(mask, send), f"mask differs at {np.flatnonzero(mask != send)[:8]}"
        assert np.array_equal(_bits(r.cpu().numpy()), _bits(r_ref))
        assert np.array_equal(_bits(v.cpu().numpy()), _bits(v_ref))
        assert overflow == 0 and total == w_ref.size and vgc.read_headers(hdrs) == h_ref
        got = words.cpu().numpy().view(U32)
        assert np.array_equal(got[:total], w_ref) and np.all(got[n:] == 0xFFFFFFFF)
        assert send[lo:hi].any() and not send[lo:hi].all()
        # without the optional outputs: the same state and message
        r2, v2 = state
        scratch2 = plan.new_scratch()
        words2 = torch.empty(n, dtype=torch.int32, device=dev)
        vgc.accumulate_select_range(gd, sd, r2, v2, plan, 0, 1, 1.0, 0.999, scratch2)
        vgc.sqgrad_accumulate_select(Xd, Dd, c, r2, v2, plan, 1, 1.0, 0.999, scratch2, ws)
        vgc.accumulate_select_range(gd, sd, r2, v2, plan, 2, 1, 1.0, 0.999, scratch2)
        vgc.pack(plan, scratch2, words2, hdrs, status)
        torch.cuda.synchronize()
        assert vgc.read_status(status) == (total, 0)
        assert torch.equal(r2.view(torch.int32), r.view(torch.int32)) and torch.equal(v2.view(torch.int32), v.view(torch.int32))
        assert np.array_equal(words2[:total].cpu().numpy().view(U32), w_ref)


def test_range_calls_equal_the_whole_model_call(dev):
    """vgc_accumulate_select_range over [0, 2), [2, 3) and [3, 6) leaves exactly what one vgc_accumulate_select leaves."""
    import torch
    from paper_1802_06058_amd import vgc
    sizes = [5000, 1, 2048 * 3 + 7, 64, 2048, 9000]
    plan = vgc.Plan(W.groups_from_sizes(sizes), dev)
    n = plan.n
    g, s = sample_stream(63, (0,), n, 16, "student", sigma=0.01)
    gd, sd = torch.from_numpy(g).to(dev), torch.from_numpy(s).to(dev)
    outs = []
    for ranges in ([(0, 6)], [(3, 3), (0, 2), (2, 1)]):
        r = torch.zeros(n, dtype=torch.float32, device=dev); v = torch.zeros(n, dtype=torch.float32, device=dev)
        scratch, hdrs, status = plan.new_scratch(), plan.new_headers(), plan.new_status()
        words = torch.empty(n, dtype=torch.int32, device=dev)
        for first, count in ranges:
            vgc.accumulate_select_range(gd, sd, r, v, plan, first, count, 1.0, 0.999, scratch)
        vgc.pack(plan, scratch, words, hdrs, status)
        torch.cuda.synchronize()
        total, _ = vgc.read_status(status)
        outs.append((r.cpu().numpy(), v.cpu().numpy(), words[:total].cpu().numpy(), vgc.read_headers(hdrs)))
    assert all(np.array_equal(_bits(a), _bits(b)) for a, b in zip(outs[0][:3], outs[1][:3])) and outs[0][3] == outs[1][3]
    with pytest.raises(vgc.VgcError):
        vgc.accumulate_select_range(gd, sd, r, v, plan, 4, 3, 1.0, 0.999, scratch)


def test_fused_rejects_what_it_cannot_do(dev):
    import torch
    from paper_1802_06058_amd import vgc
    assert vgc.sqgrad_accumulate_select_workspace_bytes(vgc.F32, 32, 100, 1000) == 0
    plan = vgc.Plan(W.groups_from_sizes([10, 20 * 1024, 30]), dev)
    n = plan.n
    r = torch.ones(n, dtype=torch.float32, device=dev); v = torch.ones(n, dtype=torch.float32, device=dev)
    X, D = torch.zeros(4, 20, device=dev), torch.zeros(4, 1024, device=dev)
    ws = torch.zeros(1 << 20, dtype=torch.uint8, device=dev)
    sc = plan.new_scratch()
    with pytest.raises(vgc.VgcError, match="does not have"):
        vgc.sqgrad_accumulate_select(X, D, 0.25, r, v, plan, 0, 1.0, 0.999, sc, ws)
    with pytest.raises(vgc.VgcError, match="workspace"):
        vgc.sqgrad_accumulate_select(X, D, 0.25, r, v, plan, 1, 1.0, 0.999, sc, ws[:100])
    lib = vgc.load()
    rc = lib.vgc_sqgrad_accumulate_select(vgc.F32, X.data_ptr(), D.data_ptr(), 4, 20, 1000, 0.25, r.data_ptr(), v.data_ptr(), n,
                                          plan.c_groups, 3, plan.plan.data_ptr(), 1, 1.0, 0.999, sc.data_ptr(), ws.data_ptr(),
                                          ws.numel(), None, None, None)
    assert rc == -2
    torch.cuda.synchronize()
    assert float(r.min()) == 1.0 == float(v.max())
