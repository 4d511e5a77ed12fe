"""Parity at the full sizes of the benchmark configurations, in the launch configuration bench.py
times (same plan, same tile size, same entry points).  Where the oracle cannot process the whole
output in seconds, whole groups / sampled outputs are recomputed by it and the rest is covered by
properties that hold at any size."""
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
    assert torch.cuda.is_available()
    vgc.load()
    return torch.device("cuda:0")


def _bits(a):
    return np.ascontiguousarray(a).view(U32)


def test_flat_1e9_stream_select_pack_decode(dev):
    """Config 5 at full size (1e9 parameters, 60 groups of 2^24, Student-t(3), batch 16): one worker,
    two steps.  Three groups (first, one in the middle, the partial last one) are recomputed whole by
    the oracle from the same inputs and compared bit for bit; the rest through size-independent
    properties of headers, words and state."""
    import torch
    from paper_1802_06058_amd import vgc
    cfg = W.CONFIGS["C5"]
    N = cfg["n"]
    groups = W.flat_groups(N, cfg["group"])
    plan = vgc.Plan(groups, dev)
    r = torch.zeros(N, dtype=torch.float32, device=dev)
    v = torch.zeros(N, dtype=torch.float32, device=dev)
    scratch = plan.new_scratch()
    words = torch.empty(N // 2, dtype=torch.int32, device=dev)
    hdrs, status = plan.new_headers(), plan.new_status()
    dense = torch.empty(N, dtype=torch.float32, device=dev)
    check = [0, 31, len(groups) - 1]
    r_ref = {k: np.zeros(groups[k][1], F32) for k in check}
    v_ref = {k: np.zeros(groups[k][1], F32) for k in check}
    for step in range(2):
        g, s = device_student_stream(N, cfg["batch"], cfg["nu"], cfg["seed"] + 17 * step, dev)
        vgc.accumulate_select(g, s, r, v, plan, cfg["alpha"], cfg["zeta"], scratch)
        vgc.pack(plan, scratch, words, hdrs, status)
        torch.cuda.synchronize()
        total, overflow = vgc.read_status(status)
        H = vgc.read_headers(hdrs)
        assert overflow == 0 and 0.1 * N < total < 0.45 * N
        # properties over all groups: offsets chain, counts add up, exponent fields plausible
        pos = 0
        for (off, size), (ef, cnt, woff) in zip(groups, H):
            assert woff == pos and cnt <= size and (cnt == 0) == (ef == 0)
            pos += cnt
        assert pos == total
        vgc.unpack_add_batch([words], [total], [hdrs], plan, 0.125, dense, overwrite=True)
        torch.cuda.synchronize()
        for k in check:
            off, size = groups[k]
            gk, sk = g[off:off + size].cpu().numpy(), s[off:off + size].cpu().numpy()
            r_acc, r_out, v_out, send = O.accumulate_select(gk, sk, r_ref[k], v_ref[k], cfg["alpha"], cfg["zeta"])
            w_ref, h_ref, _ = O.pack(r_acc, send, [(0, size)], check=False)
            ef, cnt, woff = H[k]
            assert (ef, cnt) == h_ref[0][:2]
            assert np.array_equal(words[woff:woff + cnt].cpu().numpy().view(U32), w_ref)
            assert np.array_equal(_bits(r[off:off + size].cpu().numpy()), _bits(r_out))
            assert np.array_equal(_bits(v[off:off + size].cpu().numpy()), _bits(v_out))
            d_ref = np.zeros(size, F32)
            O.unpack_add(w_ref, h_ref, [(0, size)], 0.125, d_ref)
            assert np.array_equal(_bits(dense[off:off + size].cpu().numpy()), _bits(d_ref))
            r_ref[k], v_ref[k] = r_out, v_out
        # whole-array properties of the state: sent elements are exactly the zeros of (r, v) that decoded or dropped
        nz = int(torch.count_nonzero(dense))
        assert nz == total
        del g, s


def _messages_of_workers(dev, plan, groups, cfg, N, P, check, hybrid=None):
    """P workers' messages at full size, each from a fresh state and its own seeded inputs, packed on the GPU.
    The groups in `check` are recomputed by the oracle from the same inputs and must agree bit for bit; returns the
    device messages and, per checked group, the oracle's messages [(words, headers)] in worker order."""
    import torch
    from paper_1802_06058_amd import vgc
    r = torch.empty(N, dtype=torch.float32, device=dev)
    v = torch.empty(N, dtype=torch.float32, device=dev)
    scratch = plan.new_scratch()
    words, hdrs, counts = [], [], []
    ref = {k: [] for k in check}
    for w in range(P):
        g, s = device_student_stream(N, cfg["batch"], cfg["nu"], 4000 + 31 * w, dev)
        if w % 2:
            g *= 0.25 * (w + 1); s *= (0.25 * (w + 1)) ** 2          # workers of different gradient scale: exponent fields differ
        r.zero_(); v.zero_()
        wd = torch.empty(N // 2, dtype=torch.int32, device=dev)
        hd, st = plan.new_headers(), plan.new_status()
        if hybrid is None:
            vgc.accumulate_select(g, s, r, v, plan, cfg["alpha"], cfg["zeta"], scratch)
        else:
            vgc.accumulate_select_hybrid(g, s, r, v, plan, hybrid[0], cfg["zeta"], hybrid[1], scratch)
        vgc.pack(plan, scratch, wd, hd, st)
        torch.cuda.synchronize()
        total, overflow = vgc.read_status(st)
        assert overflow == 0 and total > 0
        H = vgc.read_headers(hd)
        for k in check:
            off, size = groups[k]
            gk, sk = g[off:off + size].cpu().numpy(), s[off:off + size].cpu().numpy()
            z = np.zeros(size, F32)
            if hybrid is None:
                r_acc, r_out, v_out, send = O.accumulate_select(gk, sk, z, z, cfg["alpha"], cfg["zeta"])
                w_ref, h_ref, _ = O.pack(r_acc, send, [(0, size)], check=False)
            else:
                r_out, v_out, send, sign = O.accumulate_select_hybrid(gk, sk, z, z, hybrid[0], cfg["zeta"], hybrid[1])
                w_ref, h_ref = O.pack_hybrid(sign, send, [(0, size)])
            ef, cnt, woff = H[k]
            assert (ef, cnt) == h_ref[0][:2]
            assert np.array_equal(wd[woff:woff + cnt].cpu().numpy().view(U32), w_ref)
            assert np.array_equal(_bits(r[off:off + size].cpu().numpy()), _bits(r_out))
            assert np.array_equal(_bits(v[off:off + size].cpu().numpy()), _bits(v_out))
            ref[k].append((w_ref, h_ref))
        words.append(wd); hdrs.append(hd); counts.append(total)
        del g, s
    return words, hdrs, counts, ref


def test_flat_1e9_eight_messages_batched_decode_and_update(dev):
    """What the benchmark times after the exchange, at its size: the messages of 8 workers over 1e9 parameters
    decoded in one pass (vgc_unpack_add_batch, overwrite) and decoded fused with a Momentum SGD and an Adam step
    (vgc_unpack_apply).  Three groups (first, middle, the partial last one) are recomputed whole by the oracle,
    messages applied in worker order, and compared bit for bit; over the whole array the fused decoder must
    reproduce the batched decoder's sums exactly."""
    import torch
    from paper_1802_06058_amd import vgc
    cfg = W.CONFIGS["C5"]
    N, P = cfg["n"], cfg["workers"]
    groups = W.flat_groups(N, cfg["group"])
    plan = vgc.Plan(groups, dev)
    check = [0, 29, len(groups) - 1]
    words, hdrs, counts, ref = _messages_of_workers(dev, plan, groups, cfg, N, P, check)
    scale = 1.0 / P
    dense = torch.full((N,), float("nan"), dtype=torch.float32, device=dev)
    vgc.unpack_add_batch(words, counts, hdrs, plan, scale, dense, overwrite=True)
    torch.cuda.synchronize()
    for k in check:
        off, size = groups[k]
        d_ref = np.zeros(size, F32)
        for w_ref, h_ref in ref[k]:
            O.unpack_add(w_ref, h_ref, [(0, size)], scale, d_ref)
        assert np.array_equal(_bits(dense[off:off + size].cpu().numpy()), _bits(d_ref))
    assert bool(torch.isfinite(dense).all())
    # the same messages added on top of what is there (no overwrite): exactly twice the sums in float32
    vgc.unpack_add_batch(words[:1], counts[:1], hdrs[:1], plan, scale, dense, overwrite=True)
    vgc.unpack_add_batch(words[1:], counts[1:], hdrs[1:], plan, scale, dense, overwrite=False)
    torch.cuda.synchronize()
    for k in check:
        off, size = groups[k]
        d_ref = np.zeros(size, F32)
        for w_ref, h_ref in ref[k]:
            O.unpack_add(w_ref, h_ref, [(0, size)], scale, d_ref)
        assert np.array_equal(_bits(dense[off:off + size].cpu().numpy()), _bits(d_ref))

    # decode fused with the update; lr = 1, momentum = 0, zero parameters: w = -ghat must be the batched decoder's sum, negated
    gen = torch.Generator(device=dev); gen.manual_seed(77)
    param = torch.zeros(N, dtype=torch.float32, device=dev)
    m1 = torch.zeros(N, dtype=torch.float32, device=dev)
    vgc.unpack_apply(words, counts, hdrs, plan, scale, param, m1, kind=vgc.MOMENTUM_SGD, lr=1.0, momentum=0.0)
    torch.cuda.synchronize()
    assert bool(torch.equal(param, -dense))
    del dense
    # general steps against the oracle on the three groups
    for kind, name, hyper in ((vgc.MOMENTUM_SGD, "momentum_sgd", dict(lr=0.05, mu=0.9)),
                              (vgc.ADAM, "adam", dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, t=3))):
        param = torch.randn(N, generator=gen, device=dev, dtype=torch.float32)
        m1 = torch.randn(N, generator=gen, device=dev, dtype=torch.float32) * 0.01
        m2 = torch.rand(N, generator=gen, device=dev, dtype=torch.float32) * 1e-4 if kind == vgc.ADAM else None
        before = {k: tuple(x[groups[k][0]:groups[k][0] + groups[k][1]].cpu().numpy() if x is not None else None
                           for x in (param, m1, m2)) for k in check}
        if kind == vgc.ADAM:
            vgc.unpack_apply(words, counts, hdrs, plan, scale, param, m1, m2, kind=kind, lr=hyper["lr"], beta1=hyper["beta1"],
                             beta2=hyper["beta2"], eps=hyper["eps"], step=hyper["t"])
        else:
            vgc.unpack_apply(words, counts, hdrs, plan, scale, param, m1, kind=kind, lr=hyper["lr"], momentum=hyper["mu"])
        torch.cuda.synchronize()
        for k in check:
            off, size = groups[k]
            w0, a0, b0 = before[k]
            out = O.unpack_apply(ref[k], [(0, size)], scale, size, name, w0, a0, b0, **hyper)
            got = (param, m1, m2)
            for x_ref, x in zip(out, got):
                assert np.array_equal(_bits(x[off:off + size].cpu().numpy()), _bits(x_ref)), f"{name} group {k}"
        del param, m1, m2


def test_flat_1e9_hybrid_select_pack_decode(dev):
    """Alg. 2 at the benchmark's size (1e9 parameters, alpha 2, tau 0.05 as bench.py times it): two workers'
    messages, three groups recomputed whole by the oracle (mask via the words, state, headers, words), then both
    messages decoded with scale tau / 2 in one pass and compared with the oracle's decode in worker order."""
    import torch
    from paper_1802_06058_amd import vgc
    cfg = W.CONFIGS["C5"]
    N = cfg["n"]
    groups = W.flat_groups(N, cfg["group"])
    plan = vgc.Plan(groups, dev)
    check = [0, 37, len(groups) - 1]
    alpha, tau = 2.0, 0.05
    words, hdrs, counts, ref = _messages_of_workers(dev, plan, groups, cfg, N, 2, check, hybrid=(alpha, tau))
    assert all(0.001 * N < c < 0.3 * N for c in counts)
    dense = torch.empty(N, dtype=torch.float32, device=dev)
    vgc.unpack_add_batch(words, counts, hdrs, plan, tau / 2, dense, overwrite=True)
    torch.cuda.synchronize()
    for k in check:
        off, size = groups[k]
        d_ref = np.zeros(size, F32)
        for w_ref, h_ref in ref[k]:
            O.unpack_add(w_ref, h_ref, [(0, size)], tau / 2, d_ref)
        assert np.array_equal(_bits(dense[off:off + size].cpu().numpy()), _bits(d_ref))
    # every decoded value is a multiple of tau / 2 with at most two contributions
    vals = torch.unique(dense[: 1 << 26])
    assert vals.numel() <= 5


def test_vgg_parameter_set_hybrid_full_oracle(dev):
    """Alg. 2 on the VGG-16-shaped parameter set (32 groups, 138 M parameters, per-layer gradient scales), two steps
    with state carry: every output against the oracle."""
    import torch
    from paper_1802_06058_amd import vgc
    cfg = W.CONFIGS["C4"]
    layers = cfg["layers"]
    sizes = [L["size"] for L in layers]
    groups = W.groups_from_sizes(sizes)
    plan = vgc.Plan(groups, dev)
    n = plan.n
    sig = W.layer_sigmas(cfg["seed"], len(layers))
    alpha, tau, B = 2.0, 2e-4, cfg["batch"]
    r = torch.zeros(n, dtype=torch.float32, device=dev); v = torch.zeros(n, dtype=torch.float32, device=dev)
    scratch, hdrs, status = plan.new_scratch(), plan.new_headers(), plan.new_status()
    words = torch.empty(n, dtype=torch.int32, device=dev)
    dense = torch.zeros(n, dtype=torch.float32, device=dev)
    r_ref, v_ref, d_ref = np.zeros(n, F32), np.zeros(n, F32), np.zeros(n, F32)
    rng = np.random.default_rng(15)
    sent = 0
    for step in range(2):
        sg = np.repeat(sig, sizes)
        z = rng.standard_normal(n)
        g = (sg * z / np.sqrt(B)).astype(F32)
        s = (sg * sg * (rng.chisquare(B - 1, n) + z * z) / (B * B)).astype(F32)
        del z, sg
        vgc.accumulate_select_hybrid(torch.from_numpy(g).to(dev), torch.from_numpy(s).to(dev), r, v, plan, alpha, cfg["zeta"], tau, scratch)
        mask = plan.send_mask(scratch)
        vgc.pack(plan, scratch, words, hdrs, status)
        torch.cuda.synchronize()
        total, overflow = vgc.read_status(status)
        vgc.unpack_add(words, total, hdrs, plan, tau / 8, dense)
        r_ref, v_ref, send, sign = O.accumulate_select_hybrid(g, s, r_ref, v_ref, alpha, cfg["zeta"], tau)
        w_ref, h_ref = O.pack_hybrid(sign, send, groups)
        O.unpack_add(w_ref, h_ref, groups, tau / 8, d_ref)
        assert np.array_equal(mask, send)
        assert overflow == 0 and total == w_ref.size and vgc.read_headers(hdrs) == h_ref
        assert np.array_equal(words[:total].cpu().numpy().view(U32), w_ref)
        assert np.array_equal(_bits(r.cpu().numpy()), _bits(r_ref)) and np.array_equal(_bits(v.cpu().numpy()), _bits(v_ref))
        torch.cuda.synchronize()
        assert np.array_equal(_bits(dense.cpu().numpy()), _bits(d_ref))
        sent += total
    assert sent > 0


def test_group_of_maximum_size(dev):
    """One group of exactly 2^28 elements (the most a 28-bit index can address, Section 4.2), sixteen scan
    segments, followed by a small group: every output against the oracle, and the last index uses all 28 bits."""
    import torch
    from paper_1802_06058_amd import vgc
    sizes = [1 << 28, 1000]
    groups = W.groups_from_sizes(sizes)
    n = sum(sizes)
    plan = vgc.Plan(groups, dev)
    rng = np.random.default_rng(28)
    g = rng.standard_normal(n, dtype=F32)
    g *= F32(0.01)
    s = rng.random(n, dtype=F32)
    s *= F32(2e-4)
    g[(1 << 28) - 1] = F32(1.0)                                   # the last element of the big group is sent for sure
    r = torch.zeros(n, dtype=torch.float32, device=dev); v = torch.zeros(n, dtype=torch.float32, device=dev)
    scratch, hdrs, status = plan.new_scratch(), plan.new_headers(), plan.new_status()
    words = torch.empty(n // 2, dtype=torch.int32, device=dev)
    vgc.accumulate_select(torch.from_numpy(g).to(dev), torch.from_numpy(s).to(dev), r, v, plan, 2.0, 0.999, scratch)
    vgc.pack(plan, scratch, words, hdrs, status)
    torch.cuda.synchronize()
    total, overflow = vgc.read_status(status)
    z = np.zeros(n, F32)
    r_acc, r_ref, v_ref, send = O.accumulate_select(g, s, z, z, 2.0, 0.999)
    del z
    w_ref, h_ref, _ = O.pack(r_acc, send, groups, check=False)
    assert overflow == 0 and total == w_ref.size and vgc.read_headers(hdrs) == h_ref
    got = words[:total].cpu().numpy().view(U32)
    assert np.array_equal(got, w_ref)
    assert (got[h_ref[0][1] - 1] & U32(0x0FFFFFFF)) == U32(0x0FFFFFFF)
    assert np.array_equal(_bits(r.cpu().numpy()), _bits(r_ref)) and np.array_equal(_bits(v.cpu().numpy()), _bits(v_ref))


@pytest.mark.parametrize("name,alpha,steps", [("C3", 1.0, 20), ("C4", 0.5, 1), ("C4", 1.0, 1), ("C4", 2.0, 2), ("C4", 4.0, 1)])
def test_model_parameter_sets_full_oracle(dev, name, alpha, steps):
    """ResNet-50-shaped (161 groups, 25.6 M; all 20 iterations of the configuration, state carried) and
    VGG-16-shaped (32 groups, 138 M; every alpha of the configuration's sweep) parameter sets with per-layer
    gradient scales: every output of every step compared with the oracle."""
    import torch
    from paper_1802_06058_amd import vgc
    cfg = W.CONFIGS[name]
    layers = cfg["layers"]
    groups = W.groups_from_sizes([L["size"] for L in layers])
    plan = vgc.Plan(groups, dev)
    n = plan.n
    sig = W.layer_sigmas(cfg["seed"], len(layers))
    r = torch.zeros(n, dtype=torch.float32, device=dev)
    v = torch.zeros(n, dtype=torch.float32, device=dev)
    scratch = plan.new_scratch()
    words = torch.empty(n, dtype=torch.int32, device=dev)
    hdrs, status = plan.new_headers(), plan.new_status()
    r_ref, v_ref = np.zeros(n, F32), np.zeros(n, F32)
    dense = torch.zeros(n, dtype=torch.float32, device=dev)
    d_ref = np.zeros(n, F32)
    rng = np.random.default_rng(5)
    for step in range(steps):
        # (g, s) with the distribution of `batch` i.i.d. N(0, sigma_l^2) samples, drawn directly:
        # mean = sigma z / sqrt(B), sum of squares of y/B = sigma^2 (chi2_{B-1} + z^2) / B^2
        B = cfg["batch"]
        sg = np.repeat(sig, [L["size"] for L in layers])
        z = rng.standard_normal(n)
        g = (sg * z / np.sqrt(B)).astype(F32)
        s = (sg * sg * (rng.chisquare(B - 1, n) + z * z) / (B * B)).astype(F32)
        del z, sg
        gd, sd = torch.from_numpy(g).to(dev), torch.from_numpy(s).to(dev)
        vgc.accumulate_select(gd, sd, r, v, plan, alpha, cfg["zeta"], scratch)
        mask = plan.send_mask(scratch)
        vgc.pack(plan, scratch, words, hdrs, status)
        torch.cuda.synchronize()
        total, overflow = vgc.read_status(status)
        vgc.unpack_add(words, total, hdrs, plan, 1.0 / 16, dense)
        r_acc, r_ref, v_ref, send = O.accumulate_select(g, s, r_ref, v_ref, alpha, cfg["zeta"])
        w_ref, h_ref, _ = O.pack(r_acc, send, groups, check=False)
        O.unpack_add(w_ref, h_ref, groups, 1.0 / 16, d_ref)
        assert np.array_equal(mask, send)
        assert overflow == 0 and total == w_ref.size
        assert vgc.read_headers(hdrs) == h_ref
        assert np.array_equal(words[:total].cpu().numpy().view(U32), w_ref)
        assert np.array_equal(_bits(r.cpu().numpy()), _bits(r_ref))
        assert np.array_equal(_bits(v.cpu().numpy()), _bits(v_ref))
        torch.cuda.synchronize()
        assert np.array_equal(_bits(dense.cpu().numpy()), _bits(d_ref))


@pytest.mark.parametrize("B,P,J,C,prec", [(64, 784, 4608, 512, "bf16"), (64, 196, 4608, 512, "bf16"),
                                          (32, 3136, 576, 64, "f32"), (32, 196, 2304, 256, "f32")])
def test_conv_statistic_every_output_at_config_shapes(dev, B, P, J, C, prec):
    """3x3 convolution shapes of the VGG-16 (bf16, batch 64) and ResNet-50 (float32, batch 32) configs as patch
    matrices, in the launch configuration the benchmark times: every output of s against the float64 oracle at the
    stated relative tolerance (1e-2 / 1e-5), every output of g against the magnitudes summed."""
    import torch
    from paper_1802_06058_amd import vgc
    bf16 = prec == "bf16"
    gen = torch.Generator(device=dev)
    gen.manual_seed(B * 7 + P)
    dt = torch.bfloat16 if bf16 else torch.float32
    U = torch.randn((B, P, J), generator=gen, device=dev, dtype=torch.float32).to(dt)
    D = (torch.randn((B, P, C), generator=gen, device=dev, dtype=torch.float32) * 3e-3).to(dt)
    s = torch.empty(J, C, dtype=torch.float32, device=dev)
    g = torch.empty(J, C, dtype=torch.float32, device=dev)
    nb = vgc.sqgrad_workspace_bytes(vgc.CONV, vgc.BF16 if bf16 else vgc.F32, B, P, J, C)
    ws = torch.empty(max(nb, 16), dtype=torch.uint8, device=dev)
    vgc.sqgrad(vgc.CONV, U, D, 1.0 / B, s, g, workspace=ws if nb else None)
    s_only = torch.empty_like(s)
    vgc.sqgrad(vgc.CONV, U, D, 1.0 / B, s_only, None, workspace=ws if nb else None)
    torch.cuda.synchronize()
    tol = 1e-2 if bf16 else 1e-5
    sh, gh = s.cpu().numpy(), g.cpu().numpy()
    Uh, Dh = U.to(torch.float32).cpu().numpy(), D.to(torch.float32).cpu().numpy()      # exact widening
    del U, D
    g64, s64 = O.sqgrad_conv(Uh, Dh, 1.0 / B)
    assert (s64 > 0).all()
    rel = np.abs(sh - s64) / s64
    print(f"observed max rel err of s: conv {prec} B{B} P{P} J{J} C{C}: {rel.max():.3e}")
    assert rel.max() <= tol, f"s relative error {rel.max():.3e} at {np.unravel_index(rel.argmax(), rel.shape)}"
    absG = np.zeros((J, C))
    for z in range(B):                                             # a scale, not a reference: float32 is enough
        absG += np.abs(Uh[z]).T @ np.abs(Dh[z])
    assert (np.abs(gh - g64) / (absG / B)).max() <= tol
    assert np.array_equal(s_only.cpu().numpy(), sh)                 # the kernel the benchmark times (s alone)
