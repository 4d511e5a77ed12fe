"""vgc_sqgrad_noalloc (the entry point for callers that cannot allocate: its working memory is a static buffer
inside the library's device image) against vgc_sqgrad with a caller workspace: same kernels, so every output
must agree bit for bit, on calls in a row that reuse the buffer, a smaller input after a larger one."""
import numpy as np
import pytest

from paper_1802_06058_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dev():
    import torch
    from paper_1802_06058_amd import vgc
    assert torch.cuda.is_available()
    vgc.load()
    return torch.device("cuda:0")


def _both(kind, B, P, J, C, bf16, dev, seed):
    """(g, s) from vgc_sqgrad with a workspace of its own and from vgc_sqgrad_noalloc, as host arrays, plus the
    workspace size the shape asks for."""
    import torch
    from paper_1802_06058_amd import vgc
    if kind == vgc.FC:
        X, D = W.fc_inputs(seed, (B, J, C), B, J, C, "normal", False, 0.02, bf16=bf16)
    else:
        X, D = W.conv_inputs(seed, (B, P, J, C), B, P, J, C, d_sigma=0.02, bf16=bf16)
    Xd, Dd = torch.from_numpy(X).to(dev), torch.from_numpy(D).to(dev)
    if bf16:
        Xd, Dd = Xd.view(torch.bfloat16), Dd.view(torch.bfloat16)
    nb = vgc.sqgrad_workspace_bytes(kind, vgc.BF16 if bf16 else vgc.F32, B, P, J, C)
    ws = torch.full((max(nb, 16),), 0xFF, dtype=torch.uint8, device=dev)
    out = []
    for call in ("workspace", "noalloc"):
        s = torch.full((J, C), float("nan"), dtype=torch.float32, device=dev)
        g = torch.full((J, C), float("nan"), dtype=torch.float32, device=dev)
        if call == "workspace":
            vgc.sqgrad(kind, Xd, Dd, 1.0 / B, s, g, workspace=ws if nb else None)
        else:
            vgc.sqgrad_noalloc(kind, Xd, Dd, 1.0 / B, s, g)
        torch.cuda.synchronize()
        out.append((g.cpu().numpy(), s.cpu().numpy()))
    return out[0], out[1], nb


def test_noalloc_equals_workspace_call_on_calls_in_a_row(dev):
    from paper_1802_06058_amd import vgc
    # (kind, B, P, J, C, bf16): samples split over workgroups (partial sums through the buffer), then a smaller
    # shape of the same kind, positions split (unsquared partial products through the buffer), then shapes that
    # need no working memory at all
    cases = [(vgc.CONV, 16, 196, 1152, 256, False), (vgc.CONV, 8, 49, 576, 64, False),
             (vgc.CONV, 16, 196, 1152, 256, True), (vgc.CONV, 6, 33, 200, 136, True),
             (vgc.CONV, 8, 2000, 64, 72, False), (vgc.CONV, 3, 1111, 24, 16, True),
             (vgc.FC, 32, 1, 512, 384, False), (vgc.CONV, 2, 9, 40, 24, False)]
    used = 0
    for i, (kind, B, P, J, C, bf16) in enumerate(cases):
        (g0, s0), (g1, s1), nb = _both(kind, B, P, J, C, bf16, dev, 70 + i)
        assert nb <= vgc.NOALLOC_SCRATCH_BYTES
        used += nb > 0
        assert np.isfinite(s1).all() and np.isfinite(g1).all()
        assert np.array_equal(s0.view(np.uint32), s1.view(np.uint32)), f"s differs in case {i}"
        assert np.array_equal(g0.view(np.uint32), g1.view(np.uint32)), f"g differs in case {i}"
    assert used >= 4                                   # the buffer really was exercised


def test_noalloc_refuses_shapes_beyond_its_buffer(dev):
    import torch
    from paper_1802_06058_amd import vgc
    B, P, J, C = 8, 49, 9216, 1024                     # 9.4 M outputs, eight-way sample split: 288 MiB of partial sums
    nb = vgc.sqgrad_workspace_bytes(vgc.CONV, vgc.F32, B, P, J, C)
    assert nb > vgc.NOALLOC_SCRATCH_BYTES
    lib = vgc.load()
    x = torch.zeros(16, device=dev)
    s = torch.full((16,), 7.0, device=dev)
    rc = lib.vgc_sqgrad_noalloc(vgc.CONV, vgc.F32, x.data_ptr(), x.data_ptr(), B, P, J, C, 1.0, None, s.data_ptr(), None)
    assert rc == -2 and b"static buffer" in lib.vgc_last_error()
    torch.cuda.synchronize()
    assert float(s.sum()) == 7.0 * 16                  # nothing was launched
