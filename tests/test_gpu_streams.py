"""The statistic of several layers issued on several streams at once, each call with a workspace of its own,
against the same calls issued one after another: the layers of a network are independent and a caller may overlap them."""
import numpy as np
import pytest

from paper_1802_06058_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dev():
    import torch
    from paper_1802_06058_amd import vgc
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    vgc.load()
    return torch.device("cuda:0")


LAYERS = [  # B, H, W, Cin, C, k, stride, pad, bf16
    (8, 28, 28, 64, 64, 3, 1, 1, True),
    (8, 28, 28, 64, 128, 1, 1, 0, True),
    (8, 14, 14, 128, 128, 3, 2, 1, True),
    (6, 28, 28, 32, 64, 3, 1, 1, False),
    (6, 14, 14, 64, 256, 1, 1, 0, False),
    (6, 56, 56, 16, 16, 3, 1, 1, False),
]


def test_layers_on_three_streams_equal_serial(dev):
    import torch
    from paper_1802_06058_amd import vgc
    from oracle import vgc_oracle as O
    calls = []
    for i, (B, H, Wd, Cin, C, k, st, pd, bf16) in enumerate(LAYERS):
        Ho, Wo = O.conv_out_size(H, k, st, pd), O.conv_out_size(Wd, k, st, pd)
        A, D = W.conv2d_inputs(70 + i, (i,), B, H, Wd, Cin, Ho, Wo, C, d_sigma=0.02, bf16=bf16)
        At, Dt = torch.from_numpy(np.ascontiguousarray(A)).to(dev), torch.from_numpy(np.ascontiguousarray(D)).to(dev)
        if bf16:
            At, Dt = At.view(torch.bfloat16), Dt.view(torch.bfloat16)
        code = vgc.BF16 if bf16 else vgc.F32
        nb = vgc.sqgrad_conv2d_workspace_bytes(code, B, H, Wd, Cin, C, k, k, (st, st), (pd, pd))
        J = k * k * Cin

        def make(J=J, C=C, nb=nb):                                     # (bound now: the loop variables move on)
            s = torch.full((J, C), float("nan"), dtype=torch.float32, device=dev)
            ws = torch.full((max(nb, 1),), 0xFF, dtype=torch.uint8, device=dev) if nb else None
            return s, ws
        calls.append((At, Dt, k, st, pd, B, make))

    def run(streams):
        outs = []
        torch.cuda.synchronize()
        for rep in range(3):                                       # several rounds so that kernels of different layers meet
            for i, (At, Dt, k, st, pd, B, make) in enumerate(calls):
                s, ws = make()
                ctx = torch.cuda.stream(streams[i % len(streams)]) if streams else torch.cuda.stream(torch.cuda.current_stream())
                with ctx:
                    vgc.sqgrad_conv2d(At, Dt, k, k, (st, st), (pd, pd), 1.0 / B, s, None, workspace=ws)
                outs.append((s, ws))
        torch.cuda.synchronize()
        return [s.cpu().numpy() for s, _ in outs]

    serial = run(None)
    overlapped = run([torch.cuda.Stream() for _ in range(3)])
    for a, b in zip(serial, overlapped):
        assert np.isfinite(a).all()
        assert np.array_equal(a, b)
