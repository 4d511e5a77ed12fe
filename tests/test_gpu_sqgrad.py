"""Parity of the HIP squared-gradient statistic against the float64 oracle, through the C ABI.

Tolerances (stated by the benchmark spec): s to relative error 1e-5 for float32 inputs and
1e-2 for bfloat16 inputs.  g is a signed sum, so its error is measured against the sum of the
magnitudes of its terms (the quantity float32 accumulation error scales with)."""
import numpy as np
import pytest

from oracle import vgc_oracle as O
from paper_1802_06058_amd import workloads as W

pytestmark = pytest.mark.gpu

RTOL = {"f32": 1e-5, "bf16": 1e-2}


@pytest.fixture(scope="module")
def dev():
    import torch
    from paper_1802_06058_amd import vgc
    assert torch.cuda.is_available()
    vgc.load()
    return torch.device("cuda:0")


def _to_dev(a, dev, bf16):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    return t.view(torch.bfloat16) if bf16 else t


def _run(kind, X, D, c, dev, bf16, want_g=True, use_workspace=True):
    import torch
    from paper_1802_06058_amd import vgc
    Xd, Dd = _to_dev(X, dev, bf16), _to_dev(D, dev, bf16)
    J, C = X.shape[-1], D.shape[-1]
    s = torch.full((J, C), float("nan"), dtype=torch.float32, device=dev)
    g = torch.full((J, C), float("nan"), dtype=torch.float32, device=dev) if want_g else None
    ws = None
    if use_workspace:
        B = X.shape[0]
        P = X.shape[1] if kind == vgc.CONV else 1
        nb = vgc.sqgrad_workspace_bytes(kind, vgc.BF16 if bf16 else vgc.F32, B, P, J, C)
        if nb:
            ws = torch.full((nb,), 0xFF, dtype=torch.uint8, device=dev)
    vgc.sqgrad(kind, Xd, Dd, c, s, g, workspace=ws)
    torch.cuda.synchronize()
    return (g.cpu().numpy() if want_g else None), s.cpu().numpy()


def _check(g, s, g64, s64, absG, tol):
    assert np.isfinite(s).all()
    err_s = np.abs(s - s64) / np.maximum(s64, np.finfo(np.float64).tiny)
    assert err_s[s64 > 0].max() <= tol, f"s relative error {err_s[s64 > 0].max():.3e}"
    assert np.all(s[s64 == 0] == 0)
    if g is not None:
        err_g = np.abs(g - g64) / np.maximum(absG, np.finfo(np.float64).tiny)
        assert err_g.max() <= tol, f"g error {err_g.max():.3e}"


def _widen(a, bf16):
    return W.bf16_bits_to_f32(a).astype(np.float64) if bf16 else a.astype(np.float64)


@pytest.mark.parametrize("B,J,C", [(32, 1024, 1024), (128, 784, 1000), (128, 1000, 10), (1, 5, 3), (7, 33, 65), (64, 2500, 300)])
@pytest.mark.parametrize("prec", ["f32", "bf16"])
def test_fc_form(dev, B, J, C, prec):
    from paper_1802_06058_amd import vgc
    bf16 = prec == "bf16"
    X, D = W.fc_inputs(21, (B, J, C), B, J, C, "normal", relu_sparse=(J % 2 == 0), d_sigma=0.01, bf16=bf16)
    c = 1.0 / B
    Xw, Dw = _widen(X, bf16), _widen(D, bf16)
    g64, s64 = O.sqgrad_fc(Xw, Dw, c)
    absG = (np.abs(Xw).T @ np.abs(Dw)) * c
    g, s = _run(vgc.FC, X, D, c, dev, bf16)
    _check(g, s, g64, s64, absG, RTOL[prec])
    _, s2 = _run(vgc.FC, X, D, c, dev, bf16, want_g=False)     # g_out is optional
    assert np.array_equal(s, s2)


@pytest.mark.parametrize("B,P,J,C", [(4, 49, 64, 64), (3, 5, 27, 16), (2, 1, 40, 40), (8, 196, 576, 64), (5, 9, 100, 33),
                                     (6, 33, 200, 136), (3, 64, 384, 256), (2, 784, 128, 128),
                                     (3, 2000, 64, 72), (2, 1111, 24, 16),       # few tiles, many positions: split over positions
                                     (40, 100, 1024, 512)])                      # more (tile, sample) pairs than workgroup slots: several samples per workgroup
@pytest.mark.parametrize("prec", ["f32", "bf16"])
def test_conv_form(dev, B, P, J, C, prec):
    from paper_1802_06058_amd import vgc
    bf16 = prec == "bf16"
    U, D = W.conv_inputs(22, (B, P, J, C), B, P, J, C, d_sigma=0.02, bf16=bf16)
    c = 1.0 / B
    Uw, Dw = _widen(U, bf16), _widen(D, bf16)
    g64, s64 = O.sqgrad_conv(Uw, Dw, c)
    absG = np.einsum("zpj,zpc->jc", np.abs(Uw), np.abs(Dw)) * c
    g, s = _run(vgc.CONV, U, D, c, dev, bf16)
    # the per-sample gradient is a signed sum over positions: its float32 error scales with the
    # magnitudes summed, and s inherits twice that relative to (sum |terms|)^2
    tol = RTOL[prec]
    err_g = np.abs(g - g64) / absG
    assert err_g.max() <= tol
    sabs = np.einsum("zjc->jc", np.einsum("zpj,zpc->zjc", np.abs(Uw), np.abs(Dw)) ** 2) * c * c
    assert (np.abs(s - s64) / sabs).max() <= tol
    well = s64 > 0.05 * sabs                                   # where cancellation is mild, plain relative error
    if prec == "f32" and well.any():
        assert (np.abs(s - s64)[well] / s64[well]).max() <= 20 * tol
    # without a workspace the samples are not split over workgroups; same tolerances, and s alone is the same
    g1, s1 = _run(vgc.CONV, U, D, c, dev, bf16, use_workspace=False)
    assert (np.abs(g1 - g64) / absG).max() <= tol and (np.abs(s1 - s64) / sabs).max() <= tol
    _, s2 = _run(vgc.CONV, U, D, c, dev, bf16, want_g=False)
    assert np.array_equal(s, s2)
    # ... also when one workgroup walks through all the samples (the s-only kernel has a loop of its own)
    _, s3 = _run(vgc.CONV, U, D, c, dev, bf16, want_g=False, use_workspace=False)
    assert np.array_equal(s1, s3)


def test_sampled_outputs_at_vgg_fc6_shape(dev):
    """Largest FC layer of config 4 (25088 x 4096, batch 64, bfloat16): outputs are sampled and
    each is recomputed on the CPU from the definition, one per-sample gradient at a time."""
    from paper_1802_06058_amd import vgc
    B, J, C = 64, 25088, 4096
    X, D = W.fc_inputs(23, (0,), B, J, C, "normal", relu_sparse=True, d_sigma=1e-3, bf16=True)
    g, s = _run(vgc.FC, X, D, 1.0 / B, dev, True)
    Xw, Dw = _widen(X, True), _widen(D, True)
    rng = np.random.default_rng(0)
    jj = np.concatenate([rng.integers(0, J, 400), [0, J - 1, J - 1, 0]])
    cc = np.concatenate([rng.integers(0, C, 400), [0, C - 1, 0, C - 1]])
    for j, c_ in zip(jj, cc):
        per_sample = Xw[:, j] * Dw[:, c_] / B
        s_ref, g_ref = (per_sample ** 2).sum(), per_sample.sum()
        assert abs(s[j, c_] - s_ref) <= 1e-2 * s_ref
        assert abs(g[j, c_] - g_ref) <= 1e-2 * np.abs(per_sample).sum() + 1e-30


def test_rejects_bad_arguments(dev):
    import torch
    from paper_1802_06058_amd import vgc
    X = torch.zeros(4, 8, device=dev)
    D = torch.zeros(4, 8, device=dev)
    s = torch.zeros(8, 8, device=dev)
    lib = vgc.load()
    import ctypes as C
    rc = lib.vgc_sqgrad(vgc.FC, 7, X.data_ptr(), D.data_ptr(), 4, 1, 8, 8, 1.0, None, s.data_ptr(), None, 0, None)
    assert rc == -4
    rc = lib.vgc_sqgrad(vgc.FC, vgc.F32, X.data_ptr(), D.data_ptr(), 4, 2, 8, 8, 1.0, None, s.data_ptr(), None, 0, None)
    assert rc == -2
    rc = lib.vgc_sqgrad(vgc.FC, vgc.F32, X.data_ptr(), None, 4, 1, 8, 8, 1.0, None, s.data_ptr(), None, 0, None)
    assert rc == -1 and b"required" in lib.vgc_last_error()
