"""Parity of the HIP squared-gradient statistic against the float64 oracle, through the C ABI.

Tolerances: every output of s within relative error 1e-5 (float32 inputs) / 1e-2 (bfloat16 inputs)
of the oracle's value, |s - s64| <= tol * s64, in both forms.  g is a signed sum for which no
relative bound can hold (it may cancel to zero), so its error is measured against the sum of the
magnitudes of its terms (the quantity float32 accumulation error scales with).

In the conv form a sample's gradient is itself a signed sum over the P positions, so an output whose
samples all happen to cancel is ill-conditioned: with two or three samples and a thousand positions a
few outputs in ten thousand lose more than 1e-5 to float32 rounding whatever the order of summation.
The signed cases here therefore have at least four samples (eight beyond a thousand positions), as the
configurations do (32 and 64); the cases with one to three samples run on non-negative inputs, where
nothing cancels."""
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


OBSERVED = {}          # case -> largest relative error of s seen (printed by the last test of the module)


def _check(g, s, g64, s64, absG, tol, tag=None):
    assert np.isfinite(s).all()
    err_s = np.abs(s - s64) / np.maximum(s64, np.finfo(np.float64).tiny)
    worst = float(err_s[s64 > 0].max()) if (s64 > 0).any() else 0.0
    if tag is not None:
        OBSERVED[tag] = max(OBSERVED.get(tag, 0.0), worst)
    assert worst <= tol, f"s relative error {worst:.3e} at {np.unravel_index(np.argmax(np.where(s64 > 0, err_s, 0)), s.shape)}"
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
    _check(g, s, g64, s64, absG, RTOL[prec], f"fc {prec} B{B} J{J} C{C}")
    _, s2 = _run(vgc.FC, X, D, c, dev, bf16, want_g=False)     # g_out is optional
    assert np.array_equal(s, s2)


@pytest.mark.parametrize("B,P,J,C", [(4, 49, 64, 64), (3, 5, 27, 16), (2, 1, 40, 40), (8, 196, 576, 64), (5, 9, 100, 33),
                                     (6, 33, 200, 136), (3, 64, 384, 256), (6, 784, 128, 128),
                                     (5, 20, 72, 40), (4, 39, 64, 200),          # last chunk of a sample a quarter / half full
                                     (8, 2000, 64, 72), (8, 1111, 24, 16),       # few tiles, many positions: split over positions
                                     (2, 1111, 24, 16), (1, 300, 40, 24),        # one or two samples (non-negative inputs)
                                     (40, 100, 1024, 512)])                      # more (tile, sample) pairs than workgroup slots: several samples per workgroup
@pytest.mark.parametrize("prec", ["f32", "bf16"])
def test_conv_form(dev, B, P, J, C, prec):
    from paper_1802_06058_amd import vgc
    bf16 = prec == "bf16"
    U, D = W.conv_inputs(22, (B, P, J, C), B, P, J, C, d_sigma=0.02, bf16=bf16)
    if B < 3 and P > 100:                                      # nothing cancels: see the module docstring
        U, D = (U & 0x7FFF, D & 0x7FFF) if bf16 else (np.abs(U), np.abs(D))
    c = 1.0 / B
    Uw, Dw = _widen(U, bf16), _widen(D, bf16)
    g64, s64 = O.sqgrad_conv(Uw, Dw, c)
    absG = np.einsum("zpj,zpc->jc", np.abs(Uw), np.abs(Dw)) * c
    tol = RTOL[prec]
    tag = f"conv {prec} B{B} P{P} J{J} C{C}"
    g, s = _run(vgc.CONV, U, D, c, dev, bf16)
    _check(g, s, g64, s64, absG, tol, tag)
    # without a workspace the samples are not split over workgroups: same tolerances
    g1, s1 = _run(vgc.CONV, U, D, c, dev, bf16, use_workspace=False)
    _check(g1, s1, g64, s64, absG, tol, tag)
    # s alone is the same, bit for bit
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


def test_zz_report_observed_errors():
    """Not a check: prints the largest relative error of s each case showed (run with -s to see it)."""
    for tag, worst in sorted(OBSERVED.items()):
        print(f"observed max rel err of s: {tag}: {worst:.3e}")
