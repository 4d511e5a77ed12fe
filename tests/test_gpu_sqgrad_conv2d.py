"""vgc_sqgrad_conv2d (the convolution statistic read from the NHWC input, no patch matrix) against the
float64 oracle, and against vgc_sqgrad on the materialised patch matrix.  Every output of s within relative
error 1e-2 (bfloat16 inputs) / 1e-5 (float32 inputs) of the oracle's, |s - s64| <= tol * s64; g, a signed sum,
against the magnitudes summed.  Signed inputs come with at least four samples, the geometries with one to
three samples with non-negative inputs (a sample's gradient is a signed sum over the positions: with so few
samples some outputs cancel to where no float32 summation keeps 1e-5; see tests/test_gpu_sqgrad.py)."""
import numpy as np
import pytest

from oracle import vgc_oracle as O
from paper_1802_06058_amd import workloads as W

pytestmark = pytest.mark.gpu
RTOL = {"bf16": 1e-2, "f32": 1e-5}


@pytest.fixture(scope="module")
def dev():
    import torch
    from paper_1802_06058_amd import vgc
    assert torch.cuda.is_available()
    vgc.load()
    return torch.device("cuda:0")


def _bf(a, dev):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).to(dev).view(torch.bfloat16)


def _in(a, dev):
    import torch
    return _bf(a, dev) if a.dtype == np.uint16 else torch.from_numpy(np.ascontiguousarray(a)).to(dev)


def _run(A, D, kh, kw, stride, pad, c, dev, want_g=True, use_workspace=True):
    import torch
    from paper_1802_06058_amd import vgc
    dtype = vgc.BF16 if A.dtype == np.uint16 else vgc.F32
    B, H, Wd, Cin = A.shape
    C = D.shape[3]
    J = kh * kw * Cin
    s = torch.full((J, C), float("nan"), dtype=torch.float32, device=dev)
    g = torch.full((J, C), float("nan"), dtype=torch.float32, device=dev) if want_g else None
    ws = None
    if use_workspace:
        nb = vgc.sqgrad_conv2d_workspace_bytes(dtype, B, H, Wd, Cin, C, kh, kw, stride, pad)
        if nb:
            ws = torch.full((nb,), 0xFF, dtype=torch.uint8, device=dev)
    vgc.sqgrad_conv2d(_in(A, dev), _in(D, dev), kh, kw, stride, pad, c, s, g, workspace=ws)
    torch.cuda.synchronize()
    return (g.cpu().numpy() if want_g else None), s.cpu().numpy()


def _patches(a, kh, kw, stride, pad, Ho, Wo):
    """[B, Ho*Wo, kh*kw*Cin] patch matrix of a float array, zero padded (test-side helper)."""
    B, H, Wd, Cin = a.shape
    ap = np.zeros((B, H + 2 * pad[0], Wd + 2 * pad[1], Cin), a.dtype)
    ap[:, pad[0]:pad[0] + H, pad[1]:pad[1] + Wd] = a
    cols = [ap[:, ky:ky + stride[0] * (Ho - 1) + 1:stride[0], kx:kx + stride[1] * (Wo - 1) + 1:stride[1]]
            for ky in range(kh) for kx in range(kw)]
    return np.concatenate(cols, axis=3).reshape(B, Ho * Wo, kh * kw * Cin)


GEOMS = [  # B, H, W, Cin, C, kh, kw, stride, pad
    (3, 8, 8, 8, 16, 3, 3, (1, 1), (1, 1)),        # one tile, taps narrower than the 16-byte pieces' tile
    (4, 14, 14, 64, 64, 3, 3, (1, 1), (1, 1)),     # VGG-like, small
    (4, 9, 7, 16, 24, 3, 3, (2, 2), (1, 1)),       # stride 2, ragged everything
    (4, 12, 10, 32, 40, 1, 1, (1, 1), (0, 0)),     # 1x1
    (5, 11, 13, 8, 8, 5, 3, (2, 1), (2, 0)),       # rectangular kernel, mixed stride and padding
    (2, 6, 1, 24, 16, 3, 1, (1, 1), (1, 0)),       # output one column wide
    (8, 28, 28, 128, 136, 3, 3, (1, 1), (1, 1)),   # several row tiles and a ragged column tile, samples split
    (6, 16, 16, 256, 128, 3, 3, (1, 1), (1, 1)),   # a 256-column tile inside one tap
    (8, 40, 37, 16, 16, 3, 3, (1, 1), (1, 1)),     # one tile, 1480 positions: the positions are split over workgroups
    (8, 64, 50, 8, 24, 3, 3, (2, 1), (1, 1)),      # the same with a stride
    (8, 39, 27, 112, 96, 5, 5, (3, 1), (3, 1)),    # 5x5, stride 3 down, padding larger than the stride
    (5, 9, 11, 144, 128, 2, 5, (1, 2), (1, 2)),    # even kernel height, wide kernel
    (6, 23, 31, 32, 24, 4, 2, (3, 3), (0, 0)),     # stride larger than the kernel's width: input columns skipped
    (1, 73, 72, 32, 32, 5, 4, (1, 2), (0, 0)),     # one sample, 2415 positions
    (2, 40, 37, 16, 16, 3, 3, (1, 1), (1, 1)),     # two samples, positions split
    (4, 12, 25, 16, 24, 3, 3, (1, 1), (0, 1)),     # unit strides, output as wide as the input but less high; column pattern of period 25
    (3, 10, 20, 8, 16, 1, 3, (1, 1), (0, 1)),      # one kernel row, period 5
    (2, 30, 96, 8, 8, 3, 3, (1, 1), (1, 1)),       # width a multiple of the chunk: period 3, positions split
]

OBSERVED = {}


def _rel_s(s, s64):
    ok = s64 > 0
    return float((np.abs(s - s64)[ok] / s64[ok]).max()) if ok.any() else 0.0


@pytest.mark.parametrize("prec", ["bf16", "f32"])
@pytest.mark.parametrize("geom", GEOMS)
def test_conv2d_matches_oracle(dev, geom, prec):
    B, H, Wd, Cin, C, kh, kw, stride, pad = geom
    TOL = RTOL[prec]
    Ho, Wo = O.conv_out_size(H, kh, stride[0], pad[0]), O.conv_out_size(Wd, kw, stride[1], pad[1])
    A, D = W.conv2d_inputs(41, geom[:7], B, H, Wd, Cin, Ho, Wo, C, d_sigma=0.02, bf16=prec == "bf16")
    if B < 4 and Ho * Wo > 100:                     # nothing cancels: see the module docstring
        A, D = (A & 0x7FFF, D & 0x7FFF) if prec == "bf16" else (np.abs(A), np.abs(D))
    if prec == "bf16":
        Aw, Dw = W.bf16_bits_to_f32(A).astype(np.float64), W.bf16_bits_to_f32(D).astype(np.float64)
    else:
        Aw, Dw = A.astype(np.float64), D.astype(np.float64)
    c = 1.0 / B
    g64, s64 = O.sqgrad_conv_nhwc(Aw, Dw, kh, kw, stride, pad, c)
    Uabs = _patches(np.abs(Aw), kh, kw, stride, pad, Ho, Wo)
    absG = np.einsum("zpj,zpc->jc", Uabs, np.abs(Dw).reshape(B, Ho * Wo, C)) * c
    tag = f"conv2d {prec} {geom}"
    g, s = _run(A, D, kh, kw, stride, pad, c, dev)
    assert np.isfinite(g).all() and np.isfinite(s).all()
    assert (np.abs(g - g64) / np.maximum(absG, 1e-300)).max() <= TOL
    OBSERVED[tag] = _rel_s(s, s64)
    assert OBSERVED[tag] <= TOL, f"s relative error {OBSERVED[tag]:.3e}"
    assert np.all(s[s64 == 0] == 0)
    # no workspace (no sample split), and s alone: same bounds; s alone equals s with g bit for bit
    g1, s1 = _run(A, D, kh, kw, stride, pad, c, dev, use_workspace=False)
    assert (np.abs(g1 - g64) / np.maximum(absG, 1e-300)).max() <= TOL and _rel_s(s1, s64) <= TOL
    _, s2 = _run(A, D, kh, kw, stride, pad, c, dev, want_g=False)
    assert np.array_equal(s2, s)
    # ... also when one workgroup walks through all the samples (the s-only kernel has a loop of its own)
    _, s3 = _run(A, D, kh, kw, stride, pad, c, dev, want_g=False, use_workspace=False)
    assert np.array_equal(s3, s1)


def test_conv2d_equals_patch_matrix_path(dev):
    """Same inputs through vgc_sqgrad on the materialised patch matrix: the two kernels multiply the same
    bfloat16 numbers and add them in float32 in the same order per output, so they agree to rounding noise."""
    import torch
    from paper_1802_06058_amd import vgc
    B, H, Wd, Cin, C, kh, kw, stride, pad = 4, 14, 14, 128, 128, 3, 3, (1, 1), (1, 1)
    Ho, Wo = 14, 14
    A, D = W.conv2d_inputs(42, (0,), B, H, Wd, Cin, Ho, Wo, C, d_sigma=0.02, bf16=True)
    g, s = _run(A, D, kh, kw, stride, pad, 1.0 / B, dev)
    U = _patches(A, kh, kw, stride, pad, Ho, Wo)
    J = kh * kw * Cin
    s_ref = torch.empty(J, C, dtype=torch.float32, device=dev); g_ref = torch.empty(J, C, dtype=torch.float32, device=dev)
    nb = vgc.sqgrad_workspace_bytes(vgc.CONV, vgc.BF16, B, Ho * Wo, J, C)
    ws = torch.empty(nb, dtype=torch.uint8, device=dev) if nb else None
    vgc.sqgrad(vgc.CONV, _bf(U, dev), _bf(D.reshape(B, Ho * Wo, C), dev), 1.0 / B, s_ref, g_ref, workspace=ws)
    torch.cuda.synchronize()
    assert np.array_equal(s, s_ref.cpu().numpy()) and np.array_equal(g, g_ref.cpu().numpy())


@pytest.mark.parametrize("B,H,Cin,C,prec", [(64, 28, 512, 512, "bf16"),      # VGG-16 conv4_2
                                            (64, 14, 512, 512, "bf16"),      # VGG-16 conv5_x
                                            (64, 112, 128, 128, "bf16"),     # VGG-16 conv2_2 (s alone: the nine-tap kernel)
                                            (64, 224, 64, 64, "bf16"),       # VGG-16 conv1_2 (the same, positions split)
                                            (32, 56, 64, 64, "f32"),         # ResNet-50 stage 1, 3x3
                                            (32, 14, 256, 256, "f32")])      # ResNet-50 stage 3, 3x3
def test_conv2d_every_output_at_config_shapes(dev, B, H, Cin, C, prec):
    """3x3 / stride 1 / pad 1 convolutions of the VGG-16 (bfloat16, batch 64) and ResNet-50 (float32, batch 32)
    configurations, in the launch configuration the benchmark times (workspace, s alone): every output of s
    against the oracle at the stated relative tolerance, every output of g against the magnitudes summed."""
    stride, pad = (1, 1), (1, 1)
    A, D = W.conv2d_inputs(43, (B, H, Cin, C), B, H, H, Cin, H, H, C, d_sigma=1e-3, bf16=prec == "bf16")
    Aw = W.bf16_bits_to_f32(A) if prec == "bf16" else A
    Dw = W.bf16_bits_to_f32(D) if prec == "bf16" else D
    g64, s64 = O.sqgrad_conv_nhwc(Aw, Dw, 3, 3, stride, pad, 1.0 / B)
    g, s = _run(A, D, 3, 3, stride, pad, 1.0 / B, dev)
    tol = RTOL[prec]
    tag = f"conv2d {prec} config shape B{B} {H}x{H}x{Cin}->{C}"
    OBSERVED[tag] = _rel_s(s, s64)
    assert OBSERVED[tag] <= tol, f"s relative error {OBSERVED[tag]:.3e}"
    absG = np.zeros_like(g64)
    Ap = np.zeros((B, H + 2, H + 2, Cin), np.float32); Ap[:, 1:H + 1, 1:H + 1] = np.abs(Aw)
    Dm = np.abs(Dw).reshape(B * H * H, C)
    for ky in range(3):
        for kx in range(3):
            win = Ap[:, ky:ky + H, kx:kx + H].reshape(B * H * H, Cin)
            absG[(ky * 3 + kx) * Cin:(ky * 3 + kx + 1) * Cin] = (win.T.astype(np.float64) @ Dm) / B
    assert (np.abs(g - g64) / np.maximum(absG, 1e-300)).max() <= tol
    _, s_only = _run(A, D, 3, 3, stride, pad, 1.0 / B, dev, want_g=False)    # the kernel the benchmark times
    if prec == "bf16" and Cin in (64, 128) and H % 16 == 0:                  # another kernel, another grouping of the samples
        OBSERVED[tag + " (s alone)"] = _rel_s(s_only, s64)
        assert OBSERVED[tag + " (s alone)"] <= tol
    else:
        assert np.array_equal(s_only, s)


TAP_GEOMS = [  # B, H, W, Cin, C: 3x3, stride 1, padding 1, 64 or 128 input channels, a width that is a multiple of 16
    (4, 16, 16, 64, 64),        # one tile, one half-chunk per output row: the column pattern has period 1
    (1, 16, 16, 64, 64),        # one sample
    (3, 6, 48, 64, 128),        # width 48: period 3; two column tiles
    (5, 9, 32, 128, 64),        # two channel blocks, odd height
    (2, 7, 16, 128, 192),       # 112 positions: the last chunk has one half only
    (8, 36, 32, 64, 64),        # 36 chunks per sample: the positions are split over workgroups
    (4, 24, 112, 64, 64),       # width 112 (period 7, a chunk straddles two rows), positions split ten ways
    (6, 10, 224, 64, 128),      # width 224 (period 7), as the first VGG layers
]


@pytest.mark.parametrize("geom", TAP_GEOMS)
def test_conv2d_tap_kernel_matches_oracle(dev, geom):
    """s alone of a 3x3 layer on 64 or 128 channels goes through the kernel that stages the input block of a chunk
    once for all nine taps: every output against the oracle at the stated tolerance; the call that also returns g
    (the generic kernel) and the call without a workspace agree with it to the same tolerance (they add the samples'
    squares in a different grouping, so not bit for bit)."""
    B, H, Wd, Cin, C = geom
    TOL = RTOL["bf16"]
    A, D = W.conv2d_inputs(44, geom, B, H, Wd, Cin, H, Wd, C, d_sigma=0.02, bf16=True)
    if B < 4:                                       # nothing cancels: see the module docstring
        A, D = A & 0x7FFF, D & 0x7FFF
    Aw, Dw = W.bf16_bits_to_f32(A).astype(np.float64), W.bf16_bits_to_f32(D).astype(np.float64)
    c = 1.0 / B
    g64, s64 = O.sqgrad_conv_nhwc(Aw, Dw, 3, 3, (1, 1), (1, 1), c)
    _, s = _run(A, D, 3, 3, (1, 1), (1, 1), c, dev, want_g=False)
    assert np.isfinite(s).all()
    tag = f"conv2d bf16 tap kernel {geom}"
    OBSERVED[tag] = _rel_s(s, s64)
    assert OBSERVED[tag] <= TOL, f"s relative error {OBSERVED[tag]:.3e}"
    assert np.all(s[s64 == 0] == 0)
    _, s_g = _run(A, D, 3, 3, (1, 1), (1, 1), c, dev, want_g=True)
    assert _rel_s(s_g, s64) <= TOL
    _, s_nows = _run(A, D, 3, 3, (1, 1), (1, 1), c, dev, want_g=False, use_workspace=False)
    assert _rel_s(s_nows, s64) <= TOL


STEM_GEOMS = [  # B, H, W, Cin, C, kh, kw, stride, pad: first layers, input channels not a multiple of 16 bytes
    (4, 12, 12, 3, 64, 3, 3, (1, 1), (1, 1)),      # an RGB input under a 3x3 filter
    (4, 20, 18, 3, 64, 7, 7, (2, 2), (3, 3)),      # ... under a 7x7 filter with stride 2: J = 147, five row tiles
    (5, 9, 11, 3, 24, 3, 3, (1, 1), (1, 1)),       # fewer than 64 output channels
    (4, 30, 31, 1, 8, 5, 5, (1, 1), (2, 2)),       # one input channel
    (4, 10, 10, 6, 72, 3, 3, (1, 1), (1, 1)),      # six channels, two ragged column tiles
    (8, 40, 40, 3, 64, 3, 3, (1, 1), (1, 1)),      # 1600 positions: split into parts
    (6, 33, 29, 2, 40, 4, 3, (3, 2), (0, 1)),      # two channels, uneven strides
]


@pytest.mark.parametrize("prec", ["bf16", "f32"])
@pytest.mark.parametrize("geom", STEM_GEOMS)
def test_conv2d_first_layer_matches_oracle(dev, geom, prec):
    """Layers whose input channels are not a multiple of 16 bytes (the kernel that gathers the patch rows element by
    element): every output of s against the oracle at the stated tolerance, g against the magnitudes summed, s alone
    equal to s with g; without the workspace the call is refused."""
    from paper_1802_06058_amd import vgc
    B, H, Wd, Cin, C, kh, kw, stride, pad = geom
    TOL = RTOL[prec]
    Ho, Wo = O.conv_out_size(H, kh, stride[0], pad[0]), O.conv_out_size(Wd, kw, stride[1], pad[1])
    A, D = W.conv2d_inputs(45, geom[:7], B, H, Wd, Cin, Ho, Wo, C, d_sigma=0.02, bf16=prec == "bf16")
    if prec == "bf16":
        Aw, Dw = W.bf16_bits_to_f32(A).astype(np.float64), W.bf16_bits_to_f32(D).astype(np.float64)
    else:
        Aw, Dw = A.astype(np.float64), D.astype(np.float64)
    c = 1.0 / B
    g64, s64 = O.sqgrad_conv_nhwc(Aw, Dw, kh, kw, stride, pad, c)
    Uabs = _patches(np.abs(Aw), kh, kw, stride, pad, Ho, Wo)
    absG = np.einsum("zpj,zpc->jc", Uabs, np.abs(Dw).reshape(B, Ho * Wo, C)) * c
    g, s = _run(A, D, kh, kw, stride, pad, c, dev)
    assert np.isfinite(g).all() and np.isfinite(s).all()
    assert (np.abs(g - g64) / np.maximum(absG, 1e-300)).max() <= TOL
    tag = f"conv2d {prec} first layer {geom}"
    OBSERVED[tag] = _rel_s(s, s64)
    assert OBSERVED[tag] <= TOL, f"s relative error {OBSERVED[tag]:.3e}"
    assert np.all(s[s64 == 0] == 0)
    _, s2 = _run(A, D, kh, kw, stride, pad, c, dev, want_g=False)
    assert np.array_equal(s2, s)
    with pytest.raises(vgc.VgcError):
        _run(A, D, kh, kw, stride, pad, c, dev, use_workspace=False)


def test_zz_report_observed_errors():
    """Not a check: prints the largest relative error of s each case showed (run with -s to see it)."""
    for tag, worst in sorted(OBSERVED.items()):
        print(f"observed max rel err of s: {tag}: {worst:.3e}")


def test_conv2d_rejects_what_it_cannot_do(dev):
    import torch
    from paper_1802_06058_amd import vgc
    lib = vgc.load()
    a = torch.zeros(2, 8, 8, 8, dtype=torch.bfloat16, device=dev)
    d = torch.zeros(2, 8, 8, 8, dtype=torch.bfloat16, device=dev)
    s = torch.zeros(72, 8, device=dev)
    args = lambda dtype, Cin, C, kh, ph: (dtype, a.data_ptr(), d.data_ptr(), 2, 8, 8, Cin, C, kh, 3, 1, 1, ph, 1, 1.0, None,
                                          s.data_ptr(), None, 0, None)
    assert lib.vgc_sqgrad_conv2d(*args(7, 8, 8, 3, 1)) == -4                # unknown dtype
    assert lib.vgc_sqgrad_conv2d(*args(vgc.BF16, 4, 8, 3, 1)) == -2         # Cin not a multiple of 8 bfloat16: needs the workspace
    assert lib.vgc_sqgrad_conv2d(*args(vgc.F32, 6, 8, 3, 1)) == -2          # Cin not a multiple of 4 floats: the same
    assert lib.vgc_sqgrad_conv2d(*args(vgc.BF16, 8, 8, 3, 3)) == -2         # padding as large as the kernel
    assert lib.vgc_sqgrad_conv2d(*args(vgc.BF16, 8, 8, 0, 0)) == -2         # empty kernel
    assert float(s.abs().sum()) == 0.0
