"""Pins of the oracle's convolution form that takes the layer's input and output gradient as stored
(NHWC), without an im2col matrix: brute force, a hand-computed case, torch's own convolution
weight gradient per sample, and the already-pinned im2col form fed with an independently written
im2col."""
import numpy as np
import pytest

from oracle import vgc_oracle as O


def _im2col(act, kh, kw, stride, pad):
    """Patch matrix written with explicit index arithmetic (not the oracle's slicing)."""
    B, H, W, Cin = act.shape
    sh, sw = stride
    ph, pw = pad
    Ho, Wo = (H + 2 * ph - kh) // sh + 1, (W + 2 * pw - kw) // sw + 1
    U = np.zeros((B, Ho * Wo, kh * kw * Cin))
    for y in range(Ho):
        for x in range(Wo):
            for ky in range(kh):
                for kx in range(kw):
                    iy, ix = y * sh + ky - ph, x * sw + kx - pw
                    if 0 <= iy < H and 0 <= ix < W:
                        U[:, y * Wo + x, (ky * kw + kx) * Cin:(ky * kw + kx + 1) * Cin] = act[:, iy, ix, :]
    return U, Ho, Wo


GEOMS = [  # H, W, Cin, Cout, kh, kw, stride, pad
    (6, 5, 3, 4, 3, 3, (1, 1), (1, 1)),
    (7, 8, 2, 3, 3, 3, (2, 2), (1, 1)),
    (5, 5, 4, 2, 1, 1, (1, 1), (0, 0)),
    (9, 7, 2, 2, 5, 3, (2, 1), (2, 0)),
    (4, 4, 1, 1, 2, 2, (2, 2), (0, 0)),
]


def test_hand_computed_single_tap():
    # one sample, 1x1 input channel, 2x2 input, 2x2 kernel, no padding: a single output position, so the
    # weight gradient is the input itself times the output gradient
    act = np.array([[[[1.0], [2.0]], [[3.0], [-4.0]]]])          # [1, 2, 2, 1]
    D = np.array([[[[0.5]]]])                                      # [1, 1, 1, 1]
    g, s = O.sqgrad_conv_nhwc(act, D, 2, 2, (1, 1), (0, 0), 1.0)
    assert np.array_equal(g[:, 0], [0.5, 1.0, 1.5, -2.0])          # rows (ky, kx) = (0,0), (0,1), (1,0), (1,1)
    assert np.array_equal(s[:, 0], [0.25, 1.0, 2.25, 4.0])
    # padding 1, 3x3 kernel on the same input: output 2x2; with D one-hot at output (0, 0) tap (ky, kx) sees
    # input (ky - 1, kx - 1): only taps with ky, kx in {1, 2} are inside
    D = np.zeros((1, 2, 2, 1)); D[0, 0, 0, 0] = 1.0
    g, _ = O.sqgrad_conv_nhwc(act, D, 3, 3, (1, 1), (1, 1), 1.0)
    assert np.array_equal(g[:, 0].reshape(3, 3), [[0, 0, 0], [0, 1, 2], [0, 3, -4]])


@pytest.mark.parametrize("geom", GEOMS)
def test_bruteforce_and_im2col(geom):
    H, W, Cin, Cout, kh, kw, stride, pad = geom
    rng = np.random.default_rng(hash(geom) % 1000)
    B = 3
    act = rng.standard_normal((B, H, W, Cin))
    Ho, Wo = O.conv_out_size(H, kh, stride[0], pad[0]), O.conv_out_size(W, kw, stride[1], pad[1])
    D = rng.standard_normal((B, Ho, Wo, Cout))
    g, s = O.sqgrad_conv_nhwc(act, D, kh, kw, stride, pad, 1.0 / B)
    gb, sb = O.sqgrad_conv_nhwc_bruteforce(act, D, kh, kw, stride, pad, 1.0 / B)
    assert np.allclose(g, gb, rtol=1e-12, atol=1e-14) and np.allclose(s, sb, rtol=1e-12, atol=1e-14)
    U, Ho2, Wo2 = _im2col(act, kh, kw, stride, pad)
    assert (Ho2, Wo2) == (Ho, Wo)
    gi, si = O.sqgrad_conv(U, D.reshape(B, Ho * Wo, Cout), 1.0 / B)
    assert np.allclose(g, gi, rtol=1e-12, atol=1e-14) and np.allclose(s, si, rtol=1e-12, atol=1e-14)


@pytest.mark.parametrize("geom", GEOMS[:4])
def test_against_torch_conv2d_weight_gradient(geom):
    """Per-sample weight gradient of torch's conv2d (autograd), summed and square-summed."""
    import torch
    H, W, Cin, Cout, kh, kw, stride, pad = geom
    rng = np.random.default_rng(11)
    B = 4
    act = rng.standard_normal((B, H, W, Cin))
    Ho, Wo = O.conv_out_size(H, kh, stride[0], pad[0]), O.conv_out_size(W, kw, stride[1], pad[1])
    D = rng.standard_normal((B, Ho, Wo, Cout))
    wt = torch.zeros(Cout, Cin, kh, kw, dtype=torch.float64, requires_grad=True)
    g_ref = np.zeros((kh * kw * Cin, Cout)); s_ref = np.zeros_like(g_ref)
    c = 1.0 / B
    for z in range(B):
        x = torch.from_numpy(act[z].transpose(2, 0, 1)[None])                     # NCHW
        out = torch.nn.functional.conv2d(x, wt, stride=stride, padding=pad)
        assert out.shape == (1, Cout, Ho, Wo)
        (gw,) = torch.autograd.grad(out, wt, torch.from_numpy(D[z].transpose(2, 0, 1)[None]))
        G = gw.numpy().transpose(2, 3, 1, 0).reshape(kh * kw * Cin, Cout) * c     # [Cout,Cin,kh,kw] -> [(ky,kx,i), o]
        g_ref += G; s_ref += G * G
    g, s = O.sqgrad_conv_nhwc(act, D, kh, kw, stride, pad, c)
    assert np.allclose(g, g_ref, rtol=1e-10, atol=1e-12) and np.allclose(s, s_ref, rtol=1e-10, atol=1e-12)


def test_one_by_one_convolution_is_the_shared_weight_form():
    rng = np.random.default_rng(3)
    act = rng.standard_normal((2, 3, 4, 5)); D = rng.standard_normal((2, 3, 4, 6))
    g, s = O.sqgrad_conv_nhwc(act, D, 1, 1, (1, 1), (0, 0), 0.5)
    g2, s2 = O.sqgrad_conv(act.reshape(2, 12, 5), D.reshape(2, 12, 6), 0.5)
    assert np.allclose(g, g2, rtol=1e-13) and np.allclose(s, s2, rtol=1e-13)
