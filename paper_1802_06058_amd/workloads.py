"""Seeded synthetic inputs with the shapes of the benchmark configurations.

This module serves both the HIP path's tests / benchmark and the CPU oracle's tests.
It holds input synthesis only: shapes, distributions, seeds and raw draws.  None of the
method's arithmetic (the sums over the mini-batch, test, quantiser, packing, decode) lives here.

Every stream is `numpy.random.default_rng` on a `SeedSequence(seed, spawn_key=path)`,
so the tensor for (config, iteration, layer, role) is the same bytes wherever it is
drawn.  bf16 tensors are carried as uint16 bit patterns (numpy has no bf16).
"""
from __future__ import annotations

import math

import numpy as np

# ---------------------------------------------------------------------------------------
# random streams and dtype helpers
# ---------------------------------------------------------------------------------------


def stream(seed: int, *path: int) -> np.random.Generator:
    """Independent generator for one tensor: child `path` of the root seed."""
    return np.random.default_rng(np.random.SeedSequence(entropy=seed, spawn_key=tuple(int(p) for p in path)))


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns uint16 bit patterns."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return rounded.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns to float32 exactly."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def groups_from_sizes(sizes):
    """[(offset, size)] tiling [0, sum(sizes)) in order."""
    out, off = [], 0
    for s in sizes:
        out.append((off, int(s)))
        off += int(s)
    return out


# ---------------------------------------------------------------------------------------
# layer tables
# ---------------------------------------------------------------------------------------


def _conv(name, cin, k, cout, spatial):
    return dict(name=name, kind="conv", J=cin * k * k, C=cout, P=spatial * spatial, size=cin * k * k * cout)


def _fc(name, fin, fout):
    return dict(name=name, kind="fc", J=fin, C=fout, P=1, size=fin * fout)


def _vec(name, n):
    return dict(name=name, kind="vector", J=n, C=1, P=1, size=n)


def resnet50_layers():
    """Weight tensors of a ResNet-50 (bottleneck stages 3/4/6/3, widths 64..512, x4
    expansion, output spatial 56/28/14/7, stride carried by the 3x3 convolution), each
    convolution followed by a norm layer's scale and shift vectors; 25 557 032 parameters.
    P is the number of output positions of the convolution (the K of its per-sample GEMM)."""
    L = [_conv("stem.conv", 3, 7, 64, 112), _vec("stem.norm.scale", 64), _vec("stem.norm.shift", 64)]
    cin, prev_sp = 64, 56
    for stage, (width, blocks, sp) in enumerate([(64, 3, 56), (128, 4, 28), (256, 6, 14), (512, 3, 7)]):
        for b in range(blocks):
            p = f"s{stage + 1}.b{b}"
            in_sp = prev_sp if b == 0 else sp
            convs = [
                _conv(p + ".conv1", cin, 1, width, in_sp),
                _conv(p + ".conv2", width, 3, width, sp),
                _conv(p + ".conv3", width, 1, 4 * width, sp),
            ]
            if b == 0:
                convs.append(_conv(p + ".down", cin, 1, 4 * width, sp))
            for c in convs:
                L += [c, _vec(c["name"] + ".norm.scale", c["C"]), _vec(c["name"] + ".norm.shift", c["C"])]
            cin = 4 * width
        prev_sp = sp
    L += [_fc("fc", 2048, 1000), _vec("fc.bias", 1000)]
    return L


def vgg16_layers():
    """Weight tensors of VGG-16 (13 3x3 convolutions at 224..14 spatial, then
    25088x4096, 4096x4096, 4096x1000), each with a bias; 138 357 544 parameters."""
    cfg = [(3, 64, 224), (64, 64, 224), (64, 128, 112), (128, 128, 112),
           (128, 256, 56), (256, 256, 56), (256, 256, 56),
           (256, 512, 28), (512, 512, 28), (512, 512, 28),
           (512, 512, 14), (512, 512, 14), (512, 512, 14)]
    L = []
    for i, (cin, cout, sp) in enumerate(cfg):
        L += [_conv(f"conv{i + 1}", cin, 3, cout, sp), _vec(f"conv{i + 1}.bias", cout)]
    for i, (fin, fout) in enumerate([(25088, 4096), (4096, 4096), (4096, 1000)]):
        L += [_fc(f"fc{i + 6}", fin, fout), _vec(f"fc{i + 6}.bias", fout)]
    return L


def mlp_layers():
    """784-1000-1000-10 perceptron, weights only (three groups)."""
    return [_fc("fc1", 784, 1000), _fc("fc2", 1000, 1000), _fc("fc3", 1000, 10)]


# ---------------------------------------------------------------------------------------
# per-layer activations / output-gradients (inputs of the squared-gradient statistic)
# ---------------------------------------------------------------------------------------


def fc_inputs(seed, path, B, J, C, x_dist="normal", relu_sparse=False, d_sigma=1.0, bf16=False):
    """X [B, J] and Delta [B, C] for one fully-connected layer."""
    rx, rm, rd = stream(seed, *path, 0), stream(seed, *path, 1), stream(seed, *path, 2)
    if x_dist == "normal":
        X = rx.standard_normal((B, J), dtype=np.float32)
    elif x_dist == "uniform":
        X = rx.random((B, J), dtype=np.float32)
    else:
        raise ValueError(x_dist)
    if relu_sparse:
        X = X * (rm.random((B, J), dtype=np.float32) < 0.5)
    D = rd.standard_normal((B, C), dtype=np.float32) * np.float32(d_sigma)
    if bf16:
        return f32_to_bf16_bits(X), f32_to_bf16_bits(D)
    return np.ascontiguousarray(X, np.float32), np.ascontiguousarray(D, np.float32)


def conv_inputs(seed, path, B, P, J, C, d_sigma=1.0, bf16=False):
    """im2col patches U [B, P, J] ~ N(0,1) and Delta [B, P, C] ~ N(0, d_sigma^2)."""
    ru, rd = stream(seed, *path, 0), stream(seed, *path, 2)
    U = ru.standard_normal((B, P, J), dtype=np.float32)
    D = rd.standard_normal((B, P, C), dtype=np.float32) * np.float32(d_sigma)
    if bf16:
        return f32_to_bf16_bits(U), f32_to_bf16_bits(D)
    return U, D


def conv2d_inputs(seed, path, B, H, W, Cin, Ho, Wo, C, d_sigma=1.0, bf16=False):
    """Layer input [B, H, W, Cin] ~ N(0,1) and output gradient [B, Ho, Wo, C] ~ N(0, d_sigma^2), NHWC."""
    ra, rd = stream(seed, *path, 0), stream(seed, *path, 2)
    A = ra.standard_normal((B, H, W, Cin), dtype=np.float32)
    D = rd.standard_normal((B, Ho, Wo, C), dtype=np.float32) * np.float32(d_sigma)
    if bf16:
        return f32_to_bf16_bits(A), f32_to_bf16_bits(D)
    return A, D


def layer_sigmas(seed, n_layers, lo=1e-5, hi=1e-2):
    """Per-layer gradient scale, log-uniform in [lo, hi], drawn once per layer."""
    u = stream(seed, 9001).random(n_layers)
    return np.exp(math.log(lo) + u * (math.log(hi) - math.log(lo)))


# ---------------------------------------------------------------------------------------
# per-sample gradient draws for the elementwise stages
# ---------------------------------------------------------------------------------------


def sample_draws(seed, path, n, batch, dist="normal", sigma=1.0, nu=3.0, chunk=1 << 20):
    """`batch` i.i.d. per-sample gradients for each of n parameters, chunk by chunk so that no
    [batch, n] array is ever held: yields (lo, y) with y [batch, m] float64 the draws of parameters
    lo .. lo + m - 1.  dist: "normal" N(0, sigma^2) or "student" sigma * t(nu).  What a step's two
    inputs are made of is the caller's business (tests and the benchmark reduce the draws)."""
    rng = stream(seed, *path)
    for lo in range(0, n, chunk):
        m = min(chunk, n - lo)
        if dist == "normal":
            y = rng.standard_normal((batch, m))
        elif dist == "student":
            y = rng.standard_t(nu, (batch, m))
        else:
            raise ValueError(dist)
        y *= sigma
        yield lo, y


def flat_groups(n, group=1 << 24):
    """Split a flat stream of n parameters into groups of `group` (last one partial)."""
    return groups_from_sizes([min(group, n - lo) for lo in range(0, n, group)])


def device_student_draw(m, nu, gen, device):
    """One per-sample gradient for each of m parameters, Student-t(nu) with integer nu, drawn on `device` from the
    seeded torch generator `gen` as z / sqrt(chi2_nu / nu) (float32).  The flat-stream configuration draws
    `batch` of these per parameter and step."""
    import torch

    k = int(nu)
    assert k == nu, "integer degrees of freedom only"
    z = torch.randn(m, generator=gen, device=device, dtype=torch.float32)
    chi = torch.zeros(m, dtype=torch.float32, device=device)
    for _ in range(k):
        w = torch.randn(m, generator=gen, device=device, dtype=torch.float32)
        chi += w * w
    return z / torch.sqrt(chi / k)


# ---------------------------------------------------------------------------------------
# the five configurations
# ---------------------------------------------------------------------------------------

CONFIGS = {
    "C1": dict(desc="single FC layer 1024x1024 fp32, batch 32", layers=[_fc("fc", 1024, 1024)],
               batch=32, iterations=10, alpha=1.0, zeta=0.999, seed=0),
    "C2": dict(desc="MLP 784-1000-1000-10 fp32, batch 128, ReLU-sparse inputs", layers=mlp_layers(),
               batch=128, iterations=50, alpha=2.0, zeta=0.999, seed=0),
    "C3": dict(desc="ResNet-50-shaped parameter set fp32, batch 32", layers=resnet50_layers(),
               batch=32, iterations=20, alpha=1.0, zeta=0.999, seed=0),
    "C4": dict(desc="VGG-16-shaped parameter set, bf16 activations/deltas, batch 64", layers=vgg16_layers(),
               batch=64, iterations=10, alpha=(0.5, 1.0, 2.0, 4.0), zeta=0.999, seed=0),
    "C5": dict(desc="flat 1e9-parameter fp32 stream, Student-t(3) per-sample gradients, batch 16, 8 workers",
               n=1_000_000_000, group=1 << 24, batch=16, nu=3.0, workers=8, iterations=5,
               alpha=1.0, zeta=0.999, seed=0),
}


def c1_inputs(iteration):
    """Config 1: X ~ N(0,1), Delta ~ N(0, 0.01^2), fresh every iteration."""
    c = CONFIGS["C1"]
    return fc_inputs(c["seed"], (1, iteration, 0), c["batch"], 1024, 1024, "normal", False, 0.01)


def c2_inputs(iteration, layer):
    """Config 2: layer 0 sees U(0,1) inputs, the hidden layers U(0,1) with half the
    entries zeroed (post-ReLU sparsity); Delta ~ N(0, 1e-3^2)."""
    c = CONFIGS["C2"]
    L = c["layers"][layer]
    return fc_inputs(c["seed"], (2, iteration, layer), c["batch"], L["J"], L["C"], "uniform", layer > 0, 1e-3)
