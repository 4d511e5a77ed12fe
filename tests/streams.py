"""Test-side preparation of the inputs of the elementwise stages: the raw per-sample draws of
`workloads` reduced to the two per-parameter inputs of a step,
    g = sum_z y_z / B,   s = sum_z (y_z / B)^2        (first two lines of Alg. 1's loop body).
Both the GPU path and the oracle read the arrays these helpers return; neither computes them."""
import numpy as np

from paper_1802_06058_amd import workloads as W


def sample_stream(seed, path, n, batch, dist="normal", sigma=1.0, nu=3.0):
    """(g, s) float32 for n parameters from `batch` i.i.d. draws each (float64 reduction, rounded once)."""
    g = np.empty(n, np.float32)
    s = np.empty(n, np.float32)
    for lo, y in W.sample_draws(seed, path, n, batch, dist=dist, sigma=sigma, nu=nu):
        y /= batch
        g[lo:lo + y.shape[1]] = y.sum(axis=0)
        s[lo:lo + y.shape[1]] = (y * y).sum(axis=0)
    return g, s


def device_student_stream(n, batch, nu, seed, device, chunk=1 << 24):
    """The flat-stream configuration on the GPU: (g, s) float32 device tensors from `batch` Student-t(nu)
    draws per parameter out of a seeded torch generator (float32 reduction in draw order)."""
    import torch
    gen = torch.Generator(device=device)
    gen.manual_seed(int(seed))
    g = torch.empty(n, dtype=torch.float32, device=device)
    s = torch.empty(n, dtype=torch.float32, device=device)
    for lo in range(0, n, chunk):
        m = min(chunk, n - lo)
        gacc = torch.zeros(m, dtype=torch.float32, device=device)
        sacc = torch.zeros(m, dtype=torch.float32, device=device)
        for _ in range(batch):
            y = W.device_student_draw(m, nu, gen, device) / batch
            gacc += y
            sacc += y * y
        g[lo:lo + m] = gacc
        s[lo:lo + m] = sacc
    return g, s
