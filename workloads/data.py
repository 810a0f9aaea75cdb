"""Seeded synthetic datasets with the shapes and value distributions of the
benchmark configurations.  They stand in for the paper's workloads (generic
convex f_i for the linear models, a small dense network for the perceptron);
none of the paper's datasets is used.
"""
from __future__ import annotations

import numpy as np


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even conversion of fp32 to bf16 bit patterns (uint16).
    Storage format of the perceptron's input features."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    return ((u + 0x7FFF + lsb) >> 16).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << 16).view(np.float32)


def lsq_data(n, rows, d, seed=0, noise=0.1, feature_var=1.0, shared=False):
    """Least squares: per worker A_i (rows x d) ~ N(0, feature_var), one shared
    x* ~ N(0,1), b_i = A_i x* + noise * N(0,1).  ``shared`` gives every worker the
    same (A, b) (all f_i equal)."""
    rng = np.random.default_rng([seed, 11])
    xstar = rng.standard_normal(d).astype(np.float32)
    feats, targs = [], []
    for i in range(n):
        if shared and i > 0:
            feats.append(feats[0])
            targs.append(targs[0])
            continue
        A = rng.standard_normal((rows, d), dtype=np.float32)
        if feature_var != 1.0:
            A *= np.float32(np.sqrt(feature_var))
        b = (A.astype(np.float64) @ xstar.astype(np.float64)
             + noise * rng.standard_normal(rows)).astype(np.float32)
        feats.append(A)
        targs.append(b)
    return feats, targs, xstar


def logreg_data(n, rows, d, seed=0, noise=0.1):
    """Logistic regression: dense features a ~ N(0, 1/d), labels
    y = sign(a.x* + noise * N(0,1)) in {-1,+1} with sign(0) = +1."""
    rng = np.random.default_rng([seed, 12])
    xstar = rng.standard_normal(d).astype(np.float32)
    feats, targs = [], []
    scale = np.float32(1.0 / np.sqrt(d))
    for _ in range(n):
        A = rng.standard_normal((rows, d), dtype=np.float32) * scale
        z = A.astype(np.float64) @ xstar.astype(np.float64) + noise * rng.standard_normal(rows)
        feats.append(A)
        targs.append(np.where(z >= 0.0, 1.0, -1.0).astype(np.float32))
    return feats, targs, xstar


def mixture_data(n, rows, din=784, classes=10, seed=0):
    """Gaussian mixture: class means ~ N(0, I), sample = mean + N(0, I), classes
    uniform, the same mixture on every worker.  Features stored as bf16 bit
    patterns (uint16), labels int32."""
    rng = np.random.default_rng([seed, 13])
    means = rng.standard_normal((classes, din)).astype(np.float32)
    feats, targs = [], []
    for _ in range(n):
        lab = rng.integers(0, classes, size=rows).astype(np.int32)
        x = means[lab] + rng.standard_normal((rows, din), dtype=np.float32)
        feats.append(f32_to_bf16_bits(x))
        targs.append(lab)
    return feats, targs, means


def mlp_init(din=784, hid=1024, out=10, seed=0):
    """One initial parameter vector for every worker (Algorithm 1 requires equal
    initial models): W1 ~ N(0, 1/din), W2 ~ N(0, 1/hid), biases 0; flattened as
    [W1 (din x hid), b1, W2 (hid x out), b2]."""
    rng = np.random.default_rng([seed, 14])
    w1 = rng.standard_normal((din, hid)).astype(np.float32) / np.float32(np.sqrt(din))
    w2 = rng.standard_normal((hid, out)).astype(np.float32) / np.float32(np.sqrt(hid))
    return np.concatenate([w1.ravel(), np.zeros(hid, np.float32), w2.ravel(),
                           np.zeros(out, np.float32)]).astype(np.float32)


def linear_data_on_device(model, n, rows, d, seed=0, noise=0.1, feature_var=None, device="cuda:0"):
    """Large linear-model datasets generated directly in GPU memory (PyTorch's seeded device
    generator), for the full-size configurations whose data (tens of GB) would take minutes to draw
    on the host.  Same recipe as lsq_data / logreg_data: features ~ N(0, feature_var) (default 1/d),
    one x* ~ N(0,1), targets A x* + noise N(0,1) (least squares) or their sign (logistic).
    Returns per-worker lists of device tensors (features rows x d fp32, targets rows fp32)."""
    import torch
    gen = torch.Generator(device=device)
    gen.manual_seed(1000003 * seed + 17)
    var = (1.0 / d) if feature_var is None else feature_var
    xstar = torch.randn(d, device=device, generator=gen)
    feats, targs = [], []
    for _ in range(n):
        A = torch.randn((rows, d), device=device, generator=gen)
        if var != 1.0:
            A *= var ** 0.5
        z = A @ xstar + noise * torch.randn(rows, device=device, generator=gen)
        feats.append(A)
        targs.append(z if model == "lsq" else torch.where(z >= 0, 1.0, -1.0).to(torch.float32))
    return feats, targs


def mixture_data_on_device(n, rows, din=784, classes=10, seed=0, device="cuda:0"):
    """Gaussian-mixture inputs of the perceptron workload generated in GPU memory (same recipe as
    mixture_data): per worker bf16 features (rows x din, leading dimension padded to 8) and int32 labels."""
    import torch
    gen = torch.Generator(device=device)
    gen.manual_seed(1000003 * seed + 19)
    means = torch.randn((classes, din), device=device, generator=gen)
    ld = (din + 7) // 8 * 8
    feats, targs = [], []
    for _ in range(n):
        lab = torch.randint(0, classes, (rows,), device=device, generator=gen, dtype=torch.int32)
        x = torch.zeros((rows, ld), dtype=torch.bfloat16, device=device)
        x[:, :din] = (means[lab.long()] + torch.randn((rows, din), device=device, generator=gen)).to(torch.bfloat16)
        feats.append(x)
        targs.append(lab)
    return feats, targs
