"""Seeded synthetic inputs shared by the tests, the benchmark and the oracle checks.

This module holds none of the method's arithmetic: it only draws the tensors
that stand in for real per-sample gradients (MNIST-MLP, ResNet-18-sized,
Llama-style linear-layer factors), with the shapes and sparsity structure the
paper motivates in Sec. 3.1 (ReLU zeros in per-sample gradients).  Everything
is drawn with torch on the requested device from an explicit seed; the oracle
is always fed a host copy of the very tensor the GPU consumed.
"""
from __future__ import annotations

import torch

# MLP 784-1024-1024-10, per-layer blocks concatenated: [W1 | b1 | W2 | b2 | W3 | b3]
MLP_SIZES = (784, 1024, 1024, 10)


def mlp_num_params(sizes=MLP_SIZES) -> int:
    return sum(sizes[i + 1] * sizes[i] + sizes[i + 1] for i in range(len(sizes) - 1))


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def bernoulli_sparse_normal(n: int, p: int, zero_frac: float, std: float, seed: int,
                            device="cpu") -> torch.Tensor:
    """n x p fp32; each entry is exactly 0 with probability zero_frac, else N(0, std^2)."""
    gen = _gen(seed, device)
    out = torch.empty((n, p), dtype=torch.float32, device=device)
    rows = max(1, min(n, (1 << 28) // max(p, 1)))
    for a in range(0, n, rows):
        blk = out[a:a + rows]
        blk.normal_(0.0, std, generator=gen)
        keep = torch.rand(blk.shape, device=device, generator=gen) >= zero_frac
        blk.mul_(keep)
    return out


def laplace_sparse(n: int, p: int, zero_frac: float, scale: float, seed: int,
                   device="cpu") -> torch.Tensor:
    """n x p fp32; exact zeros with probability zero_frac, else Laplace(0, scale)."""
    gen = _gen(seed, device)
    out = torch.empty((n, p), dtype=torch.float32, device=device)
    rows = max(1, min(n, (1 << 28) // max(p, 1)))
    for a in range(0, n, rows):
        blk = out[a:a + rows]
        blk.exponential_(1.0 / scale, generator=gen)          # |value| ~ Exp(mean = scale)
        u = torch.rand(blk.shape, device=device, generator=gen)
        # u < zero_frac -> 0 ; remaining mass split evenly between the two signs
        half = zero_frac + (1.0 - zero_frac) * 0.5
        sign = (u >= zero_frac).to(torch.float32) - 2.0 * (u >= half).to(torch.float32)
        blk.mul_(sign)
        del u, sign
    return out


def mlp_relu_gradients(n: int, seed: int, device="cpu", std: float = 0.1,
                       dead_frac: float = 0.5, sizes=MLP_SIZES) -> torch.Tensor:
    """Per-sample gradients of a ReLU MLP, flattened layer by layer.

    For every sample each hidden neuron is dead with probability dead_frac;
    a dead neuron's whole fan-in run of weights (contiguous) and its bias entry
    are exactly zero.  The last layer is dense.  Non-zeros are N(0, std^2).
    """
    gen = _gen(seed, device)
    p = mlp_num_params(sizes)
    out = torch.empty((n, p), dtype=torch.float32, device=device)
    rows = max(1, min(n, (1 << 28) // p))
    n_layers = len(sizes) - 1
    for a in range(0, n, rows):
        blk = out[a:a + rows]
        blk.normal_(0.0, std, generator=gen)
        off = 0
        for l in range(n_layers):
            fan_in, fan_out = sizes[l], sizes[l + 1]
            w = blk[:, off:off + fan_out * fan_in].unflatten(1, (fan_out, fan_in))
            b = blk[:, off + fan_out * fan_in: off + fan_out * fan_in + fan_out]
            if l < n_layers - 1:
                alive = (torch.rand((blk.shape[0], fan_out), device=device, generator=gen)
                         >= dead_frac).to(torch.float32)
                w.mul_(alive[:, :, None])
                b.mul_(alive)
            off += fan_out * fan_in + fan_out
    return out


def linear_layer_factors(n: int, T: int, d_in: int, d_out: int, seed: int, device="cpu",
                         x_std: float = 1.0, g_std: float = 1e-3 ** 0.5):
    """Layer input x (n, T, d_in) ~ N(0, x_std^2) and pre-activation gradient
    g (n, T, d_out) ~ N(0, g_std^2), both rounded to bf16 (the paper's Eq. (2)
    factors z_in and D z_out with tokens along the middle axis)."""
    gen = _gen(seed, device)
    x = torch.empty((n, T, d_in), dtype=torch.float32, device=device).normal_(0.0, x_std, generator=gen)
    x = x.to(torch.bfloat16)
    g = torch.empty((n, T, d_out), dtype=torch.float32, device=device).normal_(0.0, g_std, generator=gen)
    g = g.to(torch.bfloat16)
    return x, g


def dense_normal(rows: int, cols: int, seed: int, device="cpu", std: float = 1.0) -> torch.Tensor:
    gen = _gen(seed, device)
    return torch.empty((rows, cols), dtype=torch.float32, device=device).normal_(0.0, std, generator=gen)


# Llama-style 1.2B block: hidden 2048, MLP 8192; (name, d_in, d_out) of its 7 linears.
LLAMA_BLOCK_LINEARS = (
    ("q", 2048, 2048), ("k", 2048, 2048), ("v", 2048, 2048), ("o", 2048, 2048),
    ("gate", 2048, 8192), ("up", 2048, 8192), ("down", 8192, 2048),
)


def compressed_gradients(rows: int, k: int, seed: int, device="cpu", decay: float = 0.5) -> torch.Tensor:
    """rows x k fp32 stand-in for compressed per-sample gradients with a decaying spectrum: column c is
    N(0, (1+c)^(-2*decay)), so the FIM has eigenvalues spread over k^(2*decay) instead of a flat identity."""
    gen = _gen(seed, device)
    out = torch.empty((rows, k), dtype=torch.float32, device=device).normal_(0.0, 1.0, generator=gen)
    scale = (1.0 + torch.arange(k, dtype=torch.float32, device=device)) ** (-decay)
    return out * scale[None, :]


def planted_gradients(n: int, m: int, p: int, informative: int, seed: int, device="cpu", strong: float = 3.0,
                      weak: float = 0.3):
    """Train (n x p) and test (m x p) fp32 gradients in which `informative` coordinates, spread evenly over [0, p),
    carry most of the variance (std `strong`) and the rest is weak noise (std `weak`): a stand-in for per-sample
    gradients whose attribution scores are dominated by a small set of parameters, the situation the Selective Mask is
    built for.  Returns (G, Gt, planted) with planted the ascending int64 indices of the informative coordinates."""
    gen = _gen(seed, device)
    planted = (torch.arange(informative, dtype=torch.float64) * (p / informative)).floor().to(torch.int64)
    std = torch.full((p,), weak, dtype=torch.float32, device=device)
    std[planted.to(device)] = strong
    G = torch.empty((n, p), dtype=torch.float32, device=device).normal_(0.0, 1.0, generator=gen) * std[None, :]
    Gt = torch.empty((m, p), dtype=torch.float32, device=device).normal_(0.0, 1.0, generator=gen) * std[None, :]
    return G, Gt, planted

