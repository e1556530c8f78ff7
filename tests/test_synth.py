"""The synthetic input generators produce the shapes and sparsity structure the
workload recipes state (CPU only, small sizes)."""
import numpy as np
import torch

import synth


def test_mlp_layout_and_dead_neuron_runs():
    assert synth.mlp_num_params() == 1863690
    sizes = (6, 5, 4, 3)
    p = synth.mlp_num_params(sizes)
    assert p == 5 * 6 + 5 + 4 * 5 + 4 + 3 * 4 + 3
    g = synth.mlp_relu_gradients(64, seed=1, device="cpu", sizes=sizes).numpy()
    assert g.shape == (64, p)
    w1 = g[:, :30].reshape(64, 5, 6)
    b1 = g[:, 30:35]
    dead = (b1 == 0)
    assert 0.3 < dead.mean() < 0.7
    assert np.all((w1 == 0).all(axis=2) == dead)            # a dead neuron zeroes its whole fan-in run and its bias
    last = g[:, p - 15:]
    assert not (last == 0).any()                             # last layer is dense
    again = synth.mlp_relu_gradients(64, seed=1, device="cpu", sizes=sizes).numpy()
    assert np.array_equal(g, again)                          # seeded


def test_bernoulli_and_laplace_sparsity():
    g = synth.bernoulli_sparse_normal(50, 4000, 0.8, 1.0, seed=2).numpy()
    assert abs((g == 0).mean() - 0.8) < 0.01
    assert abs(g[g != 0].std() - 1.0) < 0.02
    h = synth.laplace_sparse(50, 4000, 0.3, 1e-3, seed=3).numpy()
    assert abs((h == 0).mean() - 0.3) < 0.01
    nz = h[h != 0]
    assert abs(np.abs(nz).mean() - 1e-3) < 3e-5             # E|X| = scale for Laplace(0, scale)
    assert abs((nz > 0).mean() - 0.5) < 0.01


def test_linear_layer_factors_are_bf16_with_stated_scales():
    x, g = synth.linear_layer_factors(4, 16, 256, 128, seed=4)
    assert x.dtype == torch.bfloat16 and g.dtype == torch.bfloat16
    assert x.shape == (4, 16, 256) and g.shape == (4, 16, 128)
    assert abs(x.float().std().item() - 1.0) < 0.05
    assert abs(g.float().var().item() - 1e-3) < 1e-4          # N(0, 1e-3): the second argument is a variance


def test_llama_block_shapes():
    shapes = [(d_in, d_out) for _, d_in, d_out in synth.LLAMA_BLOCK_LINEARS]
    assert len(shapes) == 7
    assert shapes.count((2048, 2048)) == 4 and shapes.count((2048, 8192)) == 2 and shapes.count((8192, 2048)) == 1


def test_planted_gradients_shapes_and_structure():
    G, Gt, planted = synth.planted_gradients(200, 16, 1000, 50, seed=3)
    assert G.shape == (200, 1000) and Gt.shape == (16, 1000) and planted.numel() == 50
    assert planted[0] == 0 and torch.all(planted[1:] > planted[:-1]) and planted[-1] < 1000
    rest = torch.ones(1000, dtype=torch.bool)
    rest[planted] = False
    assert G[:, planted].std() > 5 * G[:, rest].std()
    G2, _, _ = synth.planted_gradients(200, 16, 1000, 50, seed=3)
    assert torch.equal(G, G2)
