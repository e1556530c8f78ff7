"""Bit-reproducibility of the paths whose reductions have a fixed order (matrix-core products with fixed K ranges and
fixed-order partial sums, the fp64 factorisation, integer index work): the same call on the same inputs twice gives the
same bits.  (The sparse projection accumulates with LDS atomics in fp64, whose order may vary; it is held to its
tolerance against the oracle instead.)"""
import pytest
import torch

import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def grass():
    import paper_2505_18976_amd as g
    g.load_library()
    return g


def _dev():
    return torch.device("cuda:0")


def _twice(fn):
    a = fn()
    torch.cuda.synchronize()
    b = fn()
    torch.cuda.synchronize()
    a = a if isinstance(a, (tuple, list)) else (a,)
    b = b if isinstance(b, (tuple, list)) else (b,)
    for x, y in zip(a, b):
        assert torch.equal(x, y)


def test_score_products_are_bit_reproducible(grass):
    train = synth.dense_normal(700, 2048, seed=5000, device=_dev())
    test = synth.dense_normal(130, 2048, seed=5001, device=_dev())
    for mode in (0, 1):
        _twice(lambda: grass.grass_score(train, test, compute_mode=mode, ws=True))
    _twice(lambda: grass.grass_score_bf16(grass.grass_to_bf16(train), grass.grass_to_bf16(test)))
    long_k = synth.dense_normal(130, 40000, seed=5002, device=_dev())            # few tiles, long K: split over K ranges
    _twice(lambda: grass.grass_score(long_k, long_k[:64].contiguous(), compute_mode=0, ws=True))


def test_cache_stage_is_bit_reproducible(grass):
    G = synth.dense_normal(3000, 576, seed=5003, device=_dev())
    _twice(lambda: grass.grass_fim(G))
    F = grass.grass_fim(G)
    _twice(lambda: grass.grass_fim_inverse(F, 1e-3))
    W = grass.grass_fim_inverse(F, 1e-3)
    _twice(lambda: grass.grass_ifvp(G, W))


def test_logra_and_factorised_mask_are_bit_reproducible(grass):
    n, T, d = 8, 300, 1024
    x, g = synth.linear_layer_factors(n, T, d, d, seed=5004, device=_dev())
    Pi = grass.grass_to_bf16(grass.grass_gauss_matrix(0, 40, d, 64, 0, d, device=_dev()))
    Po = grass.grass_to_bf16(grass.grass_gauss_matrix(0, 41, d, 64, 0, d, device=_dev()))
    _twice(lambda: grass.logra_linear(x, g, Pi, Po))
    ii = grass.grass_mask_indices(0, 16, d, 64, device=_dev())
    io = grass.grass_mask_indices(0, 17, d, 64, device=_dev())
    _twice(lambda: grass.factmask_linear(x, g, ii, io))


def test_selective_mask_step_and_extraction_are_bit_reproducible(grass):
    n, m, p = 300, 130, 4100
    G = synth.dense_normal(n, p, seed=5005, device=_dev())
    Gt = synth.dense_normal(m, p, seed=5006, device=_dev())
    S = synth.dense_normal(1, p, seed=5007, device=_dev()).reshape(-1).contiguous()
    A = grass.grass_score(G, Gt, compute_mode=0)
    _twice(lambda: grass.grass_selective_mask_grad(G, Gt, A, S, 1e-3, 0.8))
    _twice(lambda: grass.grass_selective_mask_indices(S, 512))
    _twice(lambda: grass.grass_mask_indices(3, 5, 1 << 20, 4096, device=_dev()))
