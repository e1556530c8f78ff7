"""GPU parity of the paths the benchmark times, at the sizes and in the launch configuration it times them.

* FactGraSS over all 112 Llama-style linear layers in ONE launch (Sec. 3.3.2; n = 8 sequences of 1,024 tokens, masks
  64/64, k_l = 4,096 per layer, every layer with its own tensors, masks and SJLT stream): the layer table travels in
  two packs of descriptors and each workgroup owns a whole sequence.  Layers from both packs are compared with the
  oracle, every layer block with the per-layer entry point.
* ResNet-scale SJLT (Sec. 3.1; n = 1,024, p = 11,173,962, k = 8,192): 64 evenly spaced rows against the oracle.
* Cache stage on one layer block (Sec. 2.1 steps 2 and 3): FIM of 65,536 x 4,096 compressed gradients, damped inverse
  at k = 4,096, iFVP of all 65,536 rows, on the inputs the benchmark uses.
"""
import numpy as np
import pytest
import torch

import synth
from oracle import grass_oracle as orc

pytestmark = pytest.mark.gpu

TOL_FACT = 2e-3          # FactGraSS bar (row-relative); exact bf16 products, fp32 accumulation
TOL_SJLT = 1e-5


@pytest.fixture(scope="module")
def grass():
    import paper_2505_18976_amd as g
    g.load_library()
    return g


def _dev():
    return torch.device("cuda:0")


def _sample_rows(n, count):
    return sorted(set(np.linspace(0, n - 1, count).round().astype(int).tolist()))


def test_factgrass_112_layers_in_one_launch(grass):
    n, T, kf, k_l, seed = 8, 1024, 64, 4096, 0
    n_layers = 16 * 7
    layers = []
    for layer in range(n_layers):
        _, d_in, d_out = synth.LLAMA_BLOCK_LINEARS[layer % 7]
        x, g = synth.linear_layer_factors(n, T, d_in, d_out, seed=2000 + layer, device=_dev())
        s_in, s_out, s_sjlt = orc.layer_streams(layer)
        ii = grass.grass_mask_indices(seed, s_in, d_in, kf, device=_dev())
        io = grass.grass_mask_indices(seed, s_out, d_out, kf, device=_dev())
        layers.append((x, g, ii, io, s_sjlt))
    cat = torch.full((n, k_l * n_layers + 5), -3.0, dtype=torch.float32, device=_dev())
    grass.factgrass_layers(layers, k_l, 1, seed, cat)
    torch.cuda.synchronize()
    got = cat.cpu().numpy()
    assert np.all(got[:, k_l * n_layers:] == -3.0)                  # nothing written past the last block

    # oracle on layers of both descriptor packs (0..63 and 64..111), all three shapes, pack boundaries included
    checked = [0, 1, 4, 6, 31, 62, 63, 64, 65, 69, 90, 104, 110, 111]
    for layer in checked:
        x, g, ii, io, s_sjlt = layers[layer]
        _, d_in, d_out = synth.LLAMA_BLOCK_LINEARS[layer % 7]
        ii_h, io_h = ii.cpu().numpy(), io.cpu().numpy()
        s_in, s_out, _ = orc.layer_streams(layer)
        assert np.array_equal(ii_h, orc.mask_indices(seed, s_in, d_in, kf))
        assert np.array_equal(io_h, orc.mask_indices(seed, s_out, d_out, kf))
        xs = x[:, :, ii.long()].float().cpu().numpy()              # the oracle only needs the kept columns
        gs = g[:, :, io.long()].float().cpu().numpy()
        ref = orc.factgrass_linear(xs, gs, np.arange(kf), np.arange(kf), k_l, 1, seed, s_sjlt)
        err = orc.max_rel_err(got[:, layer * k_l:(layer + 1) * k_l], ref)
        assert err <= TOL_FACT, (layer, err)

    # every block against the per-layer call (same arithmetic, other chunking of the tokens)
    single = torch.empty((n, k_l), dtype=torch.float32, device=_dev())
    for layer, (x, g, ii, io, s_sjlt) in enumerate(layers):
        grass.factgrass_linear(x, g, ii, io, k_l, 1, seed, s_sjlt, out=single)
        torch.cuda.synchronize()
        err = orc.max_rel_err(got[:, layer * k_l:(layer + 1) * k_l], single.cpu().numpy().astype(np.float64))
        assert err <= 1e-5, (layer, err)


def test_resnet_scale_sjlt_on_64_rows(grass):
    n, p, k = 1024, 11173962, 8192
    g = synth.laplace_sparse(n, p, 0.3, 1e-3, seed=1003, device=_dev())
    out = grass.grass_sjlt(g, k, 1, seed=0, stream_id=1)
    torch.cuda.synchronize()
    rows = _sample_rows(n, 64)
    assert len(rows) == 64 and rows[0] == 0 and rows[-1] == n - 1
    got = out[rows].cpu().numpy()
    bucket, sign = orc.sjlt_tables(0, 1, p, k, 1)
    worst = 0.0
    for q, r in enumerate(rows):                                     # the scan of Sec. 3.1, one row at a time
        row = g[r].cpu().numpy().astype(np.float64)
        ref = np.zeros(k)
        np.add.at(ref, bucket[:, 0], sign[:, 0] * row)
        worst = max(worst, orc.max_rel_err(got[q:q + 1], ref[None, :]))
        if q == 0:
            assert orc.max_rel_err(orc.sjlt(row[None, :], k, 1, 0, 1), ref[None, :]) == 0.0   # the oracle's own call
    assert worst <= TOL_SJLT, worst


def test_cache_stage_at_benchmark_size(grass):
    N, k, lam = 65536, 4096, 1e-3
    G = synth.dense_normal(N, k, seed=1005, device=_dev())           # the benchmark's train rows
    F = grass.grass_fim(G)
    info = torch.full((1,), -1, dtype=torch.int32, device=_dev())
    W = grass.grass_fim_inverse(F, lam, info=info)
    pre = grass.grass_ifvp(G, W)
    torch.cuda.synchronize()
    assert int(info.item()) == 0
    Gh = G.cpu().numpy().astype(np.float64)

    # FIM: every entry against G^T G / N in float64
    Fh = F.cpu().numpy()
    assert np.array_equal(Fh, Fh.T)
    ref_F = orc.fim(Gh)
    err_F = orc.max_rel_err(Fh, ref_F)
    assert err_F <= 1e-5, err_F

    # damped inverse of the same fp32 F (lower triangle), against the float64 inverse
    F64 = np.tril(Fh.astype(np.float64))
    F64 = F64 + np.tril(F64, -1).T
    A = F64 + lam * np.eye(k)
    ref_W = np.linalg.inv(A)
    cond = np.linalg.cond(A)
    Wh = W.cpu().numpy().astype(np.float64)
    assert np.array_equal(Wh, Wh.T)
    err_W = orc.max_rel_err(Wh, ref_W)
    assert err_W <= 2.0 ** -23 + cond * 1e-13, (err_W, cond)

    # iFVP of all rows: the oracle solve with the same F, element-wise bound from the fp32 rounding of W and the
    # fp32 accumulation, 4,096 rows at a time to bound host memory
    got = pre.cpu().numpy()
    absW = np.abs(ref_W)
    worst = 0.0
    for r0 in range(0, N, 4096):
        blk = Gh[r0:r0 + 4096]
        ref = orc.ifvp(blk, F64, lam)
        bound = 1e-5 * (np.abs(blk) @ absW) + 1e-30
        ratio = np.abs(got[r0:r0 + 4096] - ref) / bound
        worst = max(worst, float(ratio.max()))
    assert worst <= 1.0, worst


def test_logra_and_factorised_mask_on_the_4096_layer(grass):
    """The comparison baselines of the single-layer benchmark at its size (n = 32 sequences of 512 tokens, 4,096 x 4,096
    layer, factors of 64): LoGra with dense Gaussian factors (Sec. 3.3.2 "Recap on LoGra", Eq. (3)) on the
    producer/consumer kernel - every workgroup streams one whole token tile through all 32 K slices - and the factorised
    mask Mask_{64 (x) 64}, every output against the oracle."""
    n, T, d, kf = 32, 512, 4096, 64
    x, g = synth.linear_layer_factors(n, T, d, d, seed=1004, device=_dev())      # the benchmark's first input pair
    Pi = grass.grass_to_bf16(grass.grass_gauss_matrix(0, 40, d, kf, 0, d, device=_dev()))
    Po = grass.grass_to_bf16(grass.grass_gauss_matrix(0, 41, d, kf, 0, d, device=_dev()))
    out = grass.logra_linear(x, g, Pi, Po)
    ii = grass.grass_mask_indices(0, 16, d, kf, device=_dev())
    io = grass.grass_mask_indices(0, 17, d, kf, device=_dev())
    fm = grass.factmask_linear(x, g, ii, io)
    torch.cuda.synchronize()
    h = lambda t: t.float().cpu().numpy().astype(np.float64)
    ref = orc.logra_linear(h(x), h(g), h(Pi), h(Po))
    assert out.shape == (n, kf * kf)
    assert orc.max_rel_err(out.cpu().numpy(), ref) <= 1e-4        # exact bf16 products, fp32 sums over d and over T
    xs, gs = h(x[:, :, ii.long()]), h(g[:, :, io.long()])
    ref_m = orc.factgrass_sparsified_gradient(xs, gs, np.arange(kf), np.arange(kf))
    assert orc.max_rel_err(fm.cpu().numpy(), ref_m) <= TOL_FACT
