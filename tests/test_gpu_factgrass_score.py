"""GPU parity: FactGraSS, the score GEMM and the dense Gaussian baseline
against the CPU oracle, through the C ABI.

Bars (max relative error per row, see oracle.max_rel_err): 2e-3 for
bf16-input FactGraSS with fp32 accumulation (its inputs are exact bf16 values);
1e-5 for the fp32-mode GEMMs.  The bf16 modes of the GEMMs round fp32 operands
to bf16 (relative error <= 2^-9 each), so every output obeys
|got - exact| <= (2^-8 + 2^-17) * sum_c |a_c||b_c| plus fp32 accumulation slack;
that bound is checked element by element, next to a loose 1e-2 row-relative cap.
"""
import numpy as np
import pytest
import torch

import synth
from oracle import grass_oracle as orc

pytestmark = pytest.mark.gpu

TOL_FACT = 2e-3
TOL_F32 = 1e-5
TOL_BF16_ROW = 1e-2
BF16_TERM = 2.0 ** -8 + 2.0 ** -17 + 2.0 ** -20


def _check_bf16_mode(got, a, b):
    """got ~ a @ b.T computed from bf16-rounded operands with fp32 accumulation."""
    a = np.asarray(a, dtype=np.float64); b = np.asarray(b, dtype=np.float64)
    exact = a @ b.T
    bound = BF16_TERM * (np.abs(a) @ np.abs(b).T) + 1e-30
    assert np.all(np.abs(got - exact) <= bound)
    assert orc.max_rel_err(got, exact) <= TOL_BF16_ROW


@pytest.fixture(scope="module")
def grass():
    import paper_2505_18976_amd as g
    g.load_library()
    yield g


def _dev():
    return torch.device("cuda:0")


def _np(t):
    return t.float().cpu().numpy()


FACT_CASES = [
    # n, T, d_in, d_out, k_in', k_out', k, s, layer
    (1, 1, 8, 8, 8, 8, 16, 1, 0),               # single token: an outer product
    (2, 5, 40, 24, 7, 3, 8, 1, 1),               # ragged factor widths, T below one tile
    (3, 33, 100, 70, 32, 32, 256, 2, 2),
    (2, 100, 300, 200, 64, 64, 1024, 1, 0),
    (2, 64, 256, 512, 33, 128, 512, 4, 5),
    (1, 200, 128, 128, 128, 128, 4096, 1, 0),   # full masks: SJLT of the whole layer gradient
    (4, 96, 512, 384, 64, 32, 1000, 1, 3),
    (2, 70, 64, 128, 16, 100, 32768, 1, 0),
]


@pytest.mark.parametrize("n,T,d_in,d_out,ka,kb,k,s,layer", FACT_CASES)
def test_factgrass_parity(grass, n, T, d_in, d_out, ka, kb, k, s, layer):
    x, g = synth.linear_layer_factors(n, T, d_in, d_out, seed=40 + layer, device=_dev())
    s_in, s_out, s_sjlt = orc.layer_streams(layer)
    ii = grass.grass_mask_indices(0, s_in, d_in, ka, device=_dev())
    io = grass.grass_mask_indices(0, s_out, d_out, kb, device=_dev())
    out = grass.factgrass_linear(x, g, ii, io, k, s, 0, s_sjlt)
    torch.cuda.synchronize()
    ref = orc.factgrass_linear(_np(x), _np(g), ii.cpu().numpy(), io.cpu().numpy(), k, s, 0, s_sjlt)
    assert orc.max_rel_err(out.cpu().numpy(), ref) <= TOL_FACT


def test_factgrass_random_shapes(grass):
    """30 seeded random layers: tokens, widths, mask sizes (1..128), k and s vary, including non-multiples of every tile."""
    rng = np.random.default_rng(777)
    for case in range(30):
        n, T = int(rng.integers(1, 6)), int(rng.integers(1, 300))
        d_in, d_out = int(rng.integers(1, 700)), int(rng.integers(1, 700))
        ka, kb = int(rng.integers(1, min(d_in, 128) + 1)), int(rng.integers(1, min(d_out, 128) + 1))
        s = int(rng.choice([1, 1, 2, 4]))
        k = s * int(rng.choice([1, 5, 64, 1000, 4096]))
        x, g = synth.linear_layer_factors(n, T, d_in, d_out, seed=7000 + case, device=_dev())
        ii = grass.grass_mask_indices(case, 16, d_in, ka, device=_dev())
        io = grass.grass_mask_indices(case, 17, d_out, kb, device=_dev())
        out = grass.factgrass_linear(x, g, ii, io, k, s, case, 18)
        torch.cuda.synchronize()
        ref = orc.factgrass_linear(_np(x), _np(g), ii.cpu().numpy(), io.cpu().numpy(), k, s, case, 18)
        err = orc.max_rel_err(out.cpu().numpy(), ref)
        assert err <= TOL_FACT, (case, n, T, d_in, d_out, ka, kb, k, s, err)


@pytest.mark.parametrize("n,T,d_in,d_out,ka,kb", [(1, 1, 8, 8, 1, 1), (3, 150, 256, 384, 64, 64), (2, 70, 128, 96, 33, 17),
                                                  (4, 300, 512, 512, 128, 128), (5, 40, 64, 700, 7, 100)])
def test_factmask_parity(grass, n, T, d_in, d_out, ka, kb):
    """Mask_{k_in x k_out} (Sec. 3.3.2): the sparsified gradient itself, flat index a*k_out' + b."""
    x, g = synth.linear_layer_factors(n, T, d_in, d_out, seed=45, device=_dev())
    ii = grass.grass_mask_indices(0, 16, d_in, ka, device=_dev())
    io = grass.grass_mask_indices(0, 17, d_out, kb, device=_dev())
    wide = torch.full((n, ka * kb + 5), 3.0, dtype=torch.float32, device=_dev())
    grass.factmask_linear(x, g, ii, io, out=wide[:, :ka * kb])
    torch.cuda.synchronize()
    ref = orc.factgrass_sparsified_gradient(_np(x), _np(g), ii.cpu().numpy(), io.cpu().numpy())
    assert orc.max_rel_err(wide[:, :ka * kb].cpu().numpy(), ref) <= TOL_FACT
    assert torch.all(wide[:, ka * kb:] == 3.0)


@pytest.mark.parametrize("p,k,s,kp", [(1, 1, 1, 0), (300, 16, 1, 0), (4099, 64, 4, 0), (5000, 48, 3, 0), (5000, 64, 1, 700),
                                      (65536, 1024, 2, 8192)])
def test_projection_matrix_bit_exact(grass, p, k, s, kp):
    idx = grass.grass_mask_indices(2, 0, p, kp, device=_dev()) if kp else None
    P = grass.grass_projection_matrix(4, 1, p, k, s, idx=idx, device=_dev())
    torch.cuda.synchronize()
    if p * k <= 400000:
        ref = orc.projection_matrix(4, 1, p, k, s, None if idx is None else orc.mask_indices(2, 0, p, kp))
        assert np.array_equal(P.cpu().numpy(), ref.astype(np.float32))
    # P g equals the scan on the GPU as well
    g = synth.dense_normal(3, p, seed=46, device=_dev())
    via_matrix = (g.double() @ P.double().T).cpu().numpy()
    direct = grass.grass_sjlt(g, k, s, seed=4, stream_id=1, idx=idx)
    torch.cuda.synchronize()
    assert orc.max_rel_err(direct.cpu().numpy(), via_matrix) <= 1e-5


@pytest.mark.parametrize("n,T,d,k_in,k_out,masked", [(2, 100, 256, 16, 32, False), (3, 130, 512, 64, 64, False),
                                                     (2, 64, 1024, 64, 64, True)])
def test_factorised_sjlt_and_grass_baselines_through_the_dense_kernel(grass, n, T, d, k_in, k_out, masked):
    """SJLT_{k_in x k_out} / GraSS_{k_in x k_out}: logra_linear with the compressors' dense matrices (s = 1, exact in bf16)."""
    x, g = synth.linear_layer_factors(n, T, d, d, seed=47, device=_dev())
    ii = grass.grass_mask_indices(0, 16, d, d // 4, device=_dev()) if masked else None
    io = grass.grass_mask_indices(0, 17, d, d // 4, device=_dev()) if masked else None
    Pi = grass.grass_projection_matrix(0, 40, d, k_in, 1, idx=ii, device=_dev())
    Po = grass.grass_projection_matrix(0, 41, d, k_out, 1, idx=io, device=_dev())
    out = grass.logra_linear(x, g, grass.grass_to_bf16(Pi), grass.grass_to_bf16(Po))
    torch.cuda.synchronize()
    Pih = orc.projection_matrix(0, 40, d, k_in, 1, None if ii is None else ii.cpu().numpy())
    Poh = orc.projection_matrix(0, 41, d, k_out, 1, None if io is None else io.cpu().numpy())
    ref = orc.logra_linear(_np(x), _np(g), Pih, Poh)
    assert orc.max_rel_err(out.cpu().numpy(), ref) <= 1e-4


@pytest.mark.parametrize("tokens", [32, 64, 4096])
def test_factgrass_token_chunking(grass, tokens):
    n, T, d_in, d_out, ka, kb, k = 3, 150, 256, 256, 64, 64, 1024
    x, g = synth.linear_layer_factors(n, T, d_in, d_out, seed=50, device=_dev())
    ii = grass.grass_mask_indices(0, 16, d_in, ka, device=_dev())
    io = grass.grass_mask_indices(0, 17, d_out, kb, device=_dev())
    ref = orc.factgrass_linear(_np(x), _np(g), ii.cpu().numpy(), io.cpu().numpy(), k, 1, 0, 18)
    out = grass.factgrass_linear(x, g, ii, io, k, 1, 0, 18, tuning=dict(factgrass_tokens_per_block=tokens))
    torch.cuda.synchronize()
    assert orc.max_rel_err(out.cpu().numpy(), ref) <= TOL_FACT


def test_factgrass_concatenated_layers(grass):
    """Layer l lands at its column offset of a concatenated row (k = sum_l k_l)."""
    n, T, k_l = 2, 48, 256
    shapes = [(128, 128), (128, 512), (512, 128)]
    cat = torch.zeros((n, k_l * len(shapes)), dtype=torch.float32, device=_dev())
    refs = []
    for l, (d_in, d_out) in enumerate(shapes):
        x, g = synth.linear_layer_factors(n, T, d_in, d_out, seed=60 + l, device=_dev())
        s_in, s_out, s_sjlt = orc.layer_streams(l)
        ii = grass.grass_mask_indices(0, s_in, d_in, 64, device=_dev())
        io = grass.grass_mask_indices(0, s_out, d_out, 64, device=_dev())
        grass.factgrass_linear(x, g, ii, io, k_l, 1, 0, s_sjlt, out=cat[:, l * k_l:(l + 1) * k_l])
        refs.append(orc.factgrass_linear(_np(x), _np(g), ii.cpu().numpy(), io.cpu().numpy(), k_l, 1, 0, s_sjlt))
    torch.cuda.synchronize()
    got = cat.cpu().numpy()
    for l, ref in enumerate(refs):
        assert orc.max_rel_err(got[:, l * k_l:(l + 1) * k_l], ref) <= TOL_FACT


@pytest.mark.parametrize("tokens", [0, 32])
def test_factgrass_many_layers_in_one_launch(grass, tokens):
    """factgrass_layers == factgrass_linear layer by layer == the oracle."""
    n, T, k_l, kf = 3, 80, 512, 64
    shapes = [(128, 128), (128, 512), (512, 128), (256, 192), (128, 128)]
    cat = torch.full((n, k_l * len(shapes) + 7), -1.0, dtype=torch.float32, device=_dev())
    layers, refs = [], []
    for l, (d_in, d_out) in enumerate(shapes):
        x, g = synth.linear_layer_factors(n, T, d_in, d_out, seed=90 + l, device=_dev())
        s_in, s_out, s_sjlt = orc.layer_streams(l)
        ii = grass.grass_mask_indices(0, s_in, d_in, kf, device=_dev())
        io = grass.grass_mask_indices(0, s_out, d_out, kf, device=_dev())
        layers.append((x, g, ii, io, s_sjlt))
        refs.append(orc.factgrass_linear(_np(x), _np(g), ii.cpu().numpy(), io.cpu().numpy(), k_l, 1, 0, s_sjlt))
    grass.factgrass_layers(layers, k_l, 1, 0, cat, tuning=dict(factgrass_tokens_per_block=tokens))
    torch.cuda.synchronize()
    got = cat.cpu().numpy()
    for l, ref in enumerate(refs):
        assert orc.max_rel_err(got[:, l * k_l:(l + 1) * k_l], ref) <= TOL_FACT
    assert np.all(got[:, k_l * len(shapes):] == -1.0)          # columns beyond the last block are untouched


# ------------------------------------------------------------------- LoGra
TOL_LOGRA = 1e-4      # two chained fp32 accumulations (over d and over T) of exact bf16 products

LOGRA_CASES = [
    # n, T, d_in, d_out, k_in, k_out
    (1, 1, 8, 8, 1, 1),
    (2, 5, 40, 24, 7, 3),
    (3, 70, 128, 256, 16, 16),
    (2, 130, 264, 200, 32, 64),
    (2, 300, 512, 384, 64, 64),
    (8, 64, 2048, 2048, 64, 64),
    (64, 520, 264, 1096, 48, 64),     # two token tiles per workgroup and a ragged last chunk; d_out >> d_in, 18 half slices
]


@pytest.mark.parametrize("n,T,d_in,d_out,ki,ko", LOGRA_CASES)
def test_logra_parity(grass, n, T, d_in, d_out, ki, ko):
    x, g = synth.linear_layer_factors(n, T, d_in, d_out, seed=95, device=_dev())
    Pi = grass.grass_to_bf16(grass.grass_gauss_matrix(0, 40, d_in, ki, 0, d_in, device=_dev()))
    Po = grass.grass_to_bf16(grass.grass_gauss_matrix(0, 41, d_out, ko, 0, d_out, device=_dev()))
    out = grass.logra_linear(x, g, Pi, Po)
    torch.cuda.synchronize()
    ref = orc.logra_linear(_np(x), _np(g), _np(Pi), _np(Po))
    assert out.shape == (n, ki * ko)
    assert orc.max_rel_err(out.cpu().numpy(), ref) <= TOL_LOGRA


def test_logra_with_selection_matrices_matches_factgrass_mask_stage(grass):
    """Mask_{k_in (x) k_out}: LoGra's kernel fed selection matrices reproduces FactGraSS's sparsified gradient."""
    n, T, d_in, d_out, kf = 2, 96, 256, 128, 32
    x, g = synth.linear_layer_factors(n, T, d_in, d_out, seed=96, device=_dev())
    ii = grass.grass_mask_indices(0, 16, d_in, kf, device=_dev())
    io = grass.grass_mask_indices(0, 17, d_out, kf, device=_dev())
    Mi = torch.zeros((kf, d_in), dtype=torch.bfloat16, device=_dev()); Mi[torch.arange(kf), ii.long()] = 1
    Mo = torch.zeros((kf, d_out), dtype=torch.bfloat16, device=_dev()); Mo[torch.arange(kf), io.long()] = 1
    out = grass.logra_linear(x, g, Mi, Mo)
    torch.cuda.synchronize()
    ref = orc.factgrass_sparsified_gradient(_np(x), _np(g), ii.cpu().numpy(), io.cpu().numpy())
    assert orc.max_rel_err(out.cpu().numpy(), ref) <= TOL_LOGRA


# ------------------------------------------------------------------- score
SCORE_CASES = [(1, 1, 1), (5, 3, 7), (130, 129, 33), (256, 128, 64), (300, 200, 1000), (1024, 512, 4096), (257, 64, 70),
               (200, 130, 8192), (130, 129, 12304), (129, 3, 5000),      # few tiles, long K: split over K ranges
               (128, 128, 16), (256, 256, 48), (384, 130, 4112),         # an odd number of 64-byte slices: half group last
               (1000, 128, 8192), (700, 100, 4096), (400, 300, 4096), (2048, 384, 1040), (513, 257, 4112),   # few test rows: 128 x 384 tiles
               (4096, 4096, 96), (2048, 8192, 64)]      # many tile rows: tiles dealt to the XCDs in blocks of 8 x 4


@pytest.mark.parametrize("N,M,K", SCORE_CASES)
@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("with_ws", [True, False])
def test_score_parity(grass, N, M, K, mode, with_ws):
    """with_ws: the optional workspace (operands rounded once for mode 1, K-range partial sums); without it the
    on-the-fly paths.  Both must meet the same bars."""
    train = synth.dense_normal(N, K, seed=70, device=_dev())
    test = synth.dense_normal(M, K, seed=71, device=_dev())
    sc = grass.grass_score(train, test, compute_mode=mode, ws=True if with_ws else None)
    torch.cuda.synchronize()
    ref = orc.score(train.cpu().numpy(), test.cpu().numpy())
    assert sc.shape == (M, N)
    if mode == 0:
        assert orc.max_rel_err(sc.cpu().numpy(), ref) <= TOL_F32
    else:
        _check_bf16_mode(sc.cpu().numpy(), test.cpu().numpy(), train.cpu().numpy())


BF16_SCORE_CASES = [(1, 1, 8), (300, 200, 1000), (256, 256, 64), (257, 255, 72), (1024, 512, 4096), (700, 1024, 136),
                    (256, 256, 32), (300, 260, 96), (384, 130, 4128),       # odd numbers of 64-byte slices
                    (4096, 4096, 128), (1024, 16384, 64)]                   # many tile rows (blocks of 8 x 4 tiles per XCD)


@pytest.mark.parametrize("N,M,K", BF16_SCORE_CASES)
def test_score_bf16_inputs_parity(grass, N, M, K):
    """bf16 operands are exact inputs: only the fp32 accumulation order differs from the oracle."""
    train = synth.dense_normal(N, K, seed=76, device=_dev())
    test = synth.dense_normal(M, K, seed=77, device=_dev())
    trb, teb = grass.grass_to_bf16(train), grass.grass_to_bf16(test)
    torch.cuda.synchronize()
    # the conversion is round-to-nearest-even, bit for bit what torch does
    assert torch.equal(trb, train.to(torch.bfloat16)) and torch.equal(teb, test.to(torch.bfloat16))
    sc = grass.grass_score_bf16(trb, teb)
    torch.cuda.synchronize()
    ref = orc.score(trb.float().cpu().numpy(), teb.float().cpu().numpy())
    assert sc.shape == (M, N)
    assert orc.max_rel_err(sc.cpu().numpy(), ref) <= TOL_F32


def test_score_bf16_rejects_unaligned_k(grass):
    tr = torch.zeros((16, 12), dtype=torch.bfloat16, device=_dev())
    with pytest.raises(grass.GrassError) as e:
        grass.grass_score_bf16(tr, tr)
    assert e.value.status == grass.GRASS_EUNSUPPORTED


def test_score_unaligned_leading_dimensions(grass):
    N, M, K = 70, 40, 50
    tr = synth.dense_normal(N, K + 1, seed=72, device=_dev())[:, :K]
    te = synth.dense_normal(M, K + 3, seed=73, device=_dev())[:, :K]
    sc = grass.grass_score(tr, te, compute_mode=0)
    torch.cuda.synchronize()
    assert orc.max_rel_err(sc.cpu().numpy(), orc.score(tr.cpu().numpy(), te.cpu().numpy())) <= TOL_F32


def test_score_of_compressed_gradients_end_to_end(grass):
    """compress train and test gradients with GraSS, then score them."""
    p, kp, k = 20000, 4000, 512
    gtr = synth.bernoulli_sparse_normal(96, p, 0.7, 1.0, seed=74, device=_dev())
    gte = synth.bernoulli_sparse_normal(8, p, 0.7, 1.0, seed=75, device=_dev())
    idx = grass.grass_mask_indices(0, 0, p, kp, device=_dev())
    ctr = grass.grass_sjlt(gtr, k, 1, 0, 1, idx=idx)
    cte = grass.grass_sjlt(gte, k, 1, 0, 1, idx=idx)
    sc = grass.grass_score(ctr, cte, compute_mode=0)
    torch.cuda.synchronize()
    i = idx.cpu().numpy()
    ref = orc.score(orc.grass(gtr.cpu().numpy(), i, k, 1, 0, 1), orc.grass(gte.cpu().numpy(), i, k, 1, 0, 1))
    assert orc.max_rel_err(sc.cpu().numpy(), ref) <= 2e-5


# -------------------------------------------------------- Gaussian baseline
def test_gauss_matrix_moments_and_chunk_consistency(grass):
    p, k = 6000, 64
    P = grass.grass_gauss_matrix(3, 2, p, k, 0, p, device=_dev())
    part = grass.grass_gauss_matrix(3, 2, p, k, 1000, 500, device=_dev())
    torch.cuda.synchronize()
    Pn = P.cpu().numpy().astype(np.float64)
    assert np.array_equal(part.cpu().numpy(), P[:, 1000:1500].cpu().numpy())
    z = Pn.ravel() * np.sqrt(k)
    nz = z.size
    assert abs(z.mean()) < 4 / np.sqrt(nz)
    assert abs(z.var() - 1) < 4 * np.sqrt(2 / nz)
    assert abs((z ** 4).mean() - 3) < 4 * np.sqrt(96 / nz)
    assert abs(np.corrcoef(z[:-1], z[1:])[0, 1]) < 4 / np.sqrt(nz)


@pytest.mark.parametrize("seed,stream,p,k,p0,pc", [(1, 2, 5001, 130, 0, 5001), (7, 40, 300, 257, 0, 300),
                                                   (3, 2, 11173962, 70, 11173000, 962), (0, 2, 1, 1, 0, 1)])
def test_gauss_matrix_parity(grass, seed, stream, p, k, p0, pc):
    """Box-Muller in fp32 against the fp64 oracle: both start from the same exactly representable uniforms, so the
    only difference is the rounding of logf, sqrtf and cospif (a few ulp of a value of magnitude <= 5.8/sqrt(k))."""
    P = grass.grass_gauss_matrix(seed, stream, p, k, p0, pc, device=_dev())
    torch.cuda.synchronize()
    ref = orc.gauss_matrix(seed, stream, p, k, p0, pc)
    assert P.shape == ref.shape
    assert np.abs(P.cpu().numpy().astype(np.float64) - ref).max() * np.sqrt(k) <= 4e-6


@pytest.mark.parametrize("n,p,k,chunk,mode", [(3, 100, 8, 0, 0), (70, 5001, 130, 1024, 0), (70, 5001, 130, 1024, 1),
                                              (256, 16384, 256, 4096, 1), (33, 4098, 64, 4096, 0),
                                              # few output tiles: the contraction is split over K ranges
                                              (256, 16384, 256, 4096, 0), (130, 20000, 300, 8192, 1), (200, 5001, 128, 1024, 1), (130, 20000, 300, 8192, 0),
                                              (128, 9000, 128, 4104, 0), (200, 2048, 128, 0, 0),
                                              # rows of g not 16-byte aligned: fp32 chunks are staged in the workspace
                                              (200, 5001, 128, 1024, 0), (130, 20002, 300, 8192, 0), (129, 8191, 130, 0, 0)])
def test_gauss_project_parity(grass, n, p, k, chunk, mode):
    g = synth.laplace_sparse(n, p, 0.3, 1e-3, seed=80, device=_dev())
    out = grass.grass_gauss_project(g, k, seed=1, stream_id=2, p_chunk=chunk, compute_mode=mode)
    torch.cuda.synchronize()
    P = orc.gauss_matrix(1, 2, p, k)
    ref = orc.gauss_project(g.cpu().numpy(), P)
    if mode == 0:
        assert orc.max_rel_err(out.cpu().numpy(), ref) <= TOL_F32
    else:
        _check_bf16_mode(out.cpu().numpy(), g.cpu().numpy(), P.astype(np.float32))
