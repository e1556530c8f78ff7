"""GPU parity at the full benchmark sizes, in the launch configuration bench.py
times, checked on sampled outputs the oracle can compute one by one.

Workloads (seeded synthetic stand-ins from synth.py for gradients that are not
available): MLP-scale Mask+SJLT
(n=4,096, p=1,863,690, k'=65,536, k=4,096, s=1 and 4); ResNet-scale SJLT
(n=1,024, p=11,173,962, k=8,192) and a column slice of the dense Gaussian
baseline; FactGraSS on a 4,096 x 4,096 linear layer (n=32, T=512); FactGraSS
over Llama-style layers (hidden 2,048, MLP 8,192, n=8, T=1,024) written into a
concatenated row; the score GEMM of 65,536 train rows against 1,024 test rows.
"""
import numpy as np
import pytest
import torch

import synth
from oracle import grass_oracle as orc

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def grass():
    import paper_2505_18976_amd as g
    g.load_library()
    return g


def _dev():
    return torch.device("cuda:0")


def _sample_rows(n, count):
    return sorted(set(np.linspace(0, n - 1, count).round().astype(int).tolist()))


def test_mlp_scale_mask_sjlt(grass):
    n, p, kp, k = 4096, synth.mlp_num_params(), 65536, 4096
    assert p == 1863690
    g = synth.mlp_relu_gradients(n, seed=1002, device=_dev())
    idx = grass.grass_mask_indices(0, 0, p, kp, device=_dev())
    idx_h = idx.cpu().numpy()
    assert np.array_equal(idx_h, orc.mask_indices(0, 0, p, kp))
    rows = _sample_rows(n, 64)
    g_rows = g[rows].cpu().numpy()
    zero_frac = float((g_rows == 0).mean())
    assert 0.45 < zero_frac < 0.55                       # ReLU-style zeros, about half
    for s in (1, 4):
        out = grass.grass_sjlt(g, k, s, seed=0, stream_id=1, idx=idx)
        torch.cuda.synchronize()
        ref = orc.grass(g_rows, idx_h, k, s, 0, 1)
        assert orc.max_rel_err(out[rows].cpu().numpy(), ref) <= 1e-5
    # the un-fused gather is a copy: exact
    gm = grass.grass_mask(g, idx)
    torch.cuda.synchronize()
    assert np.array_equal(gm[rows].cpu().numpy(), g_rows[:, idx_h])


def test_resnet_scale_sjlt_and_gaussian_slice(grass):
    n, p, k = 1024, 11173962, 8192
    g = synth.laplace_sparse(n, p, 0.3, 1e-3, seed=1003, device=_dev())
    out = grass.grass_sjlt(g, k, 1, seed=0, stream_id=1)
    torch.cuda.synchronize()
    rows = _sample_rows(n, 5)
    g_rows = g[rows].cpu().numpy()
    assert 0.29 < float((g_rows == 0).mean()) < 0.31
    ref = orc.sjlt(g_rows, k, 1, 0, 1)
    assert orc.max_rel_err(out[rows].cpu().numpy(), ref) <= 1e-5
    # properties that hold at any size: every non-zero lands in exactly one bucket with a
    # +-1 sign, so the bucket sums cannot exceed the row's L1 norm, and E||.||^2 is preserved
    o = out[rows].cpu().numpy().astype(np.float64)
    assert np.all(np.abs(o).sum(axis=1) <= np.abs(g_rows.astype(np.float64)).sum(axis=1) * (1 + 1e-6))
    ratio = (o ** 2).sum(axis=1) / (g_rows.astype(np.float64) ** 2).sum(axis=1)
    assert np.all(np.abs(ratio - 1) < 6 * np.sqrt(2.0 / k))

    # dense Gaussian baseline on the first 131,072 columns (the full P would be 366 GB)
    pc, chunk = 131072, 32768
    gs = g[:, :pc]
    for mode in (0, 1):
        og = grass.grass_gauss_project(gs, k, seed=0, stream_id=2, p_chunk=chunk, compute_mode=mode)
        torch.cuda.synchronize()
        buckets = [0, 1, 4095, 8191]
        Prows = orc.gauss_matrix(0, 2, pc, k, rows=buckets)
        gr = g_rows[:, :pc].astype(np.float64)
        exact = gr @ Prows.T
        got = og[rows][:, buckets].cpu().numpy()
        if mode == 0:
            assert np.abs(got - exact).max() <= 1e-5 * np.abs(exact).max() * 4
        else:
            bound = (2.0 ** -8 + 2.0 ** -17 + 2.0 ** -20) * (np.abs(gr) @ np.abs(Prows).T)
            assert np.all(np.abs(got - exact) <= bound)


def test_factgrass_one_4096_layer(grass):
    n, T, d, kf, k = 32, 512, 4096, 64, 1024
    x, g = synth.linear_layer_factors(n, T, d, d, seed=1004, device=_dev())
    s_in, s_out, s_sjlt = orc.layer_streams(0)
    ii = grass.grass_mask_indices(0, s_in, d, kf, device=_dev())
    io = grass.grass_mask_indices(0, s_out, d, kf, device=_dev())
    out = grass.factgrass_linear(x, g, ii, io, k, 1, 0, s_sjlt)
    torch.cuda.synchronize()
    ii_h, io_h = ii.cpu().numpy(), io.cpu().numpy()
    assert np.array_equal(ii_h, orc.mask_indices(0, s_in, d, kf))
    assert np.array_equal(io_h, orc.mask_indices(0, s_out, d, kf))
    xs = x[:, :, ii.long()].float().cpu().numpy()        # the oracle only needs the kept columns
    gs = g[:, :, io.long()].float().cpu().numpy()
    ref = orc.factgrass_linear(xs, gs, np.arange(kf), np.arange(kf), k, 1, 0, s_sjlt)
    assert orc.max_rel_err(out.cpu().numpy(), ref) <= 2e-3


def test_factgrass_llama_style_layers_and_score(grass):
    n, T, kf, k_l = 8, 1024, 64, 4096
    linears = synth.LLAMA_BLOCK_LINEARS
    layers = list(range(7)) + [7 * 15 + 4, 7 * 15 + 6]           # first block, and two of the last
    buffers = {}
    for name, d_in, d_out in linears:                              # one input buffer per distinct shape
        if (d_in, d_out) not in buffers:
            buffers[(d_in, d_out)] = synth.linear_layer_factors(n, T, d_in, d_out, seed=1005 + len(buffers),
                                                                device=_dev())
    cat = torch.zeros((n, k_l * len(layers)), dtype=torch.float32, device=_dev())
    refs = []
    for slot, layer in enumerate(layers):
        name, d_in, d_out = linears[layer % 7]
        x, g = buffers[(d_in, d_out)]
        s_in, s_out, s_sjlt = orc.layer_streams(layer)
        ii = grass.grass_mask_indices(0, s_in, d_in, kf, device=_dev())
        io = grass.grass_mask_indices(0, s_out, d_out, kf, device=_dev())
        grass.factgrass_linear(x, g, ii, io, k_l, 1, 0, s_sjlt, out=cat[:, slot * k_l:(slot + 1) * k_l])
        xs = x[:, :, ii.long()].float().cpu().numpy()
        gs = g[:, :, io.long()].float().cpu().numpy()
        refs.append(orc.factgrass_linear(xs, gs, np.arange(kf), np.arange(kf), k_l, 1, 0, s_sjlt))
    torch.cuda.synchronize()
    got = cat.cpu().numpy()
    for slot, ref in enumerate(refs):
        assert orc.max_rel_err(got[:, slot * k_l:(slot + 1) * k_l], ref) <= 2e-3

    # score GEMM: 65,536 compressed train rows against 1,024 test rows, one layer block wide
    N, M, K = 65536, 1024, 4096
    train = synth.dense_normal(N, K, seed=1010, device=_dev())
    test = synth.dense_normal(M, K, seed=1011, device=_dev())
    tr_rows = _sample_rows(N, 48)
    te_rows = _sample_rows(M, 24)
    exact = orc.score(train[tr_rows].cpu().numpy(), test[te_rows].cpu().numpy())
    sc = grass.grass_score(train, test, compute_mode=0)
    torch.cuda.synchronize()
    got = sc[te_rows][:, tr_rows].cpu().numpy()
    assert np.abs(got - exact).max() <= 1e-5 * np.abs(exact).max() * 4
    sc = grass.grass_score(train, test, compute_mode=1)
    torch.cuda.synchronize()
    got = sc[te_rows][:, tr_rows].cpu().numpy()
    a = np.abs(test[te_rows].cpu().numpy().astype(np.float64))
    b = np.abs(train[tr_rows].cpu().numpy().astype(np.float64))
    assert np.all(np.abs(got - exact) <= (2.0 ** -8 + 2.0 ** -17 + 2.0 ** -20) * (a @ b.T))


def test_sjlt_at_the_largest_input_dimension(grass):
    """p = 2**31 - 1, the largest the entry points accept (indices are int32): two rows of 8.6 GB, zero except for
    a few thousand entries that include the first and the last position, so that the oracle needs the table entries
    of those positions only.  Unmasked (s = 1 and 2) and through a mask that keeps the last coordinate."""
    p, k = 2**31 - 1, 4096
    rng = np.random.default_rng(77)
    g = torch.zeros((2, p), dtype=torch.float32, device=_dev())
    pos, val = [], []
    for i in range(2):
        j = np.unique(np.concatenate([[0, p - 1, p - 2, 2**30, 2**24 + 1], rng.integers(0, p, 3000)])).astype(np.int64)
        v = rng.standard_normal(j.size).astype(np.float32)
        g[i, torch.from_numpy(j).to(_dev())] = torch.from_numpy(v).to(_dev())
        pos.append(j); val.append(v)
    for s in (1, 2):
        out = grass.grass_sjlt(g, k, s, seed=5, stream_id=1)
        torch.cuda.synchronize()
        ref = np.zeros((2, k))
        for i in range(2):
            bucket, sign = orc.sjlt_entries(5, 1, pos[i], k, s)
            for r in range(s):
                np.add.at(ref[i], bucket[:, r], sign[:, r] * val[i].astype(np.float64) / np.sqrt(s))
        assert orc.max_rel_err(out.cpu().numpy(), ref) <= 1e-5, s
    # fused mask: 6,000 kept coordinates, among them the first and last coordinates and every planted non-zero of row 0
    keep = np.unique(np.concatenate([pos[0][:2500], [0, p - 1], rng.integers(0, p, 3500)])).astype(np.int32)
    idx = torch.from_numpy(keep).to(_dev())
    assert grass.grass_check_indices(idx, p)
    out = grass.grass_sjlt(g, k, 1, seed=5, stream_id=1, idx=idx)
    gathered = grass.grass_mask(g, idx)
    torch.cuda.synchronize()
    small = g[:, idx.long()].cpu().numpy()
    assert np.array_equal(gathered.cpu().numpy(), small)
    ref = orc.sjlt(small, k, 1, 5, 1)
    assert orc.max_rel_err(out.cpu().numpy(), ref) <= 1e-5
    # one past the limit is refused before any launch
    with pytest.raises(Exception):
        grass.grass_sjlt_workspace_bytes(2, 2**31, 0, k, 1)


def test_mask_indices_at_the_largest_input_dimension(grass):
    """Random Mask over p = 2**31 - 1 coordinates.  The oracle cannot rank two billion keys in the time a test has, so
    the result is checked through what defines it: k' ascending distinct indices in range whose keys (oracle hash of
    exactly those indices) are all smaller than the key of every coordinate left out -- verified on four million
    left-out coordinates, among them the neighbours of every kept one and both ends -- and whose largest key sits
    where the k'-th order statistic of p uniform 64-bit keys must (k'/p of the key range, within 6 sigma)."""
    p, kp, seed, stream = 2**31 - 1, 65536, 3, 0
    idx = grass.grass_mask_indices(seed, stream, p, kp, device=_dev())
    torch.cuda.synchronize()
    assert grass.grass_check_indices(idx, p)
    kept = idx.cpu().numpy().astype(np.int64)
    assert kept.size == kp and np.all(np.diff(kept) > 0) and kept[0] >= 0 and kept[-1] < p
    keys = orc.stream_hash(seed, stream, kept.astype(np.uint64))
    T = int(keys.max())
    rng = np.random.default_rng(5)
    probe = np.unique(np.concatenate([rng.integers(0, p, 4_000_000), kept + 1, kept - 1, [0, 1, p - 2, p - 1]]))
    probe = probe[(probe >= 0) & (probe < p)]
    probe = np.setdiff1d(probe, kept)
    other = orc.stream_hash(seed, stream, probe.astype(np.uint64))
    assert int(other.min()) > T
    frac = T / 2.0**64
    assert abs(frac - kp / p) <= 6 * np.sqrt(kp) / p
    # the same call at a small size agrees with the oracle's full ranking (same kernels, same launch path)
    small = grass.grass_mask_indices(seed, stream, 100003, 777, device=_dev())
    assert np.array_equal(small.cpu().numpy(), orc.mask_indices(seed, stream, 100003, 777))


def test_calls_follow_the_callers_stream(grass):
    """Every entry point enqueues on the stream it is given (torch's current stream in the binding): run a chain on a
    side stream while the default stream is kept busy, and compare with the same chain on the default stream."""
    n, p, kp, k = 64, 30000, 4000, 256
    g = synth.bernoulli_sparse_normal(n, p, 0.5, 1.0, seed=1400, device=_dev())
    x, go = synth.linear_layer_factors(4, 96, 256, 256, seed=1401, device=_dev())

    def chain():
        idx = grass.grass_mask_indices(1, 0, p, kp, device=_dev())
        c = grass.grass_sjlt(g, k, 1, seed=1, stream_id=1, idx=idx)
        W = grass.grass_fim_inverse(grass.grass_fim(c), 0.1)
        s = grass.grass_score(grass.grass_ifvp(c, W), c)
        ii = grass.grass_mask_indices(1, 16, 256, 64, device=_dev())
        io = grass.grass_mask_indices(1, 17, 256, 64, device=_dev())
        f = grass.factgrass_linear(x, go, ii, io, 512, 1, 1, 18)
        return s, f

    ref_s, ref_f = chain()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    busy = torch.empty(1 << 26, dtype=torch.float32, device=_dev())
    with torch.cuda.stream(side):
        side.wait_stream(torch.cuda.current_stream())
    for _ in range(3):
        busy.normal_()                                # default stream has work queued
    with torch.cuda.stream(side):
        s, f = chain()
    side.synchronize()
    assert torch.equal(s, ref_s) and torch.equal(f, ref_f)
    torch.cuda.synchronize()
