"""The hot-path entry points only enqueue kernels on the caller's stream (no allocation, no host synchronisation, no
memset nodes), so a chain of them can be captured into a HIP graph and replayed: callers with launch-bound loops (many
small layers, small batches) do that.  Every replay is checked against the eager result on the same inputs, with eager
work and synchronisations in between, and the inputs change between replays."""
import numpy as np
import pytest
import torch

import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def grass():
    import paper_2505_18976_amd as g
    g.load_library()
    return g


def test_compression_chain_replays_from_a_graph(grass):
    dev = torch.device("cuda:0")
    n, p, kp, k = 24, 70001, 9000, 1024
    nl, T, kf, kl = 3, 96, 16, 256
    shapes = [(128, 256), (256, 128), (192, 192)]
    g = synth.bernoulli_sparse_normal(n, p, 0.5, 1.0, seed=41, device=dev)
    idx = grass.grass_mask_indices(0, 0, p, kp, device=dev)
    layers = []
    for l, (d_in, d_out) in enumerate(shapes):
        x, go = synth.linear_layer_factors(n, T, d_in, d_out, seed=50 + l, device=dev)
        layers.append((x, go, grass.grass_mask_indices(0, 16 + 4 * l, d_in, kf, device=dev),
                       grass.grass_mask_indices(0, 17 + 4 * l, d_out, kf, device=dev), 18 + 4 * l))
    test_rows = synth.dense_normal(8, k, seed=60, device=dev)

    # static buffers: everything the captured calls touch is allocated up front
    out_a = torch.empty((n, k), dtype=torch.float32, device=dev)
    out_u = torch.empty((n, k), dtype=torch.float32, device=dev)
    out_f = torch.empty((n, nl * kl), dtype=torch.float32, device=dev)
    scores = torch.empty((8, n), dtype=torch.float32, device=dev)
    ws_a = torch.empty(max(grass.grass_sjlt_workspace_bytes(n, p, kp, k, 1), 256), dtype=torch.uint8, device=dev)
    ws_u = torch.empty(max(grass.grass_sjlt_workspace_bytes(n, p, 0, k, 2), 256), dtype=torch.uint8, device=dev)
    ws_f = torch.empty(max(grass.factgrass_layers_workspace_bytes(nl, n, T, kf, kf, kl, 1), 256), dtype=torch.uint8, device=dev)
    ws_s = torch.empty(max(grass.grass_score_workspace_bytes(n, 8, k, 0), 256), dtype=torch.uint8, device=dev)

    def chain():
        grass.grass_sjlt(g, k, 1, seed=0, stream_id=1, idx=idx, out=out_a, ws=ws_a)        # fused GraSS
        grass.grass_sjlt(g, k, 2, seed=0, stream_id=1, out=out_u, ws=ws_u)                 # unmasked SJLT, chunked
        grass.factgrass_layers(layers, kl, 1, 0, out_f, ws=ws_f)                           # three layers, one launch
        grass.grass_score(out_a, test_rows, compute_mode=0, out=scores, ws=ws_s)           # scores of the fresh rows

    def eager():
        chain()
        torch.cuda.synchronize()
        return [t.clone() for t in (out_a, out_u, out_f, scores)]

    want = eager()                                    # also the warm-up every kernel needs before capture
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        chain()
    for replay in range(4):
        if replay:                                    # new inputs in the same buffers; eager reference first
            g.copy_(synth.bernoulli_sparse_normal(n, p, 0.5, 1.0, seed=41 + replay, device=dev))
            for l, (x, go, _, _, _) in enumerate(layers):
                x2, go2 = synth.linear_layer_factors(n, T, shapes[l][0], shapes[l][1], seed=50 + l + 10 * replay, device=dev)
                x.copy_(x2); go.copy_(go2)
            want = eager()
        for t in (out_a, out_u, out_f, scores):
            t.fill_(float("nan"))                     # a replay that skipped a kernel would leave this behind
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, ref in zip((out_a, out_u, out_f, scores), want):
            assert torch.equal(got, ref), replay      # same kernels, same fixed reduction order: bit for bit


def test_cache_and_attribute_stage_replays_from_a_graph(grass):
    """FIM, damped inverse (fp64 Cholesky, tens of dependent launches), iFVP and the score product of the preconditioned
    rows, captured as one graph and replayed on new compressed gradients in the same buffers."""
    dev = torch.device("cuda:0")
    N, k, M, lam = 1500, 320, 40, 1e-2
    G = synth.compressed_gradients(N, k, seed=70, device=dev)
    test_rows = synth.dense_normal(M, k, seed=71, device=dev)
    F = torch.empty((k, k), dtype=torch.float32, device=dev)
    W = torch.empty((k, k), dtype=torch.float32, device=dev)
    pre = torch.empty((N, k), dtype=torch.float32, device=dev)
    scores = torch.empty((M, N), dtype=torch.float32, device=dev)
    info = torch.zeros(1, dtype=torch.int32, device=dev)
    ws_f = torch.empty(max(grass.grass_fim_workspace_bytes(N, k), 256), dtype=torch.uint8, device=dev)
    ws_i = torch.empty(max(grass.grass_fim_inverse_workspace_bytes(k), 256), dtype=torch.uint8, device=dev)
    ws_s = torch.empty(max(grass.grass_score_workspace_bytes(N, M, k, 0), 256), dtype=torch.uint8, device=dev)

    def chain():
        grass.grass_fim(G, out=F, ws=ws_f)
        grass.grass_fim_inverse(F, lam, out=W, info=info, ws=ws_i)
        grass.grass_ifvp(G, W, out=pre)
        grass.grass_score(pre, test_rows, compute_mode=0, out=scores, ws=ws_s)

    def eager():
        chain()
        torch.cuda.synchronize()
        return [t.clone() for t in (F, W, pre, scores)]

    want = eager()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        chain()
    for replay in range(3):
        if replay:
            G.copy_(synth.compressed_gradients(N, k, seed=70 + replay, device=dev))
            want = eager()
        for t in (F, W, pre, scores):
            t.fill_(float("nan"))
        info.fill_(-1)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert int(info.item()) == 0, replay
        for got, ref in zip((F, W, pre, scores), want):
            assert torch.equal(got, ref), replay


def test_selective_mask_training_replays_from_a_graph(grass):
    """The device-side training loop (its temperature schedule is read on the host at capture time) as one graph:
    every replay restarts from the same logits on new gradients and must match the eager run bit for bit."""
    dev = torch.device("cuda:0")
    n, m, p, steps = 140, 128, 5004, 6
    G, Gt, _ = synth.planted_gradients(n, m, p, 64, seed=80, device=dev)
    S0 = synth.dense_normal(1, p, seed=81, device=dev, std=0.1).reshape(-1).contiguous()
    S = S0.clone()
    A = torch.empty((m, n), dtype=torch.float32, device=dev)
    objs = torch.empty(steps, dtype=torch.float64, device=dev)
    temps = np.geomspace(1.0, 0.6, steps)
    ws_a = torch.empty(max(grass.grass_score_workspace_bytes(n, m, p, 0), 256), dtype=torch.uint8, device=dev)
    ws_t = torch.empty(grass.grass_selective_mask_train_workspace_bytes(n, m, p), dtype=torch.uint8, device=dev)

    def chain():
        grass.grass_score(G, Gt, compute_mode=0, out=A, ws=ws_a)
        grass.grass_selective_mask_train(G, Gt, A, S, 1e-4, 50.0, temps, objectives=objs, ws=ws_t)

    def eager():
        S.copy_(S0)
        chain()
        torch.cuda.synchronize()
        return S.clone(), objs.clone()

    want = eager()
    assert not torch.equal(want[0], S0)
    S.copy_(S0)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        chain()
    for replay in range(3):
        if replay:
            G2, Gt2, _ = synth.planted_gradients(n, m, p, 64, seed=80 + replay, device=dev)
            G.copy_(G2); Gt.copy_(Gt2)
            want = eager()
        S.copy_(S0)
        objs.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(S, want[0]) and torch.equal(objs, want[1]), replay
