"""grass_sjlt_noalloc (the entry point for callers that cannot allocate: it keeps its scratch memory in a fixed buffer
inside the library) against grass_sjlt, through the C ABI.

Calls in a row share the buffer, so every case runs twice in sequence with a smaller problem second; the shapes are
chosen so that the kernels really use the buffer (several column chunks per row group; the transient bucket table).
Bar: the SJLT bar, 1e-5 row-relative, against the workspace entry point and against the oracle.
"""
import ctypes

import numpy as np
import pytest
import torch

import synth
from oracle import grass_oracle as orc

pytestmark = pytest.mark.gpu

TOL = 1e-5


@pytest.fixture(scope="module")
def grass():
    import paper_2505_18976_amd as g
    g.load_library()
    return g


def _dev():
    return torch.device("cuda:0")


def _raw_noalloc(grass, g, idx, k, s, seed, stream_id, out):
    """The C entry point itself, called with plain pointers and sizes."""
    lib = grass.load_library()
    n, p = g.shape
    st = lib.grass_sjlt_noalloc(ctypes.c_void_p(g.data_ptr()), n, p, g.stride(0),
                                ctypes.c_void_p(0 if idx is None else idx.data_ptr()), 0 if idx is None else idx.numel(),
                                k, s, seed, stream_id, ctypes.c_void_p(out.data_ptr()), out.stride(0),
                                ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    return st


def _case(grass, n, p, kp, k, s, seed, data_seed):
    g = synth.bernoulli_sparse_normal(n, p, 0.5, 1.0, seed=data_seed, device=_dev())
    idx = None if kp == 0 else grass.grass_mask_indices(seed, 0, p, kp, device=_dev())
    # the workspace entry point must need scratch memory here, or the case would not exercise the buffer
    need = grass.grass_sjlt_workspace_bytes(n, p, kp, k, s)
    assert 0 < need
    want = grass.grass_sjlt(g, k, s, seed, 1, idx=idx)
    out = torch.full((n, k), float("nan"), dtype=torch.float32, device=_dev())
    assert _raw_noalloc(grass, g, idx, k, s, seed, 1, out) == grass.GRASS_OK
    torch.cuda.synchronize()
    gh = g.cpu().numpy()
    ref = orc.sjlt(gh, k, s, seed, 1) if idx is None else orc.grass(gh, idx.cpu().numpy(), k, s, seed, 1)
    got = out.cpu().numpy()
    assert np.isfinite(got).all()
    assert orc.max_rel_err(got, want.cpu().numpy().astype(np.float64)) <= TOL
    assert orc.max_rel_err(got, ref) <= TOL


def test_two_calls_in_a_row_second_one_smaller(grass):
    # fused mask, small batch: 16 row groups x 16 column chunks of partial sums in the buffer
    _case(grass, n=16, p=200000, kp=65536, k=1024, s=1, seed=3, data_seed=4100)
    # smaller problem right after it, unmasked, ragged sizes, s = 2
    _case(grass, n=8, p=100003, kp=0, k=512, s=2, seed=4, data_seed=4101)


def test_table_path_then_smaller_masked(grass):
    # unmasked long rows with the transient bucket table behind the partial sums (16.8 MB + 0.26 MB)
    _case(grass, n=128, p=131072, kp=0, k=2048, s=1, seed=5, data_seed=4102)
    _case(grass, n=5, p=70001, kp=40000, k=256, s=4, seed=6, data_seed=4103)


def test_too_large_is_refused_and_large_fused_batches_need_no_scratch(grass):
    # 2 chunks x 1,024 rows x 8,192 buckets of partial sums = 64 MiB > 32 MiB: refused on the host, nothing launched
    fake = torch.empty(16, dtype=torch.float32, device=_dev())
    lib = grass.load_library()
    st = lib.grass_sjlt_noalloc(ctypes.c_void_p(fake.data_ptr()), 1024, 1 << 20, 1 << 20, ctypes.c_void_p(0), 0, 8192, 1,
                                0, 1, ctypes.c_void_p(fake.data_ptr()), 8192, ctypes.c_void_p(0))
    assert st == grass.GRASS_ETOOLARGE
    assert "scratch" in grass.strerror(st)
    # a large fused batch runs in one chunk: no scratch memory, same result as the workspace entry point bit for bit
    n, p, kp, k = 512, 300000, 65536, 4096
    g = synth.bernoulli_sparse_normal(n, p, 0.5, 1.0, seed=4104, device=_dev())
    idx = grass.grass_mask_indices(0, 0, p, kp, device=_dev())
    assert grass.grass_sjlt_workspace_bytes(n, p, kp, k, 1) == 0
    out = torch.empty((n, k), dtype=torch.float32, device=_dev())
    assert _raw_noalloc(grass, g, idx, k, 1, 0, 1, out) == grass.GRASS_OK
    want = grass.grass_sjlt(g, k, 1, 0, 1, idx=idx)
    torch.cuda.synchronize()
    rows = [0, 255, 511]
    ref = orc.grass(g[rows].cpu().numpy(), idx.cpu().numpy(), k, 1, 0, 1)
    assert orc.max_rel_err(out[rows].cpu().numpy(), ref) <= TOL
    assert orc.max_rel_err(out.cpu().numpy(), want.cpu().numpy().astype(np.float64)) <= TOL
