"""The stored worked examples of tests/golden/oracle_snapshots.txt (written by the committed script beside it, which
calls only the oracle): the oracle still reproduces them, and the GPU library reproduces them through the C ABI."""
import importlib.util
import os
import re

import numpy as np
import pytest
import torch

from oracle import grass_oracle as orc

HERE = os.path.dirname(os.path.abspath(__file__))


def _script():
    spec = importlib.util.spec_from_file_location("make_oracle_snapshots",
                                                  os.path.join(HERE, "golden", "make_oracle_snapshots.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def _args(name):
    """The key=value integers of a case name."""
    return {k: int(v) for k, v in re.findall(r"(\w+)=(\d+)", name)}


def _stored():
    out, name = {}, None
    for line in open(os.path.join(HERE, "golden", "oracle_snapshots.txt")):
        line = line.rstrip("\n")
        if line.startswith("#") or not line:
            continue
        if line.startswith("@ "):
            name = line[2:]
        else:
            out[name] = np.array([float(t) for t in line.split()])
    return out


def test_oracle_reproduces_the_stored_examples():
    stored = _stored()
    cases = _script().cases()
    assert len(cases) == len(stored) == 12
    for name, v in cases:
        v = np.asarray(v, dtype=np.float64)
        if "gauss" in name:
            assert np.allclose(v, stored[name], rtol=1e-11, atol=0), name      # written to 12 digits
        else:
            assert np.array_equal(v, stored[name]), name


def test_stored_examples_have_the_structure_the_readings_promise():
    """Independent of the oracle: facts that can be read off the stored numbers themselves."""
    st = _stored()
    for name, v in st.items():
        if name.startswith("mask_indices"):
            assert np.all(np.diff(v) > 0) and v[0] >= 0 and v[-1] < _args(name)["p"], name
        if name.startswith("sjlt_bucket"):
            k, s = _args(name)["k"], _args(name)["s"]
            b = v.reshape(-1, s)
            for r in range(s):                                   # non-zero r of a column lies in block r of k/s rows
                assert np.all((b[:, r] >= r * k // s) & (b[:, r] < (r + 1) * k // s)), name
        if name.startswith("sjlt_sign"):
            assert set(np.unique(v)) <= {-1.0, 1.0}, name
    # SJLT with s = 1 moves every input entry into exactly one bucket with a sign: the sum of squares of the output
    # can only differ from that of the input through collisions, and the plain sum of |.| never grows
    g = _script().small_ints(3, 40, 9, 4)
    out = st["sjlt seed=0 stream=1 n=3 d=40 k=8 s=1"].reshape(3, 8)
    assert np.all(np.abs(out).sum(axis=1) <= np.abs(g).sum(axis=1))
    # ... and with the stored table of the same seed and stream (first 12 positions) the first 12 entries of row 0
    # account for the stored output exactly when the rest of the row is removed
    b = st["sjlt_bucket seed=0 stream=1 d=12 k=8 s=1"].astype(int)
    sg = st["sjlt_sign seed=0 stream=1 d=12 k=8 s=1"]
    head = np.zeros(8)
    np.add.at(head, b, sg * g[0, :12])
    tail = np.zeros((1, 40)); tail[0, 12:] = g[0, 12:]
    assert np.array_equal(head + orc.sjlt(tail, 8, 1, 0, 1)[0], out[0])


@pytest.mark.gpu
def test_gpu_library_reproduces_the_stored_examples():
    import paper_2505_18976_amd as grass
    grass.load_library()
    dev = torch.device("cuda:0")
    st = _stored()
    mk = _script()
    for name, v in st.items():
        if name.startswith("mask_indices"):
            a = _args(name)
            got = grass.grass_mask_indices(a["seed"], a["stream"], a["p"], a["kprime"], device=dev)
            assert np.array_equal(got.cpu().numpy(), v.astype(np.int32)), name
        if name.startswith("sjlt_bucket"):
            a = _args(name)
            b, sg = grass.grass_sjlt_tables(a["seed"], a["stream"], a["d"], a["k"], a["s"], device=dev)
            assert np.array_equal(b.cpu().numpy().reshape(-1), v.astype(np.int32)), name
            assert np.array_equal(sg.cpu().numpy().reshape(-1), st[name.replace("sjlt_bucket", "sjlt_sign")].astype(np.int8))
    g = torch.from_numpy(mk.small_ints(3, 40, 9, 4)).to(torch.float32).to(dev)
    out = grass.grass_sjlt(g, 8, 1, seed=0, stream_id=1)
    assert np.array_equal(out.cpu().numpy().reshape(-1), st["sjlt seed=0 stream=1 n=3 d=40 k=8 s=1"])   # small integers: exact
    out = grass.grass_sjlt(g, 16, 4, seed=2, stream_id=1)
    assert np.array_equal(out.cpu().numpy().reshape(-1), st["sjlt seed=2 stream=1 n=3 d=40 k=16 s=4"])
    out = grass.grass_sjlt_bf16(g.to(torch.bfloat16), 8, 1, seed=0, stream_id=1)
    assert np.array_equal(out.cpu().numpy().reshape(-1), st["sjlt seed=0 stream=1 n=3 d=40 k=8 s=1"])
    idx = grass.grass_mask_indices(1, 0, 40, 10, device=dev)
    out = grass.grass_sjlt(g, 4, 1, seed=1, stream_id=1, idx=idx)
    assert np.array_equal(out.cpu().numpy().reshape(-1),
                          st["grass seed=1 n=3 p=40 kprime=10 k=4 s=1 (mask seed 1 stream 0, sjlt stream 1)"])
    x = torch.from_numpy(mk.small_ints(6, 10, 5, 2).reshape(2, 3, 10)).to(torch.bfloat16).to(dev)
    go = torch.from_numpy(mk.small_ints(6, 6, 7, 3).reshape(2, 3, 6)).to(torch.bfloat16).to(dev)
    s_in, s_out, s_sj = orc.layer_streams(0)
    ii = grass.grass_mask_indices(4, s_in, 10, 4, device=dev)
    io = grass.grass_mask_indices(4, s_out, 6, 3, device=dev)
    out = grass.factgrass_linear(x, go, ii, io, 6, 1, 4, s_sj)
    assert np.array_equal(out.cpu().numpy().reshape(-1),
                          st["factgrass seed=4 layer=0 n=2 T=3 d_in=10 d_out=6 kin=4 kout=3 k=6 s=1"])
    P = grass.grass_gauss_matrix(0, 1, 5, 4, 0, 5, device=dev)
    want = st["gauss_matrix seed=0 stream=1 p=5 k=4 (row-major 4 x 5, 12 significant digits)"]
    assert np.abs(P.cpu().numpy().reshape(-1) - want).max() <= 4e-6      # fp32 log, cos and sqrt against fp64
    torch.cuda.synchronize()
