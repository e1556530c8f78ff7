"""The measurement aid grass_probe_line_reads: it must run and stay inside its buffers (the traffic figures it is for
are taken by bench.py --probe)."""
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def grass():
    import paper_2505_18976_amd as g
    g.load_library()
    return g


def test_probe_runs_in_every_mode_and_writes_only_what_it_owns(grass):
    dev = torch.device("cuda:0")
    blocks = 8
    src = torch.zeros(1 << 20, dtype=torch.float32, device=dev)
    guard = 64
    dst = torch.full((blocks * 256 * 16 + guard,), -3.0, dtype=torch.float32, device=dev)
    for mode in (0, 2, 3):
        grass.grass_probe_line_reads(src, dst[:1], mode, 5, blocks)
    torch.cuda.synchronize()
    assert bool((dst == -3.0).all())                       # read-only modes leave dst alone (src holds zeros)
    grass.grass_probe_line_reads(src, dst[:blocks * 256 * 16], 1, 5, blocks)
    torch.cuda.synchronize()
    assert bool((dst[:blocks * 256 * 16] == 0.0).all()) and bool((dst[blocks * 256 * 16:] == -3.0).all())
    with pytest.raises(grass.GrassError):                  # destination too small for the write stream
        grass.grass_probe_line_reads(src, dst[:100], 1, 5, blocks)
    with pytest.raises(grass.GrassError):
        grass.grass_probe_line_reads(src, dst, 4, 5, blocks)
