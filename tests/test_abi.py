"""The C-ABI library loads and exports every symbol include/grass.h declares;
host-side argument checks answer without touching a GPU (CPU only)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "grass.h")


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"^(?:grass_status|const char\*|int|void)\s+(\w+)\s*\(", text, flags=re.M)
    return sorted(set(names))


@pytest.fixture(scope="module")
def lib():
    from paper_2505_18976_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    return binding.load_library()


def test_header_declares_the_four_entry_points():
    names = _declared_functions()
    for required in ("grass_mask", "grass_sjlt", "factgrass_linear", "grass_score"):
        assert required in names


def test_every_declared_symbol_is_exported_and_bound(lib):
    from paper_2505_18976_amd import binding
    declared = _declared_functions()
    assert declared == sorted(binding.SIGNATURES)
    for name in declared:
        assert getattr(lib, name) is not None


def test_version_and_strerror(lib):
    assert lib.grass_version() >= 100
    assert lib.grass_strerror(0) == b"ok"
    assert b"invalid" in lib.grass_strerror(1)
    assert b"unknown" in lib.grass_strerror(99)


def test_workspace_queries_validate_on_the_host(lib):
    from paper_2505_18976_amd import binding as b
    out = ctypes.c_size_t(123)
    assert lib.grass_sjlt_workspace_bytes(16, 1000, 0, 64, 1, None, ctypes.byref(out)) == b.GRASS_OK
    assert lib.grass_sjlt_workspace_bytes(16, 1000, 0, 0, 1, None, ctypes.byref(out)) == b.GRASS_EINVAL      # k = 0
    assert lib.grass_sjlt_workspace_bytes(16, 1000, 0, 64, 0, None, ctypes.byref(out)) == b.GRASS_EINVAL     # s = 0
    assert lib.grass_sjlt_workspace_bytes(16, 1000, 0, 64, 3, None, ctypes.byref(out)) == b.GRASS_EINVAL     # s does not divide k
    assert lib.grass_sjlt_workspace_bytes(16, 1000, 2000, 64, 1, None, ctypes.byref(out)) == b.GRASS_EINVAL  # k' > p
    assert lib.grass_sjlt_workspace_bytes(16, 1000, 0, 1 << 20, 1, None, ctypes.byref(out)) == b.GRASS_EUNSUPPORTED
    assert lib.grass_sjlt_workspace_bytes(16, 1000, 0, 64, 1, None, None) == b.GRASS_EINVAL
    assert lib.grass_mask_indices_workspace_bytes(1000, 10, ctypes.byref(out)) == b.GRASS_OK
    assert out.value > 4 * 65536 * 4
    assert lib.grass_mask_indices_workspace_bytes(1000, 1001, ctypes.byref(out)) == b.GRASS_EINVAL
    assert lib.grass_mask_indices_workspace_bytes(1 << 31, 10, ctypes.byref(out)) == b.GRASS_EINVAL
    assert lib.factgrass_linear_workspace_bytes(8, 128, 64, 64, 1024, 1, None, ctypes.byref(out)) == b.GRASS_OK
    assert lib.factgrass_linear_workspace_bytes(8, 128, 64, 129, 1024, 1, None, ctypes.byref(out)) == b.GRASS_EUNSUPPORTED
    assert lib.factgrass_linear_workspace_bytes(8, 0, 64, 64, 1024, 1, None, ctypes.byref(out)) == b.GRASS_EINVAL


def test_bad_arguments_are_rejected_before_any_launch(lib):
    """These calls must return on the host: this process has no GPU."""
    from paper_2505_18976_amd import binding as b
    null = ctypes.c_void_p(0)
    fake = ctypes.c_void_p(4096)
    # null pointers
    assert lib.grass_sjlt(null, 4, 100, 100, null, 0, 16, 1, 0, 1, fake, 16, null, 0, None, null) == b.GRASS_EINVAL
    # leading dimension smaller than the row
    assert lib.grass_sjlt(fake, 4, 100, 99, null, 0, 16, 1, 0, 1, fake, 16, null, 0, None, null) == b.GRASS_EINVAL
    assert lib.grass_sjlt(fake, 4, 100, 100, null, 0, 16, 1, 0, 1, fake, 15, null, 0, None, null) == b.GRASS_EINVAL
    # n = 0 is a no-op
    assert lib.grass_sjlt(fake, 0, 100, 100, null, 0, 16, 1, 0, 1, fake, 16, null, 0, None, null) == b.GRASS_OK
    assert lib.grass_mask(fake, 0, 100, 100, fake, 10, fake, 10, null) == b.GRASS_OK
    assert lib.grass_mask(fake, 4, 100, 100, fake, 101, fake, 101, null) == b.GRASS_EINVAL
    assert lib.grass_mask(fake, 4, 100, 100, null, 10, fake, 10, null) == b.GRASS_EINVAL
    # workspace required but missing: many chunks for a single long row
    assert lib.grass_sjlt(fake, 1, 1 << 22, 1 << 22, null, 0, 16, 1, 0, 1, fake, 16, null, 0, None, null) == b.GRASS_EWORKSPACE
    assert lib.grass_mask_indices(0, 0, 1000, 10, fake, null, 0, null) == b.GRASS_EWORKSPACE
    assert lib.grass_score(fake, fake, 2, 8, 8, 8, 8, 8, fake, 8, null, 0, null) == b.GRASS_EINVAL
    assert lib.grass_score(fake, fake, 0, 8, 8, 8, 7, 8, fake, 8, null, 0, null) == b.GRASS_EINVAL
    assert lib.factgrass_linear(fake, fake, 2, 16, 64, 64, fake, 65, fake, 8, 32, 1, 0, 18, fake, 32, null, 0,
                                None, null) == b.GRASS_EINVAL                                                  # k_in' > d_in
    assert lib.grass_gauss_project(fake, 2, 64, 64, 8, 0, 2, 0, 0, fake, 8, null, 0, null) == b.GRASS_EWORKSPACE


def test_logra_refuses_feature_dimensions_beyond_its_offset_range(lib):
    """logra_linear addresses a tile of 64 rows with 32-bit byte offsets: d_in, d_out above 2^24 are refused on the host."""
    from paper_2505_18976_amd import binding as b
    fake, null = ctypes.c_void_p(4096), ctypes.c_void_p(0)
    big = (1 << 24) + 8
    assert lib.logra_linear(fake, fake, 2, 64, big, 64, fake, 8, fake, 8, fake, 64, fake, 1 << 20, null) == b.GRASS_EUNSUPPORTED
    assert lib.logra_linear(fake, fake, 2, 64, 64, big, fake, 8, fake, 8, fake, 64, fake, 1 << 20, null) == b.GRASS_EUNSUPPORTED
    assert lib.logra_linear(fake, fake, 2, 64, 60, 64, fake, 8, fake, 8, fake, 64, fake, 1 << 20, null) == b.GRASS_EUNSUPPORTED  # d % 8


def test_probe_checks_its_buffers_on_the_host(lib):
    from paper_2505_18976_amd import binding as b
    fake, null = ctypes.c_void_p(4096), ctypes.c_void_p(0)
    assert lib.grass_probe_line_reads(null, 1 << 20, fake, 1, 0, 0, 8, null) == b.GRASS_EINVAL
    assert lib.grass_probe_line_reads(fake, 1 << 20, fake, 100, 1, 0, 8, null) == b.GRASS_EINVAL      # 8*256*16 floats needed
    assert lib.grass_probe_line_reads(fake, 1 << 20, fake, 1, 7, 0, 8, null) == b.GRASS_EINVAL        # no such mode
    assert lib.grass_probe_line_reads(ctypes.c_void_p(4100), 1 << 20, fake, 1, 0, 0, 8, null) == b.GRASS_EUNSUPPORTED


def test_noalloc_entry_point_refuses_oversized_problems_on_the_host(lib):
    """grass_sjlt_noalloc keeps its scratch memory in a fixed 32 MiB buffer inside the library: a problem whose
    partial sums need more is refused before anything touches a GPU (this process has none)."""
    from paper_2505_18976_amd import binding as b
    fake, null = ctypes.c_void_p(4096), ctypes.c_void_p(0)
    # 2 column chunks x 1,024 rows x 8,192 buckets x 4 bytes = 64 MiB
    assert lib.grass_sjlt_noalloc(fake, 1024, 1 << 20, 1 << 20, null, 0, 8192, 1, 0, 1, fake, 8192, null) == b.GRASS_ETOOLARGE
    assert b"scratch" in lib.grass_strerror(b.GRASS_ETOOLARGE)
    assert lib.grass_sjlt_noalloc(null, 4, 100, 100, null, 0, 16, 1, 0, 1, fake, 16, null) == b.GRASS_EINVAL
    assert lib.grass_sjlt_noalloc(fake, 0, 100, 100, null, 0, 16, 1, 0, 1, fake, 16, null) == b.GRASS_OK     # n = 0
    assert lib.grass_sjlt_noalloc(fake, 4, 100, 100, null, 0, 16, 3, 0, 1, fake, 16, null) == b.GRASS_EINVAL  # s does not divide k


def test_tuning_is_a_per_call_argument(lib):
    """Launch-shape overrides travel with the call: the same query with and without them, interleaved, keeps
    answering the same (there is no process-wide setting to leak from one call into the next)."""
    from paper_2505_18976_amd import binding as b
    plain, tuned = ctypes.c_size_t(0), ctypes.c_size_t(0)
    t = b.GrassTuning(sjlt_rows_per_block=1, sjlt_column_chunks=7, sjlt_threads=256, sjlt_accumulator=2)
    for _ in range(2):
        assert lib.grass_sjlt_workspace_bytes(64, 40000, 0, 1024, 1, None, ctypes.byref(plain)) == b.GRASS_OK
        assert lib.grass_sjlt_workspace_bytes(64, 40000, 0, 1024, 1, ctypes.byref(t), ctypes.byref(tuned)) == b.GRASS_OK
        assert tuned.value == 7 * 64 * 1024 * 4 and plain.value != tuned.value
    ft = b.GrassTuning(factgrass_tokens_per_block=64)
    for _ in range(2):
        assert lib.factgrass_linear_workspace_bytes(4, 256, 64, 64, 512, 1, None, ctypes.byref(plain)) == b.GRASS_OK
        assert lib.factgrass_linear_workspace_bytes(4, 256, 64, 64, 512, 1, ctypes.byref(ft), ctypes.byref(tuned)) == b.GRASS_OK
        assert tuned.value == 4 * 4 * 512 * 4 and plain.value != tuned.value
    # a missing workspace is reported for the tuned plan, before any launch
    fake, null = ctypes.c_void_p(4096), ctypes.c_void_p(0)
    assert lib.grass_sjlt(fake, 64, 40000, 40000, null, 0, 1024, 1, 0, 1, fake, 1024, null, 0, ctypes.byref(t),
                          null) == b.GRASS_EWORKSPACE


def test_binding_refuses_to_run_without_the_library(monkeypatch, tmp_path):
    from paper_2505_18976_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "missing.so"))
    with pytest.raises(ImportError):
        binding.load_library()
