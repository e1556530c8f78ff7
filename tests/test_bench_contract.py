"""Host-side pieces of bench.py (CPU only): the multi-GPU refusal, the touched-line count behind the roofline objects
and the parsing of the counter record in the profile summary."""
import importlib.util
import os
import subprocess
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bench():
    spec = importlib.util.spec_from_file_location("bench_module", os.path.join(ROOT, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in r.stderr and r.stdout.strip() == ""


def test_touched_lines_against_brute_force():
    b = _bench()
    rng = np.random.default_rng(0)
    for (p, kp, elem, base, rows) in [(1000, 100, 4, 24, 37), (4096, 64, 2, 0, 5), (1863690, 5000, 4, 40, 50), (77, 77, 4, 4, 9)]:
        idx = np.sort(rng.choice(p, kp, replace=False)).astype(np.int32)
        row_bytes = p * elem
        want = sum(np.unique((base + r * row_bytes + idx.astype(np.int64) * elem) // 128).size for r in range(rows))
        assert b._touched_lines(idx, elem, row_bytes, base, rows) == want
    # every element kept: all lines of the rows
    idx = np.arange(64, dtype=np.int32)
    assert b._touched_lines(idx, 2, 128, 0, 10) == 10


def test_traffic_record_of_the_committed_profile(tmp_path):
    b = _bench()
    rec = b._traffic_record(b.TRAFFIC_PROFILE)
    assert rec is not None, "profiles/sjlt_fused_mlp_pmc.txt must end in a traffic_record line"
    assert rec["kernel"].startswith("sjlt_kernel<float,") and rec["n"] == "4096" and rec["p"] == "1863690"
    assert rec["kprime"] == "65536" and rec["k"] == "4096" and rec["s"] == "1"
    # 20.9 GB of touched lines is the floor; the counters may show a little more, never less, never twice as much
    assert 20.9e9 <= int(rec["bytes_per_launch"]) <= 23e9
    assert b._traffic_record(str(tmp_path / "missing.txt")) is None
    (tmp_path / "no_record.txt").write_text("summary without the line\n")
    assert b._traffic_record(str(tmp_path / "no_record.txt")) is None


def test_describe_names_the_kernel_the_profile_was_taken_on():
    """The library's own description of the headline launch (host only, nothing is launched) must be the kernel and grid
    of the counter record, or bench.py would report traffic null."""
    import paper_2505_18976_amd as grass
    b = _bench()
    rec = b._traffic_record(b.TRAFFIC_PROFILE)
    text = grass.grass_sjlt_describe(4096, 1863690, 1863690, 65536, 4096, 1)
    assert text.split()[0] == rec["kernel"] and text.split()[1] == "grid=" + rec["grid"]
    # other shapes give other instantiations: bf16 input, unmasked rows, a tuned launch
    assert grass.grass_sjlt_describe(4096, 1863690, 1863690, 65536, 4096, 1, bf16=True).split()[0] != rec["kernel"]
    assert "false" in grass.grass_sjlt_describe(1024, 11173962, 11173962, 0, 8192, 1).split()[0]
    tuned = grass.grass_sjlt_describe(4096, 1863690, 1863690, 65536, 4096, 1, tuning=dict(sjlt_rows_per_block=2))
    assert tuned.split()[0].startswith("sjlt_kernel<float,2,")
