"""Host-only checks of bench.py's contract: what it refuses, and that the HBM traffic it reports
really is read from the committed rocprofv3 summaries."""
import os
import re
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_traffic_comes_from_the_committed_profiles():
    sys.path.insert(0, ROOT)
    import bench
    for row, name in bench.PROFILE_OF_ROW.items():
        path = os.path.join(ROOT, "profiles", name)
        assert os.path.exists(path), (row, name)
        traffic, source = bench.measured_traffic(row)
        assert source == "profiles/" + name
        text = open(path).read()
        algo = float(re.search(r"algorithmic bytes per launch \| ([0-9.e+]+)", text).group(1))
        # the counters can only see at least what the method must move (within counter granularity)
        assert traffic is not None and 0.97 * algo <= traffic <= 12 * algo, (row, traffic, algo)
        # every summary names the command that produced it, and that command runs committed files only
        assert "rocprofv3" in text and "bench.py" in text and "_work" not in text
    assert bench.measured_traffic("no_such_row") == (None, None)


def test_row_sets_are_consistent():
    sys.path.insert(0, ROOT)
    import bench
    assert bench.CORE[0] == "gemm_f64"                      # the headline row comes first
    assert not set(bench.CORE) & set(bench.EXTRA)
    summa = {f"gemm_f64_summa_chunk{k}" for k in (128, 256, 512, 1024, 2048)}       # the rows of the "summa" set
    # (a profile may belong to one row of a set that is asked for by the set's name)
    assert set(bench.PROFILE_OF_ROW) <= set(bench.CORE) | set(bench.EXTRA) | {"mttkrp_mode1", "ttm_rank32_mode2"} | summa
