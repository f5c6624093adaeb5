"""bench.py quotes two measured figures of its headline kernel as constants (HBM traffic per launch,
matrix-core busy fraction); they must be the ones in the committed profile summary they cite."""
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_constants_are_the_figures_of_the_profile_summary():
    import bench
    text = open(os.path.join(ROOT, bench.PROFILE_FILE)).read()
    m = re.search(r"total ([0-9.]+) MB = [0-9.]+ x the algorithmic ([0-9.]+) MB", text)
    assert m, "the summary no longer states the total traffic per launch"
    assert abs(float(m.group(1)) * 1e6 - bench.MEASURED_TRAFFIC_BYTES) < 0.05e6
    algo = 4 * 49 * 32 * 2 * 8192 * 3
    assert abs(float(m.group(2)) * 1e6 - algo) < 0.05e6
    m = re.search(r"MFMA busy fraction = [^\n]*?= ([0-9.]+) %", text)
    assert m, "the summary no longer states the matrix-core busy fraction"
    assert abs(float(m.group(1)) / 100 - bench.MEASURED_MFMA_BUSY_FRAC) < 5e-4
    # the kernel the constants belong to is the one the bench line names
    src = open(os.path.join(ROOT, "bench.py")).read()
    assert "fwd_bf16_staged_kernel<4,false,1>" in src and "fwd_bf16_staged_kernel<4,false,1>" in text
