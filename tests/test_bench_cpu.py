"""Host-side checks of bench.py and the profile summaries (no GPU): the figures the benchmark
line is built from, and that the recorded counter summaries belong to the sources in the tree."""
import glob
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import bench  # noqa: E402
from paper_1907_02818_amd.profile_summary import library_sources_sha256  # noqa: E402


def test_algorithmic_bytes_of_the_headline_workload():
    # read c and r_bar on the 504^3 interior, read and write u_bar on the 512^3 grid, 8 bytes each
    assert bench.wave_adjoint_bytes((512, 512, 512), 4, 8) == 16 * 512 ** 3 + 16 * 504 ** 3 == 4195868672
    assert bench.wave_adjoint_bytes((512, 512, 512), 4, 8, True) == 16 * 512 ** 3 + 32 * 504 ** 3
    assert bench.wave_adjoint_bytes((8192, 8192), 1, 4) == 8 * 8192 ** 2 + 8 * 8190 ** 2
    assert bench.interior_points((10, 20, 30), 2) == 6 * 16 * 26


def test_more_than_one_gpu_is_refused_with_a_message():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert p.returncode != 0
    assert "one GPU" in p.stderr


def test_recorded_counter_summaries_belong_to_the_sources_in_the_tree():
    """bench.py reports roofline.traffic only from a summary that records the hash of the kernel
    sources it was taken from; the committed summaries must be current."""
    cur = library_sources_sha256()
    files = sorted(glob.glob(os.path.join(ROOT, "profiles", "*_pmc.txt")))
    assert files
    for f in files:
        sha = [ln.split()[-1] for ln in open(f) if ln.startswith("library_sources_sha256")]
        assert sha == [cur], os.path.basename(f)
    val, note = bench.read_traffic(bench.HEADLINE)
    assert val is not None and 4.19e9 < val < 5e9, note
