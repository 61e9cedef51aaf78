"""Host-side checks of bench.py's contract that need no GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_the_measured_traffic_table_matches_the_committed_profiles():
    """The HBM-side decode traffic bench.py reports is the figure of the committed rocprofv3 summaries."""
    sys.path.insert(0, ROOT)
    import bench
    files = {1: "all_kernels_cfg1_7b_m2944.md", 2: "all_kernels_cfg2_7b_b4_m10368.md"}
    for cid, name in files.items():
        rows = [l for l in open(os.path.join(ROOT, "profiles", name)) if l.startswith("| decode_kernel") and l.count("|") == 5]
        big = max(rows, key=lambda l: float(l.split("|")[3]))               # the all-layer launch reads the most
        read_mib, written_mib = float(big.split("|")[3]), float(big.split("|")[4])
        assert abs(bench.MEASURED_DECODE_TRAFFIC_MIB[cid] - (read_mib + written_mib)) < 0.02 * (read_mib + written_mib)
