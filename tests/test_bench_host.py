"""Host-side checks of bench.py's contract: what it can be asked without a GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2 and "one GPU only" in r.stderr and r.stdout.strip() == ""


def test_algorithmic_bytes_and_flops_of_the_headline_shapes():
    import bench
    # cfg3: 32768 tokens x (4 x 1536 + 2 x 16) elements of 2 bytes, parameters and the final state once
    assert bench.scan_bytes(1, 32768, 1536, 16, 2) == 32768 * 12352 + 1536 * 16 * 4 + 2 * 1536 * 4 + 1536 * 16 * 4
    assert bench.scan_bytes(1, 32768, 1536, 16, 2) == 404959232
    assert bench.scan_flops(1, 32768, 1536, 16) == 32768 * 1536 * 127 == 6392119296
    # 64 branches x 4096 channels: state read and written in fp32, token operands in bf16
    assert bench.step_bytes(64, 4096, 16, 2) == 64 * (2 * 4096 * 16 * 4 + (4 * 4096 + 32) * 2) + 4096 * 16 * 4 + 2 * 4096 * 4
    assert bench.step_bytes(64, 4096, 16, 2) == 35950592
    assert bench.conv_bytes(1, 32768, 1536, 4, 2) == 32768 * 2 * 1536 * 2 + 1536 * 4 * 4 + 1536 * 4 + 1536 * 3 * 2


def test_traffic_table_is_read_from_the_committed_profile():
    import bench
    text = open(bench.SCAN_TRAFFIC_TABLE).read()
    assert os.path.abspath(bench.SCAN_TRAFFIC_TABLE) == os.path.join(ROOT, "profiles", "scan_hbm_traffic.md")
    for name in ("cfg1", "cfg3", "cfg4"):
        got = bench.scan_traffic_bytes(name)
        row = [l for l in text.splitlines() if l.startswith("| %s |" % name)]
        assert len(row) == 1
        cells = [c.strip() for c in row[0].strip().strip("|").split("|")]
        assert got == round(float(cells[3]) * 1e6)
        assert abs(float(cells[1]) + float(cells[2]) - float(cells[3])) < 0.02     # fetched + written = total
        # measured traffic is never below what the operator has to move
        shape = {"cfg1": (1, 2048, 1536), "cfg3": (1, 32768, 1536), "cfg4": (8, 8192, 4096)}[name]
        assert got >= 0.99 * bench.scan_bytes(*shape, 16, 2)
    assert bench.scan_traffic_bytes("cfg0") is None and bench.scan_traffic_bytes("no such config") is None
