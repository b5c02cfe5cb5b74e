"""bench.py's host-side helpers: the traffic figure comes from the tracked table only when workload, seed and
the digest of the dominant kernel's sources all match; the single-GPU contract of the command line."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import bench


def test_traffic_table_lookup_is_keyed_by_workload_seed_and_source_digest(tmp_path, monkeypatch):
    digest = bench.kernel_sources_digest()
    assert len(digest) == 12 and int(digest, 16) >= 0
    table = tmp_path / "t.md"
    table.write_text("# x\n| config | seed | kernel sources | FETCH_SIZE | factor | WRITE_SIZE | factor |\n|---|---|---|---|---|---|---|\n"
                     "| 3 | 0 | %s | 1000 | 2.0 | 500 | 1.0 |\n| 3 | 1 | 000000000000 | 7 | 2.0 | 7 | 1.0 |\n" % digest)
    monkeypatch.setattr(bench, "TRAFFIC_TABLE", str(table))
    assert bench.measured_traffic_bytes(3, 0) == (1000 * 2 + 500) * 1024
    assert bench.measured_traffic_bytes(3, 1) is None        # another build's row
    assert bench.measured_traffic_bytes(4, 0) is None        # no row for this workload
    monkeypatch.setattr(bench, "TRAFFIC_TABLE", str(tmp_path / "missing.md"))
    assert bench.measured_traffic_bytes(3, 0) is None


def test_committed_table_parses():
    rows = [l for l in open(bench.TRAFFIC_TABLE) if l.startswith("| 3 |")]
    assert rows, "the table carries a row for the benchmark workload"
    cells = [c.strip() for c in rows[0].strip().strip("|").split("|")]
    assert len(cells) == 7 and float(cells[3]) > 0 and float(cells[5]) > 0


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], stdout=subprocess.PIPE,
                       stderr=subprocess.PIPE, text=True, timeout=120)
    assert r.returncode == 2 and "ONE GPU" in r.stderr


def test_the_traffic_table_has_a_row_for_the_kernel_sources_as_they_stand():
    """roofline.traffic of the default bench line comes from counter runs on a particular build of the dominant
    kernel; a change to its sources without new counter runs would silently turn the figure into null."""
    import bench
    assert bench.measured_traffic_bytes(3, 0) is not None, (
        "profiles/hbm_traffic_table.md has no row for workload 3, seed 0 and kernel sources digest %s: "
        "run the FETCH_SIZE and WRITE_SIZE counter passes again and add the row" % bench.kernel_sources_digest())
