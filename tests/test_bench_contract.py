"""Host-side parts of bench.py's contract that need no GPU: the multi-GPU refusal, the source hashes, and that the
traffic figures of the roofline come from the committed counter summary and only while the kernel sources match."""
import json
import os
import subprocess
import sys

import bench

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "single-GPU" in r.stderr and r.stdout.strip() == ""


def test_source_hashes_are_printed_and_stable():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--source-hashes"], capture_output=True, text=True)
    assert r.returncode == 0
    h = json.loads(r.stdout)
    assert set(h) == set(bench.KERNEL_SOURCES) and all(len(v) == 16 for v in h.values())
    assert h == {k: bench.source_sha16(k) for k in bench.KERNEL_SOURCES}


def test_traffic_comes_from_the_counter_summary_and_goes_stale_with_the_sources(tmp_path, monkeypatch):
    # the committed rows belong to the committed sources
    for workload in ("C4", "C3"):
        for kernel in bench.KERNEL_SOURCES:
            t = bench.measured_traffic(workload, kernel)
            assert t is not None and 1e7 < t < 1e10, (workload, kernel, t)
    assert bench.measured_traffic("C5", "bwd_col") is None        # no such row
    assert bench.measured_traffic("C4", "no_such_kernel") is None
    # a row whose hash differs from the sources' is not used
    with open(bench.TRAFFIC_PROFILE) as fh:
        text = fh.read()
    stale = tmp_path / "counters.md"
    stale.write_text(text.replace(bench.source_sha16("bwd_col"), "0" * 16))
    monkeypatch.setattr(bench, "TRAFFIC_PROFILE", str(stale))
    assert bench.measured_traffic("C4", "bwd_col") is None
    assert bench.measured_traffic("C4", "fwd") is not None
    # bytes = FETCH_SIZE KiB x 1024 x 2.0 + WRITE_SIZE KiB x 1024 x 1.0 of the row
    row = tmp_path / "one.md"
    row.write_text(f"| traffic | C9 | fwd | 1000.0 | 500.0 | {bench.source_sha16('fwd')} |\n")
    monkeypatch.setattr(bench, "TRAFFIC_PROFILE", str(row))
    assert bench.measured_traffic("C9", "fwd") == 1000.0 * 1024 * 2.0 + 500.0 * 1024 * 1.0
