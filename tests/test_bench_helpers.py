"""bench.py's host-side helpers (no GPU): the traffic table that roofline.traffic is read from."""
import bench


def test_traffic_table_rows_are_found_and_scaled(tmp_path, monkeypatch):
    table = tmp_path / "t.md"
    table.write_text(
        "# title\n\n"
        "| workload | nprobe | kernel | FETCH_SIZE KiB | factor | WRITE_SIZE KiB | factor | dispatches |\n"
        "|---|---|---|---|---|---|---|---|\n"
        "| sift1m | 23 | scan_mfma_kernel | 1,000 | 2.000 | 500 | 1.000 | 11 |\n"
        "| gist1m | 45 | scan_mfma_lds_kernel | 10 | 2.5 | 4 | 1.0 | 3 |\n")
    monkeypatch.setattr(bench, "TRAFFIC_TABLE", str(table))
    assert bench.measured_traffic("sift1m", 23, "scan_mfma_kernel") == (1000 * 2.0 + 500 * 1.0) * 1024
    assert bench.measured_traffic("gist1m", 45, "scan_mfma_lds_kernel") == (10 * 2.5 + 4) * 1024
    # no row for another nprobe, another kernel or another workload: null, never a guess
    assert bench.measured_traffic("sift1m", 24, "scan_mfma_kernel") is None
    assert bench.measured_traffic("sift1m", 23, "scan_exact_kernel") is None
    assert bench.measured_traffic("sphere10m", 23, "scan_mfma_kernel") is None


def test_traffic_table_missing_file_is_null(monkeypatch, tmp_path):
    monkeypatch.setattr(bench, "TRAFFIC_TABLE", str(tmp_path / "absent.md"))
    assert bench.measured_traffic("sift1m", 23, "scan_mfma_kernel") is None


def test_tracked_traffic_table_has_the_headline_row():
    got = bench.measured_traffic("sift1m", 23, "scan_mfma_kernel")
    assert got is not None and 0.5e9 < got < 5e9
