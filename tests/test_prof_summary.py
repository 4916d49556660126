"""The profile summary tool on small hand-made rocprofv3 CSV files (CPU only)."""
import json

import prof_summary


def _write(path, header, rows):
    path.parent.mkdir(parents=True, exist_ok=True)
    path.write_text(",".join(header) + "\n" + "\n".join(",".join(str(v) for v in r) for r in rows) + "\n")


def test_traffic_scales_the_counters_by_the_calibration_copy(tmp_path, capsys):
    # FETCH_SIZE counts in units of 2 KiB here, WRITE_SIZE in KiB: a 1 MiB copy reads as 512 / 1024
    head = ["Kernel_Name", "Counter_Name", "Counter_Value"]
    _write(tmp_path / "f" / "x_counter_collection.csv", head,
           [("__amd_rocclr_copyBuffer", "FETCH_SIZE", 512), ("__amd_rocclr_copyBuffer", "FETCH_SIZE", 8),
            ("void mpq_gemv_kernel<2>(DevBlob)", "FETCH_SIZE", 100), ("void mpq_gemv_kernel<2>(DevBlob)", "FETCH_SIZE", 300),
            ("void other(int)", "FETCH_SIZE", 999), ("void mpq_gemv_kernel<2>(DevBlob)", "SQ_WAVES", 7)])
    _write(tmp_path / "w" / "x_counter_collection.csv", head,
           [("__amd_rocclr_copyBuffer", "WRITE_SIZE", 1024), ("void mpq_gemv_kernel<2>(DevBlob)", "WRITE_SIZE", 4)])
    prof_summary.traffic(str(tmp_path / "f"), str(tmp_path / "w"), float(1 << 20), "mpq_gemv_kernel")
    out = json.loads(capsys.readouterr().out)
    assert out["FETCH_SIZE"]["launches"] == 2 and out["FETCH_SIZE"]["scale"] == 2.0
    assert out["FETCH_SIZE"]["bytes_per_launch"] == 200 * 1024 * 2.0
    assert out["WRITE_SIZE"]["scale"] == 1.0 and out["WRITE_SIZE"]["bytes_per_launch"] == 4 * 1024
    assert out["hbm_bytes_per_launch"] == 200 * 2048 + 4096


def test_stats_groups_the_product_kernel_by_grid_size(tmp_path, capsys):
    _write(tmp_path / "x_kernel_stats.csv", ["Name", "Calls", "TotalDurationNs", "AverageNs", "Percentage", "MinNs", "MaxNs"],
           [("void mpq_gemv_kernel<2>(DevBlob)", 3, 24000, 8000.0, 99.0, 6000, 10000)])
    _write(tmp_path / "x_kernel_trace.csv", ["Kernel_Name", "Grid_Size_X", "Start_Timestamp", "End_Timestamp"],
           [("void mpq_gemv_kernel<2>(DevBlob)", 1024, 0, 6000), ("void mpq_gemv_kernel<2>(DevBlob)", 1024, 10, 8010),
            ("void mpq_gemv_kernel<2>(DevBlob)", 2048, 20, 10020), ("void other(int)", 64, 0, 5)])
    prof_summary.stats(str(tmp_path), "mpq_gemv_kernel")
    out = capsys.readouterr().out
    assert "grid 1024: 2, 7000, 8000, 6000" in out
    assert "grid 2048: 1, 10000, 10000, 10000" in out
    assert "all: 3 launches, average 8000 ns" in out
