"""Host logic of the tool that turns rocprofv3 CSV files into the summaries under profiles/:
the scaling of the FETCH_SIZE / WRITE_SIZE counters by a copy of known size, the per-kernel
averages, and the line format bench.py reads the dominant kernel's traffic from.  Synthetic CSV
rows in the column layout rocprofv3 writes (kernel statistics and counter collection)."""
import csv
import io
import contextlib

from paper_2505_03254_amd import rocprof_summary as R

COPY = "prom::copy_kernel(int __vector(4) const*, int __vector(4)*, long long)"
BIG = "void prom::pw_bigbatch_kernel<0>(prom::PwBatchArgs)"
OTHER = "void at::native::vectorized_elementwise_kernel<4>(int)"


def _write(path, header, rows):
    with open(path, "w", newline="") as f:
        w = csv.writer(f)
        w.writerow(header)
        w.writerows(rows)


def _run(argv):
    out = io.StringIO()
    with contextlib.redirect_stdout(out):
        assert R.main(argv) == 0
    return out.getvalue()


def test_traffic_is_scaled_by_the_copy_kernel(tmp_path):
    copy_bytes = 1 << 20
    hdr = ["Dispatch_Id", "Kernel_Name", "Counter_Name", "Counter_Value"]
    # the copy reads 1 MiB: FETCH_SIZE reports half of it in KiB (so the factor is 2), WRITE_SIZE all of it
    fetch = [(1, COPY, "FETCH_SIZE", 512), (2, COPY, "FETCH_SIZE", 512),
             (3, BIG, "FETCH_SIZE", 1000), (4, BIG, "FETCH_SIZE", 3000), (5, OTHER, "FETCH_SIZE", 777),
             (6, BIG, "SOMETHING_ELSE", 5)]
    write = [(1, COPY, "WRITE_SIZE", 1024), (2, COPY, "WRITE_SIZE", 1024),
             (3, BIG, "WRITE_SIZE", 500), (4, BIG, "WRITE_SIZE", 700), (5, OTHER, "WRITE_SIZE", 9)]
    _write(tmp_path / "f.csv", hdr, fetch)
    _write(tmp_path / "w.csv", hdr, write)
    text = _run(["traffic", str(tmp_path / "f.csv"), str(tmp_path / "w.csv"), "--copy-bytes", str(copy_bytes)])
    assert "FETCH_SIZE x 2.0000" in text and "WRITE_SIZE x 1.0000" in text
    assert "vectorized_elementwise" not in text            # only this library's kernels
    # reads: mean(1000, 3000) KiB x 2 = 4000 KiB; writes: mean(500, 700) KiB = 600 KiB
    want = int(4000 * 1024 + 600 * 1024)
    assert f"traffic_bytes_per_launch[{BIG}] = {want}" in text
    assert "traffic_bytes_per_launch[prom::copy_kernel" not in text
    # the line is what bench.py looks for
    line = next(l for l in text.splitlines() if l.startswith("traffic_bytes_per_launch[") and f"[{BIG}]" in l)
    assert int(line.rsplit("=", 1)[1]) == want


def test_stats_lists_only_library_kernels(tmp_path):
    hdr = ["Name", "Calls", "TotalDurationNs", "AverageNs", "Percentage", "MinNs", "MaxNs", "StdDev"]
    rows = [(BIG, 55, 6325000, 115000.0, 9.5, 101000, 122000, 1.0),
            (OTHER, 10, 1000, 100.0, 0.1, 90, 110, 1.0)]
    _write(tmp_path / "s.csv", hdr, rows)
    text = _run(["stats", str(tmp_path / "s.csv")])
    lines = [l for l in text.splitlines() if l.strip()]
    assert len(lines) == 2 and lines[0].split()[0] == "kernel"
    cols = lines[1].split()
    assert cols[-5:] == ["55", "115.00", "101.00", "122.00", "9.50"]


def test_counters_average_per_launch_and_match(tmp_path):
    hdr = ["Dispatch_Id", "Kernel_Name", "Counter_Name", "Counter_Value"]
    _write(tmp_path / "a.csv", hdr, [(1, BIG, "TA_BUSY_avr", 100), (2, BIG, "TA_BUSY_avr", 300),
                                    (3, COPY, "TA_BUSY_avr", 50), (4, OTHER, "TA_BUSY_avr", 1)])
    _write(tmp_path / "b.csv", hdr, [(1, BIG, "SQ_WAVES", 3072), (2, BIG, "SQ_WAVES", 3072)])
    text = _run(["counters", str(tmp_path / "a.csv"), str(tmp_path / "b.csv"), "--match", "batch"])
    assert "copy_kernel" not in text and "vectorized" not in text
    assert text.splitlines()[0] == BIG
    body = {l.split()[0]: l.split()[1] for l in text.splitlines()[1:]}
    assert body == {"TA_BUSY_avr": "200", "SQ_WAVES": "3072"}
    assert "(launches: 2)" in text
