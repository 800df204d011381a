"""Host logic of the tool that condenses rocprofv3 CSV output into the summaries under profiles/: tiny hand-made
CSV files in, the figures out.  No GPU, no profiler."""
import os

import paper_2605_16154_amd.profile_summary as ps


def _write(path, header, rows):
    os.makedirs(os.path.dirname(path), exist_ok=True)
    with open(path, "w") as f:
        f.write(",".join(header) + "\n")
        for r in rows:
            f.write(",".join(str(x) for x in r) + "\n")


def _counters(dirname, counter, rows):
    _write(os.path.join(dirname, "run", "x_counter_collection.csv"), ["Kernel_Name", "Counter_Name", "Counter_Value"],
           [(k, counter, v) for k, v in rows])


CAL = "elementwise<CUDAFunctorOnSelf_add<double>>"


def test_traffic_and_table_scale_by_the_calibration_kernel(tmp_path):
    fetch, write = str(tmp_path / "f"), str(tmp_path / "w")
    # the calibration kernel reads and writes 1 GiB: FETCH_SIZE reports half of it; it is also launched on one element
    _counters(fetch, "FETCH_SIZE", [(CAL, 524288.0), (CAL, 524288.0), (CAL, 0.25), ("pcm::gather_rows<x>", 1000.0),
                                    ("pcm::gather_rows<x>", 3000.0), ("pcm::gather_listed_rows(y)", 64.0)])
    _counters(write, "WRITE_SIZE", [(CAL, 1048576.0), (CAL, 1048576.0), (CAL, 0.5), ("pcm::gather_rows<x>", 4000.0),
                                    ("pcm::gather_listed_rows(y)", 32.0)])
    text = ps.traffic(fetch, write, "gather_rows")
    got = dict(line.split("=", 1) for line in text.strip().splitlines())
    assert got["launches_fetch"] == "2" and got["launches_write"] == "1"
    assert float(got["fetch_kib_per_launch"]) == 2000.0 and float(got["write_kib_per_launch"]) == 4000.0
    assert float(got["scale_fetch"]) == 2.0 and float(got["scale_write"]) == 1.0    # the one-element launch is left out
    assert got["source_hash"] == ps.kernel_source_hash() and len(got["source_hash"]) == 16
    rows = [l.split() for l in ps.table(fetch, write, ["gather_rows", "gather_listed_rows"]).splitlines()[2:]]
    assert rows[0][0] == "gather_rows" and int(rows[0][1]) == 2
    assert abs(float(rows[0][2]) - 2000.0 * 2.0 * 1024 / 1e6) < 1e-3 and abs(float(rows[0][3]) - 4000.0 * 1024 / 1e6) < 1e-3
    assert rows[1][0] == "gather_listed_rows" and abs(float(rows[1][2]) - 64.0 * 2.0 * 1024 / 1e6) < 1e-3


def test_stats_counter_and_tail(tmp_path):
    d = str(tmp_path / "s")
    _write(os.path.join(d, "run", "x_kernel_stats.csv"), ["Name", "Calls", "TotalDurationNs", "AverageNs"],
           [("void pcm::small(int)", 4, 4000, 1000), ("void pcm::big(int)", 2, 96000, 48000)])
    lines = ps.stats(d).splitlines()
    assert lines[1].startswith("pcm::big(int)") and "96.00%" in lines[1] and lines[-1].startswith("total kernel time: 0.100 ms")
    _write(os.path.join(d, "run", "x_kernel_trace.csv"), ["Kernel_Name", "Start_Timestamp", "End_Timestamp"],
           [("pcm::big(int)", 0, 1000), ("pcm::big(int)", 5000, 8000), ("pcm::big(int)", 9000, 14000), ("pcm::small(int)", 1, 2)])
    got = dict(line.split("=", 1) for line in ps.tail(d, "big", 2).strip().splitlines())
    assert got["launches"] == "3" and float(got["avg_us_all"]) == 3.0 and float(got["avg_us_last_n"]) == 4.0
    c = str(tmp_path / "c")
    _counters(c, "MfmaUtil", [("pcm::big(int)", 80.0), ("pcm::big(int)", 70.0)])
    assert "75" in ps.counter(c).splitlines()[1]
    assert ps.stats(str(tmp_path / "none")).startswith("no kernel_stats.csv")
