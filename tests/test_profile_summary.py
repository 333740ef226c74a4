"""profile_summary.py: rocprofv3 CSVs -> the text summaries kept under profiles/ and the
traffic table bench.py reads.  Synthetic CSVs in rocprofv3's column layout."""

import json

from paper_2001_00138_amd import profile_summary as ps

CONV = "void patdnn::tiled_conv_kernel<patdnn::Geo<16, 7, 1, 1, 16, false, 7, 0> >(patdnn::TiledArgs)"
COPY = "patdnn::copy_probe_kernel(HIP_vector_type<unsigned int, 4u> const*, HIP_vector_type<unsigned int, 4u>*, unsigned long)"


def _write_counters(path, rows):
    cols = ["Correlation_Id", "Dispatch_Id", "Kernel_Name", "Counter_Name", "Counter_Value"]
    with open(path, "w") as f:
        f.write(",".join(f'"{c}"' for c in cols) + "\n")
        for i, (k, c, v) in enumerate(rows):
            f.write(f'{i},{i},"{k}","{c}",{v}\n')


def test_counter_summary_scales_by_the_copy_kernel(tmp_path, capsys):
    fetch, write = tmp_path / "a_counter_collection.csv", tmp_path / "b_counter_collection.csv"
    # the copy kernel moved 1 MiB each way but the counters read 1100 / 1000 KiB
    _write_counters(fetch, [(COPY, "FETCH_SIZE", 1100.0), (CONV, "FETCH_SIZE", 2200.0), (CONV, "FETCH_SIZE", 4400.0)])
    _write_counters(write, [(COPY, "WRITE_SIZE", 1000.0), (CONV, "WRITE_SIZE", 500.0), (CONV, "WRITE_SIZE", 1500.0)])
    out = tmp_path / "t.json"
    rc = ps.main(["counters", str(fetch), str(write), "--command", "rocprofv3 --pmc ... -- python3 bench.py",
                  "--copy-kernel", "copy_probe_kernel", "--copy-bytes", str(1 << 20), "--json", str(out)])
    assert rc == 0
    table = json.loads(out.read_text())
    assert list(table) == [CONV]
    assert abs(table[CONV]["fetch_bytes"] - 3300.0 * 1024 * (1024 / 1100)) < 1e-3
    assert abs(table[CONV]["write_bytes"] - 1000.0 * 1024 * (1024 / 1000)) < 1e-3
    text = capsys.readouterr().out
    assert "rocprofv3 --pmc" in text and "FETCH_SIZE | 2 | 3300" in text


def test_stats_summary(tmp_path, capsys):
    p = tmp_path / "x_kernel_stats.csv"
    p.write_text('"Name","Calls","TotalDurationNs","AverageNs","Percentage","MinNs","MaxNs","StdDev"\n'
                 f'"{CONV}",240,240000000,1000000.0,91.5,1,2,3\n')
    assert ps.main(["stats", str(tmp_path), "--command", "rocprofv3 --kernel-trace --stats -- python3 bench.py"]) == 0
    text = capsys.readouterr().out
    assert f"{CONV} | 240 | 240.00 | 1000.0 | 91.50" in text
