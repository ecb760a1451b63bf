"""The tool that turns rocprofv3 output into the summaries under profiles/: checked on small
hand-made CSV files (no GPU, no profiler)."""
import json
import os

from paper_2602_08585_amd import profsum


def _write(path, header, rows):
    os.makedirs(os.path.dirname(path), exist_ok=True)
    with open(path, "w") as f:
        f.write(",".join(header) + "\n")
        for r in rows:
            f.write(",".join('"%s"' % x for x in r) + "\n")


def _counter_dir(root, name, counter, values):
    rows = []
    for kernel, vals in values.items():
        for v in vals:
            rows.append((kernel, counter, v))
    _write(os.path.join(root, name, "vm", "1_counter_collection.csv"), ["Kernel_Name", "Counter_Name", "Counter_Value"], rows)
    return os.path.join(root, name)


def test_traffic_scales_by_the_copy_kernel(tmp_path, capsys):
    copy = "void lukv::copy_kernel(HIP_vector_type<unsigned int, 4u> const*, HIP_vector_type<unsigned int, 4u>*, long)"
    stats = "void lukv::score_stats_kernel<false, 128, 4, 1>(lukv::Geom, lukv::SeqTab)"
    other = "void at::native::vectorized_elementwise_kernel<4>(int)"
    # FETCH_SIZE reads half the bytes: the 64 MiB copy shows 32768 KiB; WRITE_SIZE all of them
    fd = _counter_dir(str(tmp_path), "fetch", "FETCH_SIZE", {copy: [32768, 32768, 1000], stats: [1000, 3000], other: [5]})
    wd = _counter_dir(str(tmp_path), "write", "WRITE_SIZE", {copy: [65536, 65536, 2000], stats: [100, 300]})
    out = os.path.join(str(tmp_path), "t.json")
    profsum.traffic(fd, wd, out)
    rec = json.load(open(out))
    assert rec["score_stats"] == {"fetch_bytes": 2000 * 1024 * 2, "write_bytes": 200 * 1024,
                                  "fetch_scale": 2.0, "write_scale": 1.0}
    assert "vectorized_elementwise_kernel" not in rec and "copy_kernel" in rec
    assert "factor 2.0000" in capsys.readouterr().out


def test_trace_lists_library_kernels_and_gaps(tmp_path, capsys):
    d = os.path.join(str(tmp_path), "trace", "vm")
    _write(os.path.join(d, "1_kernel_stats.csv"), ["Name", "Calls", "AverageNs", "MinNs", "MaxNs"],
           [("void lukv::sel_tail_kernel(int)", 3, 7000, 6000, 9000), ("void other_kernel(int)", 1, 5, 5, 5)])
    _write(os.path.join(d, "1_kernel_trace.csv"), ["Kernel_Name", "Start_Timestamp", "End_Timestamp"],
           [("void lukv::a(int)", 1000, 2000), ("void lukv::b(int)", 3000, 4000), ("void lukv::c(int)", 6000, 7000)])
    profsum.trace(os.path.join(str(tmp_path), "trace"))
    text = capsys.readouterr().out
    assert "sel_tail_kernel" in text and "7.00" in text and "other_kernel" not in text
    assert "mean 1.50 us over 2 gaps" in text
