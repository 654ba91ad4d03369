"""The counter reader behind bench.py's `roofline.traffic` (no GPU, no profiler needed): small
rocprofv3-shaped CSV files written here must come back as the bytes they stand for."""
import csv
import json
import os

from paper_2505_14884_amd import rocprof

COLS = ["Correlation_Id", "Dispatch_Id", "Agent_Id", "Queue_Id", "Process_Id", "Thread_Id", "Grid_Size", "Kernel_Id",
        "Kernel_Name", "Workgroup_Size", "LDS_Block_Size", "Scratch_Size", "VGPR_Count", "Accum_VGPR_Count", "SGPR_Count",
        "Counter_Name", "Counter_Value", "Start_Timestamp", "End_Timestamp"]
STREAM = ("void polar::(anonymous namespace)::sha_partial_kernel<polar::(anonymous namespace)::F16, 128, 1, false, false>"
          "(unsigned short const*, unsigned short const*, int const*, float*)")
GQA = "void polar::(anonymous namespace)::sha_partial_gqa_kernel<true, false>(unsigned short const*)"
COPY = "__amd_rocclr_copyBuffer"


def write_pass(root, name, counter, rows, meta=None):
    d = os.path.join(root, name, "host", "1234")           # rocprofv3 nests its output; the reader searches
    os.makedirs(d)
    with open(os.path.join(d, "p_counter_collection.csv"), "w", newline="") as f:
        w = csv.writer(f, quoting=csv.QUOTE_NONNUMERIC)
        w.writerow(COLS)
        for i, (kernel, value) in enumerate(rows):
            w.writerow([i, i, "Agent 1", 1, 1, 1, 256, 7, kernel, 512, 0, 0, 90, 0, 48, counter, value, 10, 20])
    if meta is not None:
        with open(os.path.join(root, name + ".json"), "w") as f:
            f.write("some log line\n" + json.dumps(meta) + "\n")


def test_traffic_is_scaled_by_the_copy_yardstick(tmp_path):
    root = str(tmp_path)
    nbytes = 4 << 30
    # the copy reads 4 GiB: FETCH_SIZE shows half of it (factor 2), WRITE_SIZE all of it (factor 1)
    write_pass(root, "copy_fetch", "FETCH_SIZE", [(COPY, nbytes / 1024 / 2)] * 3 + [("other_kernel", 5.0)],
               {"phase": "copy", "bytes_read_per_launch": nbytes, "bytes_written_per_launch": nbytes})
    write_pass(root, "copy_write", "WRITE_SIZE", [(COPY, nbytes / 1024)] * 3)
    write_pass(root, "fetch", "FETCH_SIZE", [(STREAM, 1000.0), (STREAM, 1200.0), (GQA, 7.0), ("fill", 1.0)],
               {"phase": "partial", "algorithmic_bytes_per_launch": 2_000_000})
    write_pass(root, "write", "WRITE_SIZE", [(STREAM, 10.0), (STREAM, 30.0), (GQA, 9.0)])
    fac = rocprof.copy_factors(root)
    assert abs(fac["fetch_factor"] - 2.0) < 1e-12 and abs(fac["write_factor"] - 1.0) < 1e-12
    t = rocprof.traffic_from(root, ["sha_partial_kernel<"])
    assert [k["kernel"] for k in t["kernels"]] == ["sha_partial_kernel<F16, 128, 1, false, false>"]   # not the grouped kernel
    assert t["kernels"][0]["dispatches"] == 2
    assert t["read_bytes"] == int(1100.0 * 1024 * 2.0) and t["written_bytes"] == int(20.0 * 1024)
    assert t["bytes"] == t["read_bytes"] + t["written_bytes"]
    g = rocprof.traffic_from(root, ["sha_partial_gqa_kernel<"])
    assert g["read_bytes"] == int(7.0 * 1024 * 2) and g["written_bytes"] == int(9.0 * 1024)
    assert rocprof.traffic_from(root, ["no_such_kernel"]) is None
    assert rocprof.traffic_from(os.path.join(root, "fetch"), ["sha_partial_kernel<"]) is None      # no copy passes there
    # without a bench record the summary lists every streaming kernel the passes saw: (1100 + 7) KiB x 2 read, 29 KiB written
    text = rocprof.summarize_attention(root)
    assert "2.2968e+06" in text and "FETCH_SIZE x 2.0000" in text and "1.1484 x algorithmic" in text


def test_kernel_names_and_stats(tmp_path):
    assert rocprof.short_name(STREAM) == "sha_partial_kernel<F16, 128, 1, false, false>"
    assert rocprof.short_name("void foo(int)") == "foo"
    assert rocprof.short_name("bar<baz<int>(3)>(float)") == "bar<baz<int>(3)>"
    d = tmp_path / "trace"
    d.mkdir()
    with open(d / "t_kernel_stats.csv", "w", newline="") as f:
        w = csv.writer(f, quoting=csv.QUOTE_NONNUMERIC)
        w.writerow(["Name", "Calls", "TotalDurationNs", "AverageNs", "Percentage", "MinNs", "MaxNs", "StdDev"])
        w.writerow([STREAM, 10, 6570000, 657000.0, 90.0, 640000, 680000, 1.0])
        w.writerow(["void at::native::something<float>(int)", 5, 10, 2.0, 1.0, 1, 3, 0.1])
    rows = rocprof.kernel_stats(str(d))
    assert len(rows) == 1 and rows[0]["calls"] == 10 and abs(rows[0]["avg_us"] - 657.0) < 1e-9
    table = rocprof.summarize_kernels(["full=" + str(d)], "sha_partial", "title", "note")
    assert "| full | `sha_partial_kernel<F16, 128, 1, false, false>` | 10 | 657.00 | 640.00 | 680.00 |" in table
