"""The summarising halves of paper_2603_04716_amd/traffic_probe.py on hand-made rocprofv3 csv files:
calibration by the copy kernel, grouping by (kernel, grid), and the step-by-step decode table (steps
found by their first launch, counter files matched to the trace by dispatch order).  No GPU."""
import csv
import io
import contextlib

from paper_2603_04716_amd import traffic_probe as TP

TRACE_COLS = ["Kind", "Dispatch_Id", "Kernel_Name", "Start_Timestamp", "End_Timestamp", "Workgroup_Size_X",
              "Workgroup_Size_Y", "Workgroup_Size_Z", "Grid_Size_X", "Grid_Size_Y", "Grid_Size_Z"]
CNT_COLS = ["Dispatch_Id", "Kernel_Name", "Grid_Size", "Workgroup_Size", "Counter_Name", "Counter_Value"]


def _dispatches():
    """(name, workgroup size, grid x, grid y, duration ns, fetch KiB reading, write KiB reading)"""
    copy = ("void pd::stream_copy_kernel(void*, void const*, unsigned long)", 256, 1048576, 1, 450000,
            524288.0, 1048576.0)                      # 1 GiB each way; FETCH_SIZE reads half
    step = lambda b, t: [
        ("pd::decode_meta_norm_kernel(pd::IntChunk, int*)", 256, 256 * (b + 1), 1, 5000, 1.0, 1.0),
        ("void pd::gemm_mfma_kernel<64, 128, 2, 2, 3, 4, false>(pd::GemmArgs, int, int, int)", 256, 256 * 48, 5,
         t, 24576.0, 8192.0),
        ("pd::splitk_reduce_kernel(pd::GemmArgs, int)", 256, 256 * 384, 1, 4000, 4096.0, 1024.0),
        ("void pd::decode_attn_kernel<false, false, true>(pd::DecodeAttnArgs, int)", 256, 256 * 256, 1, 100000,
         262144.0, 2048.0),
        ("void pd::gemm_mfma_kernel<64, 128, 2, 2, 3, 4, false>(pd::GemmArgs, int, int, int)", 256, 256 * 32, 8,
         11000, 16384.0, 8192.0),
        ("pd::splitk_reduce_norm_kernel(pd::GemmArgs, int, pd::RopeArgs, int)", 512, 512 * 128, 1, 7000, 8192.0, 3072.0),
        ("void pd::gemm_mfma_kernel<64, 128, 2, 2, 2, 4, false>(pd::GemmArgs, int, int, int)", 256, 256 * 224, 1,
         45000, 229376.0, 2048.0),
        ("void pd::gemm_mfma_kernel<64, 128, 2, 2, 3, 4, false>(pd::GemmArgs, int, int, int)", 256, 256 * 32, 8,
         28000, 114688.0, 8192.0),
        ("pd::splitk_reduce_kernel(pd::GemmArgs, int)", 256, 256 * 256, 1, 5000, 8192.0, 512.0),
        ("pd::scatter_ints_kernel(int*, pd::IntChunk, int)", 128, 128, 1, 4000, 0.1, 0.1),
    ]
    return [copy] + step(64, 17000) + step(64, 19000)


def _write(tmp_path):
    d = _dispatches()
    trace, fetch, write = tmp_path / "trace.csv", tmp_path / "fetch.csv", tmp_path / "write.csv"
    t = 1000
    with open(trace, "w", newline="") as f:
        w = csv.DictWriter(f, TRACE_COLS)
        w.writeheader()
        for i, (name, wg, gx, gy, dur, _, _) in enumerate(d):
            w.writerow({"Kind": "KERNEL_DISPATCH", "Dispatch_Id": i + 1, "Kernel_Name": name, "Start_Timestamp": t,
                        "End_Timestamp": t + dur, "Workgroup_Size_X": wg, "Workgroup_Size_Y": 1,
                        "Workgroup_Size_Z": 1, "Grid_Size_X": gx, "Grid_Size_Y": gy, "Grid_Size_Z": 1})
            t += dur + 100
    for path, counter, col in ((fetch, "FETCH_SIZE", 5), (write, "WRITE_SIZE", 6)):
        with open(path, "w", newline="") as f:
            w = csv.DictWriter(f, CNT_COLS)
            w.writeheader()
            for i, row in enumerate(d):
                w.writerow({"Dispatch_Id": i + 1, "Kernel_Name": row[0], "Grid_Size": row[2] * row[3],
                            "Workgroup_Size": row[1], "Counter_Name": counter, "Counter_Value": row[col]})
    return str(trace), str(fetch), str(write)


def _run(fn, *args):
    buf = io.StringIO()
    with contextlib.redirect_stdout(buf):
        fn(*args)
    return buf.getvalue()


def _rows(text):
    return [[c.strip() for c in line.strip().strip("|").split("|")] for line in text.splitlines()
            if line.startswith("|") and not line.startswith("|---")]


def test_summarise_scales_by_the_copy_kernel(tmp_path):
    _, fetch, write = _write(tmp_path)
    out = _run(TP.summarise, fetch, write)
    assert "scale factors 2.0000 (fetch), 1.0000 (write)" in out
    rows = {(r[0], r[1]): r for r in _rows(out)[1:]}
    copy = rows[("`stream_copy_kernel`", "1048576")]
    assert copy[3] == "1073.7" and copy[4] == "1073.7"            # 1 GiB = 1073.7 MB each way
    gate_up = rows[("`gemm_mfma_kernel<64, 128, 2, 2, 2, 4, false>`", str(256 * 224))]
    assert gate_up[2] == "2"                                       # two dispatches, one per step
    assert gate_up[3] == f"{229376.0 * 2.0 * 1024 / 1e6:.1f}"      # fetched MB with the factor 2
    assert gate_up[4] == f"{2048.0 * 1024 / 1e6:.1f}"


def test_durations_groups_by_kernel_and_grid(tmp_path):
    trace, _, _ = _write(tmp_path)
    rows = _rows(_run(TP.durations, trace))[1:]
    by = {(r[0], r[1]): r for r in rows}
    qkv = by[("`gemm_mfma_kernel<64, 128, 2, 2, 3, 4, false>`", str(48 * 5))]
    assert qkv[3] == "2" and qkv[4] == "18.0" and qkv[5] == "17.0"  # mean and min of 17 and 19 us
    shared = by[("`gemm_mfma_kernel<64, 128, 2, 2, 3, 4, false>`", str(32 * 8))]
    assert shared[3] == "4"                                        # O and down share a grid


def test_decode_steps_names_the_products_by_position(tmp_path):
    trace, fetch, write = _write(tmp_path)
    rows = _rows(_run(TP.decode_steps, trace, fetch, write))[1:]
    assert all(r[0] == "64" for r in rows)
    launches = [r[1] for r in rows]
    assert launches == ["", "QKV projection", "sum of the K splits", "", "O projection + residual",
                        "sum of the K splits", "gate/up + SwiGLU", "down projection + residual",
                        "sum of the K splits", "all launches of the step"]
    qkv = rows[1]
    assert qkv[3] == "48 x 5" and qkv[5] == "18.0"                 # grid x K splits, mean of 17 and 19 us
    assert qkv[6] == f"{24576.0 * 2.0 * 1024 / 1e6:.1f}" and qkv[7] == f"{8192.0 * 1024 / 1e6:.1f}"
    o, down = rows[4], rows[7]
    assert o[5] == "11.0" and down[5] == "28.0"                    # same kernel and grid, told apart by order
    total = float(rows[-1][5])
    assert abs(total - (5 + 18 + 4 + 100 + 11 + 7 + 45 + 28 + 5)) < 0.05
