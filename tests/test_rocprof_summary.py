"""The rocprofv3 harness (paper_2601_18511_amd/rocprof_summary.py) on captured and on hand-made csv files (CPU only).

tests/golden/rocprof/ holds rows cut out of real rocprofv3 output for the wide_pc_attn workload (kernel trace,
FETCH_SIZE, WRITE_SIZE and one counter group; only the PCMM kernels, the probe and the calibration copy were kept).
"""
import csv
import os

import pytest

from paper_2601_18511_amd import rocprof_summary as rs

GOLD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "rocprof")


def test_short_names():
    assert rs.short_name('void (anonymous namespace)::gemm_kernel<4, 4, 2, 5, 1, 0>((anonymous namespace)::GemmArgs)') \
        == "gemm_kernel<4, 4, 2, 5, 1, 0>"
    assert rs.short_name("(anonymous namespace)::mfma_probe_kernel(long long*, int, int)") == "mfma_probe_kernel"
    assert rs.short_name("__amd_rocclr_copyBuffer") == "__amd_rocclr_copyBuffer"
    assert rs.short_name("void at::native::vectorized_elementwise_kernel<4, at::native::FillFunctor<long>, std::array<char*, 1ul> >(int, at::native::FillFunctor<long>, std::array<char*, 1ul>)") \
        .startswith("at::native::vectorized_elementwise_kernel<4, at::native::FillFunctor<long>")


def test_captured_run_of_the_wide_workload():
    trace = rs.read_kernel_trace(os.path.join(GOLD, "kt"))
    assert len(trace["gemm_shortk_kernel<7, 2, 2>"]) == 12 and len(trace["split_kernel<7>"]) == 12
    avg_ms = rs.mean(trace["gemm_shortk_kernel<7, 2, 2>"]) / 1e6
    assert 5.5 < avg_ms < 7.0
    counters, durations = rs.merge_counters([os.path.join(GOLD, d) for d in ("fetch", "write", "cnt")])
    g = counters["gemm_shortk_kernel<7, 2, 2>"]
    assert {"FETCH_SIZE", "WRITE_SIZE", "GRBM_GUI_ACTIVE", "SQ_VALU_MFMA_BUSY_CYCLES"} <= set(g)
    # the calibration copy moves 1 GiB each way: FETCH_SIZE counts half of it, WRITE_SIZE all of it
    dirs = [os.path.join(GOLD, d) for d in ("fetch", "write", "cnt")]
    got, scale = rs.copy_scale(dirs, "FETCH_SIZE", float(1 << 20))
    assert abs(scale - 2.0) < 0.01
    got, scale = rs.copy_scale(dirs, "WRITE_SIZE", float(1 << 20))
    assert abs(scale - 1.0) < 0.01
    fig = rs.workload_figures("wide_pc_attn")
    assert fig["mfma_kernel"] == "gemm_shortk_kernel" and fig["int8_ops"] == 2.0 * 4096 * 128 * 131072 * 6 * 14
    text = rs.traffic_summary("wide_pc_attn", fig, counters, ["rocprofv3 --pmc FETCH_SIZE ..."], float(1 << 20), dirs)
    line = [x for x in text.splitlines() if x.startswith("traffic_bytes_per_launch=")]
    assert len(line) == 1
    traffic = float(line[0].split("=")[1])
    assert 0.98 < traffic / fig["gemm_bytes"] < 1.05          # this kernel reads and writes what it has to, once
    text = rs.counter_summary("wide_pc_attn", fig, counters, durations, ["rocprofv3 --pmc GRBM_GUI_ACTIVE ..."])
    busy = [x for x in text.splitlines() if "MFMA busy" in x][0]
    assert 50.0 < float(busy.split()[2]) < 70.0
    # every int8 MFMA the kernel issues is algorithmic work: 2 * 16 * 16 * 64 ops each
    assert rs.mean(g["SQ_INSTS_VALU_MFMA_I8"]) * 32768 == fig["int8_ops"]
    text = rs.trace_summary("wide_pc_attn", fig, trace, ["rocprofv3 --kernel-trace ..."])
    assert "gemm_shortk_kernel<7, 2, 2>" in text and "% of the 8000 GB/s HBM peak" in text


def _write_csv(path, header, rows):
    os.makedirs(os.path.dirname(path), exist_ok=True)
    with open(path, "w", newline="") as f:
        w = csv.writer(f, quoting=csv.QUOTE_NONNUMERIC)
        w.writerow(header)
        w.writerows(rows)


def test_hand_made_counters_give_the_expected_figures(tmp_path):
    """Known numbers in, known numbers out: scaling by the calibration copy, MFMA busy %, clock."""
    hdr = ["Correlation_Id", "Dispatch_Id", "Agent_Id", "Queue_Id", "Process_Id", "Thread_Id", "Grid_Size", "Kernel_Id",
           "Kernel_Name", "Workgroup_Size", "LDS_Block_Size", "Scratch_Size", "VGPR_Count", "Accum_VGPR_Count", "SGPR_Count",
           "Counter_Name", "Counter_Value", "Start_Timestamp", "End_Timestamp"]
    gk = "void (anonymous namespace)::gemm_kernel<4, 4, 2, 5, 1, 0>((anonymous namespace)::GemmArgs)"

    def row(disp, kernel, counter, value, t0=1000, t1=2000):
        return [disp, disp, "Agent 1", 1, 7, 7, 64, 1, kernel, 256, 0, 0, 8, 0, 32, counter, value, t0, t1]

    _write_csv(str(tmp_path / "f" / "h" / "1_counter_collection.csv"), hdr, [
        row(1, "__amd_rocclr_copyBuffer", "FETCH_SIZE", 262144.0),           # the 1 GiB copy counted as 256 MiB: scale 4
        row(2, gk, "FETCH_SIZE", 1000.0), row(3, gk, "FETCH_SIZE", 3000.0),
        row(4, "__amd_rocclr_copyBuffer", "FETCH_SIZE", 9999999.0)])         # a later, larger copy is not the calibration
    _write_csv(str(tmp_path / "w" / "h" / "2_counter_collection.csv"), hdr, [
        row(1, "__amd_rocclr_copyBuffer", "WRITE_SIZE", 2097152.0),          # counted twice: scale 0.5
        row(2, gk, "WRITE_SIZE", 8000.0), row(3, gk, "WRITE_SIZE", 8000.0)])
    _write_csv(str(tmp_path / "c" / "h" / "3_counter_collection.csv"), hdr, [
        row(2, gk, "GRBM_GUI_ACTIVE", 8.0e6, 0, 1000000), row(2, gk, "SQ_VALU_MFMA_BUSY_CYCLES", 5.12e8, 0, 1000000)])
    counters, durations = rs.merge_counters([str(tmp_path / d) for d in ("f", "w", "c")])
    fig = rs.workload_figures("attn_proj")
    text = rs.traffic_summary("attn_proj", fig, counters, [], float(1 << 20), [str(tmp_path / d) for d in ("f", "w", "c")])
    # mean FETCH 2000 KiB x 4 + mean WRITE 8000 KiB x 0.5 = 12000 KiB
    assert "traffic_bytes_per_launch=%d" % (12000 * 1024) in text
    text = rs.counter_summary("attn_proj", fig, counters, durations, [])
    # 8e6 / 8 XCDs = 1e6 cycles in 1 ms -> 1.00 GHz; 5.12e8 / (1024 x 1e6) = 50 %
    assert "1.00 GHz" in text and "50.0 %" in text


def test_command_line_writes_the_three_summaries(tmp_path):
    out = str(tmp_path) + os.sep
    rc = rs.main(["--workload", "wide_pc_attn", "--trace", os.path.join(GOLD, "kt"),
                  "--pmc", os.path.join(GOLD, "fetch"), "--pmc", os.path.join(GOLD, "write"), "--pmc", os.path.join(GOLD, "cnt"),
                  "--command", "rocprofv3 --kernel-trace --stats -- python3 bench.py",
                  "--command", "rocprofv3 --pmc FETCH_SIZE -- python3 bench.py",
                  "--command", "rocprofv3 --pmc GRBM_GUI_ACTIVE -- python3 bench.py", "--out-prefix", out])
    assert rc == 0
    names = sorted(os.listdir(out))
    assert names == ["gemm_shortk_kernel_wide_pc_attn_counters.txt", "gemm_shortk_kernel_wide_pc_attn_hbm_traffic.txt",
                     "gemm_shortk_kernel_wide_pc_attn_kernel_trace.txt"]
    assert "rocprofv3 --pmc FETCH_SIZE" in open(os.path.join(out, names[1])).read()
    with pytest.raises(KeyError):
        rs.workload_figures("no_such_workload")


def test_streaming_summary_groups_by_kernel_and_grid():
    text = rs.streaming_summary(os.path.join(GOLD, "kt"), os.path.join(GOLD, "fetch"), os.path.join(GOLD, "write"),
                                ["rocprofv3 ..."], float(1 << 20), ["a note"])
    row = [x for x in text.splitlines() if x.startswith("split_kernel<7>")]
    assert len(row) == 1
    cols = row[0].split()
    assert int(cols[1]) == 6291456 and int(cols[2]) == 12             # grid size; launches in the trace
    assert abs(float(cols[5]) - 0.75) < 0.01 and abs(float(cols[6]) - 0.656) < 0.01   # A read, digit planes written (GiB)
    assert 4500 < float(cols[7]) < 6500


def test_streaming_summary_lists_the_transform_kernels_of_both_decode_shapes(tmp_path):
    """Two instantiations of one persistent kernel launch the same grid; the template arguments keep them apart."""
    hdr = ["Correlation_Id", "Dispatch_Id", "Agent_Id", "Queue_Id", "Process_Id", "Thread_Id", "Grid_Size", "Kernel_Id",
           "Kernel_Name", "Workgroup_Size", "LDS_Block_Size", "Scratch_Size", "VGPR_Count", "Accum_VGPR_Count", "SGPR_Count",
           "Counter_Name", "Counter_Value", "Start_Timestamp", "End_Timestamp"]
    ns = "void (anonymous namespace)::"
    mac1 = ns + "mac_intt4096_kernel<true, true>(double const*, double const*, unsigned long*, double const*, (anonymous namespace)::LimbDev const*, unsigned int, int, unsigned int, unsigned int*)"
    mac4 = mac1.replace("<true, true>", "<true, false>")
    fwd = ns + "ntt4096_kernel<0, true>(void const*, double*, double const*, (anonymous namespace)::LimbDev const*, long, unsigned int*, unsigned int)"

    def rows(counter, scale):
        def row(disp, kernel, grid, kib, t1):
            return [disp, disp, "Agent 1", 1, 7, 7, grid, 1, kernel, 256, 0, 0, 8, 0, 32, counter, kib * scale, 0, t1]
        return [row(1, "__amd_rocclr_copyBuffer", 1 << 20, float(1 << 20), 400000),
                row(2, fwd, 1024, 64.0, 6000), row(3, mac1, 131072, 262144.0, 200000), row(4, mac4, 131072, 1048576.0, 400000)]

    _write_csv(str(tmp_path / "f" / "h" / "1_counter_collection.csv"), hdr, rows("FETCH_SIZE", 0.5))
    _write_csv(str(tmp_path / "w" / "h" / "2_counter_collection.csv"), hdr, rows("WRITE_SIZE", 1.0))
    text = rs.streaming_summary(None, str(tmp_path / "f"), str(tmp_path / "w"), [], float(1 << 20), [])
    got = {x.split("  ")[0].strip(): x.split() for x in text.splitlines() if "4096_kernel" in x}
    assert set(got) == {"mac_intt4096_kernel<true, true>", "mac_intt4096_kernel<true, false>", "ntt4096_kernel<0, true>"}
    one = got["mac_intt4096_kernel<true, true>"]
    # 256 MiB read (the counter halves it, the calibration doubles it back) + 256 MiB written in 0.2 ms
    assert abs(float(one[-3]) - 0.25) < 1e-3 and abs(float(one[-2]) - 0.25) < 1e-3
    assert abs(float(one[-1]) - 2 * 268435456 / 0.2e-3 / 1e9) < 1.0
