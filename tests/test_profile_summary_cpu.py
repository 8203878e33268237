"""profile_summary.py turns rocprofv3 CSV files into the text summaries under profiles/: checked on
small hand-made CSV files (no profiler and no GPU needed)."""
import csv
import os

from paper_2406_09425_amd import profile_summary as ps


def write_csv(path, header, rows):
    os.makedirs(os.path.dirname(path), exist_ok=True)
    with open(path, "w", newline="") as f:
        w = csv.writer(f)
        w.writerow(header)
        w.writerows(rows)


def test_stats_table(tmp_path):
    write_csv(str(tmp_path / "a" / "x_kernel_stats.csv"), ["Name", "Calls", "TotalDurationNs", "AverageNs", "Percentage"],
              [["void sgprs::k1(int)", 4, 100000, 25000.0, 80.0], ["void sgprs::k2()", 2, 25000, 12500.0, 20.0]])
    out = ps.stats(str(tmp_path), "cmd --flag")
    lines = out.splitlines()
    assert lines[0] == "command: cmd --flag"
    k1 = next(l for l in lines if "k1" in l).split()
    assert k1[-4:] == ["4", "25.00", "0.100", "80.00"]


def test_pmc_scaling_by_the_calibration_copy(tmp_path):
    hdr = ["Kernel_Name", "Grid_Size", "Counter_Name", "Counter_Value"]
    # the calibration copy moves 262144 KiB each way; FETCH_SIZE reads half of it, WRITE_SIZE all of it
    write_csv(str(tmp_path / "f" / "f_counter_collection.csv"), hdr,
              [["void sgprs::bn_relu_kernel<1>()", 1000, "FETCH_SIZE", 131072.0],
               ["void sgprs::conv()", 256, "FETCH_SIZE", 1000.0], ["void sgprs::conv()", 256, "FETCH_SIZE", 3000.0]])
    write_csv(str(tmp_path / "w" / "w_counter_collection.csv"), hdr,
              [["void sgprs::bn_relu_kernel<1>()", 1000, "WRITE_SIZE", 262144.0], ["void sgprs::conv()", 256, "WRITE_SIZE", 500.0],
               ["void sgprs::conv()", 256, "WRITE_SIZE", 500.0]])
    out = ps.pmc(str(tmp_path / "f"), str(tmp_path / "w"), "cmd")
    assert "factors 2.0000 (fetch), 1.0000 (write)" in out
    conv = next(l for l in out.splitlines() if "conv()" in l).split()
    # mean 2000 KiB * 2.0 * 1024 / 1e6 = 4.10 MB fetched, 500 KiB * 1024 / 1e6 = 0.51 MB written, two dispatches
    assert conv[-3:] == ["2", "4.10", "0.51"]


def test_sq_shares(tmp_path):
    hdr = ["Kernel_Name", "Grid_Size", "Counter_Name", "Counter_Value"]
    k = "void sgprs::conv()"
    # 32 shader engines busy for 1000 cycles each = 1000 cycles; 1024 SIMDs -> 1 024 000 SIMD cycles
    write_csv(str(tmp_path / "r1" / "p_counter_collection.csv"), hdr,
              [[k, 256, "SQ_BUSY_CYCLES", 32000.0], [k, 256, "SQ_WAVES", 512.0], [k, 256, "SQ_VALU_MFMA_BUSY_CYCLES", 256000.0],
               [k, 256, "SQ_ACTIVE_INST_VALU", 51200.0], [k, 256, "SQ_ACTIVE_INST_ANY", 128000.0]])
    write_csv(str(tmp_path / "r2" / "p_counter_collection.csv"), hdr,
              [[k, 256, "SQ_INSTS_VALU", 51200.0], [k, 256, "SQ_LDS_BANK_CONFLICT", 10.0], [k, 256, "SQ_LDS_IDX_ACTIVE", 40.0]])
    out = ps.sq([str(tmp_path / "r1"), str(tmp_path / "r2")], "cmd")
    row = next(l for l in out.splitlines() if l.startswith("conv()")).split()
    assert row[1:4] == ["1000", "512", "25.0%"]      # cycles, waves, MFMA busy = 256000 / 1024000
    assert row[4] == "20.0%" and row[8] == "50.0%"   # VALU = 51200 * 4 / 1024000, any instruction = 128000 * 4 / 1024000
    assert row[10] == "100" and row[-1] == "25.0%"   # VALU instructions per wavefront, bank conflicts 10 / 40


def test_concurrency_from_a_kernel_trace(tmp_path):
    hdr = ["Kind", "Queue_Id", "Kernel_Name", "Start_Timestamp", "End_Timestamp"]
    k = "void sgprs::conv()"
    # warm-up kernel (dropped with the first 30 % of the trace), then on queue 1: [1000, 2000) and
    # [3000, 4000); on queue 2: [1500, 3500); one kernel of another library is ignored
    write_csv(str(tmp_path / "t" / "x_kernel_trace.csv"), hdr,
              [["KERNEL_DISPATCH", 1, k, 0, 10], ["KERNEL_DISPATCH", 1, k, 1000, 2000], ["KERNEL_DISPATCH", 1, k, 3000, 4000],
               ["KERNEL_DISPATCH", 2, k, 1500, 3500], ["KERNEL_DISPATCH", 3, "other_kernel", 1000, 4000]])
    out = ps.concurrency(str(tmp_path), "cmd", skip_first_fraction=0.2)
    lines = out.splitlines()
    assert lines[0] == "command: cmd" and "3 sgprs kernels" in lines[2]
    q1 = next(l for l in lines if l.startswith("1 ")).split()
    assert q1[1:3] == ["2", "2.0"]                       # two kernels, 2.0 us busy
    # interval 3000 ns: one kernel in flight during [1000,1500) + [2000,3000) + [3500,4000) = 2000, two during 1000
    i = lines.index(next(l for l in lines if l.startswith("kernels in flight")))
    assert lines[i + 1].split() == ["0", "0.000"] or lines[i + 1].split()[0] == "1"
    shares = {l.split()[0]: float(l.split()[1]) for l in lines[i + 1:i + 4] if l and l[0].isdigit()}
    assert abs(shares["1"] - 2000 / 3000) < 1e-3 and abs(shares["2"] - 1000 / 3000) < 1e-3
