"""The profile summariser (paper_2309_11071_amd.profile_summary) on hand-made rocprofv3 CSV files:
duration table, the window of large launches in launch order, medians of the large launches of a
counter and the calibration factors."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
K = "void ink::k_agg_events<false, 32, false>(ink::AggArgs)"
COPY = "void at::native::vectorized_elementwise_kernel<4, at::native::AUnaryFunctor<float, float, float, at::native::binary_internal::MulFunctor<float> > >"
GATHER = "void at::native::vectorized_gather_kernel<16, long>(char*, char*, long*, int)"


def _write(tmp_path):
    kt = tmp_path / "kt"
    kt.mkdir()
    (kt / "kt_kernel_stats.csv").write_text(
        '"Name","Calls","TotalDurationNs","AverageNs","Percentage","MinNs","MaxNs","StdDev"\n'
        '"%s",6,33000000,5500000,90.0,1000000,10000000,1.0\n'
        '"void ink::k_other(int)",2,1000,500,10.0,400,600,1.0\n' % K)
    rows = ['"Kind","Agent_Id","Queue_Id","Stream_Id","Thread_Id","Dispatch_Id","Kernel_Id","Kernel_Name","Correlation_Id",'
            '"Start_Timestamp","End_Timestamp"']
    # launch order: small, 8 ms, 9 ms, 10 ms, small, 7 ms   (large = at least 0.2 of the longest)
    for i, ms in enumerate((1.0, 8.0, 9.0, 10.0, 1.5, 7.0)):
        start = 1000000000 + i * 20000000
        rows.append('"KERNEL_DISPATCH","Agent 1",1,0,1,%d,10,"%s",%d,%d,%d' % (i + 1, K, i + 1, start, start + int(ms * 1e6)))
    (kt / "kt_kernel_trace.csv").write_text("\n".join(rows) + "\n")
    pmc = tmp_path / "fetch"
    pmc.mkdir()
    head = ('"Correlation_Id","Dispatch_Id","Agent_Id","Queue_Id","Process_Id","Thread_Id","Grid_Size","Kernel_Id","Kernel_Name",'
            '"Workgroup_Size","LDS_Block_Size","Scratch_Size","VGPR_Count","Accum_VGPR_Count","SGPR_Count","Counter_Name",'
            '"Counter_Value","Start_Timestamp","End_Timestamp"')
    lines = [head]
    d = 0

    def add(name, grid, value):
        nonlocal d
        d += 1
        lines.append('%d,%d,"Agent 1",1,1,1,%d,10,"%s",256,0,0,8,0,48,"FETCH_SIZE",%f,1,2' % (d, d, grid, name, value))
    for kib in (393216.0, 655360.0, 1179648.0):           # gathers of 2^21 rows of 192 / 512 / 1024 B
        add(GATHER, 1 << 21, kib)
    add(COPY, 1 << 28, 524288.0)                          # 1 GiB read shows as 512 MiB: factor 2
    for kib in (100.0, 9000.0, 10000.0, 11000.0, 50.0):
        add(K, 1 << 20, kib)
    (pmc / "p_counter_collection.csv").write_text("\n".join(lines) + "\n")
    return str(kt), str(pmc)


def test_summary_of_handmade_profiles(tmp_path):
    kt, pmc = _write(tmp_path)
    out = subprocess.run([sys.executable, "-m", "paper_2309_11071_amd.profile_summary", "--kernel", "k_agg_events<false, 32, false>",
                          "--stats", kt, "--window", "1", "2", "--pmc", pmc], cwd=ROOT, capture_output=True, text=True, check=True).stdout
    assert "| 6 | 33.000 | 5500.0 | 1000.0 | 10000.0 |" in out and "k_other" not in out
    # large launches: 8, 9, 10, 7 ms; the window skips the first of them and takes two: 9 and 10 ms
    assert "4 of 6; average 8.500 ms, median 9.000 ms, min 7.000 ms, max 10.000 ms" in out
    assert "large launches 2 .. 3 in launch order (the timed steps): average 9.500 ms, median 10.000 ms" in out
    assert "| FETCH_SIZE | 5 | 3 | 10000 | 11000 |" in out
    assert "elementwise copy (1 GiB read, 1 GiB written): FETCH_SIZE = 524288 KiB -> factor 2.000" in out
    assert "rows of 192 B (read side 384 MiB known): FETCH_SIZE = 393216 KiB -> factor 1.000" in out
    assert "rows of 512 B (read side 1024 MiB known): FETCH_SIZE = 655360 KiB -> factor 1.600" in out
