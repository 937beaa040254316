"""The two tools that turn rocprofv3 CSV output into the summaries under profiles/, on
hand-made miniature inputs (tests/golden/rocprof_fixture) whose figures can be checked by hand."""
import os

from paper_2401_09290_amd import pmc_summary, rocprof_summary

FIX = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "rocprof_fixture")


def test_counter_summary_pairs_builds_calibrates_and_reports_the_headline_traffic():
    ins = pmc_summary.load(os.path.join(FIX, "insts"))
    assert set(ins) == {"k_stream<0, 0, true>", "k_stream<0, 1, true>", "k_stream<2, 1, true>", "k_gemm_ring<1>"}   # foreign kernels dropped
    assert ins["k_stream<2, 1, true>"]["SQ_INSTS_VALU"] == 3000 and ins["k_stream<2, 1, true>"]["calls"] == 2
    _, rows = pmc_summary.fence_cost(ins)
    (name, dv, ds, pct), = rows                                  # only the fenced triad has an unfenced twin
    assert name == "k_stream<2, 1, true>" and dv == 1.0 and ds == 16.0 and abs(pct - 100.0 / 29.0) < 1e-9
    text = pmc_summary.summarise(FIX, copy_elems=1 << 18)        # the copy moved 1 MiB each way = 1024 KiB
    # calibration: FETCH_SIZE read 512 for 1024 KiB -> factor 2; WRITE_SIZE read 1000 -> factor 1.024
    assert "scale factors 2.00000 (fetch) and 1.02400 (write)" in text
    # fenced triad: 1025 * 2 KiB fetched + 1001 * 1.024 KiB written
    want = 1025 * 2 * 1024 + 1001 * 1.024 * 1024
    line = [ln for ln in text.splitlines() if ln.startswith("traffic_bytes_per_launch:")]
    assert len(line) == 1 and abs(float(line[0].split(":")[1]) - want) < 1.0
    # GEMM: 524288 busy cycles over (8192 / 8) cycles x 1024 SIMDs = 50 %; clock 1024 cycles / 640 ns = 1.6 GHz
    mf = [ln for ln in text.splitlines() if ln.startswith("* k_gemm_ring<1>")]
    assert len(mf) == 1 and "= 50.0 % of the matrix-pipe cycles" in mf[0] and "1.60 GHz" in mf[0] and "8.0 per instruction" in mf[0]


def test_trace_summary_separates_overlapped_from_solitary_dispatches():
    rows = rocprof_summary.load(os.path.join(FIX, "kernel_trace.csv"))
    assert rocprof_summary.alone_flags(rows) == [True, False, False, True, True]
    text = rocprof_summary.summarise(os.path.join(FIX, "kernel_trace.csv"), "gd::")
    lines = {ln.split(" | ")[0]: ln.split(" | ") for ln in text.splitlines()[2:]}
    assert set(lines) == {"gd::A<1>", "gd::B<0>"}
    a = lines["gd::A<1>"]
    assert a[1] == "3" and a[2] == "1.0" and a[3] == "2" and a[4] == "0.8" and a[5] == "0.5"     # (1+1.5+0.5)/3, (1+0.5)/2 us
    b = lines["gd::B<0>"]
    assert b[1] == "1" and b[3] == "0" and b[4] == "nan" and b[8] == "512"
