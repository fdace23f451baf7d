"""Host logic of the per-launch roofline report: which bound a launch is graded on, and the line format."""
import io

from paper_2312_16733_amd import layer_report as lr


def test_bound_follows_arithmetic_intensity():
    # 2.5 PFLOP/s over 8 TB/s: ridge at 312.5 flop/B
    assert abs(lr.RIDGE - 312.5) < 1e-9
    bound, ach, frac = lr.grade(flops=1e9, nbytes=1e7, us=10.0)          # AI = 100 < ridge: graded on bytes
    assert bound == "hbm" and abs(ach - 1000.0) < 1e-6 and abs(frac - 0.125) < 1e-9
    bound, ach, frac = lr.grade(flops=1e10, nbytes=1e7, us=10.0)         # AI = 1000 > ridge: graded on flops
    assert bound == "mfma" and abs(ach - 1000.0) < 1e-6 and abs(frac - 0.4) < 1e-9
    assert lr.grade(1e9, 0.0, 10.0)[0] == "-"                            # a launch with no algorithmic bytes is not graded


def test_launch_line_and_table_totals():
    us, cls, flops, nbytes, what = lr.parse_line("12.500 igemm_conv_linear flops=2000000000 bytes=10000000 tile=3 [M=64 K=8 C=8 1x1/1 tiles=2]")
    assert (us, cls, flops, nbytes) == (12.5, "igemm_conv_linear", 2e9, 1e7) and what.startswith("tile=3")
    assert lr.parse_line("7.000 pool flops=0 bytes=4096 ")[4] == ""
    rows = [(10.0, "a", 1e9, 1e7, "x"), (30.0, "a", 1e9, 1e7, "x"), (5.0, "b", 0.0, 4e6, "")]
    out = io.StringIO()
    lr.report(rows, "t", out)
    text = out.getvalue()
    # identical launches merge into one line with their count and mean time
    assert "  2   20.00 a" in text and "  1    5.00 b" in text
    # sum of per-launch roofline times: 2 x max(0.4 us, 1.25 us) + 0.5 us = 3.0 us of 45 us
    assert "total: 3 launches, 45.0 us" in text and "roofline times 3.0 us = 0.067" in text
