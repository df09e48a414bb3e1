"""The fp64 exponential used by the device's exact path, compiled for the host
from the same header and compared with libm."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_exp_nonpos_matches_libm_within_one_ulp(tmp_path):
    exe = str(tmp_path / "exp64_check")
    subprocess.run(["g++", "-O2", "-ffp-contract=off", "-I", os.path.join(ROOT, "paper_2410_03355_amd", "csrc"),
                    os.path.join(ROOT, "tests", "exp64_check.cpp"), "-o", exe, "-lm"], check=True)
    worst, n_diff, n, specials, worst_tab, n_diff_tab, specials_tab = (
        int(x) for x in subprocess.run([exe], check=True, capture_output=True, text=True).stdout.split())
    assert worst <= 1            # never more than one ulp from libm
    assert n_diff < 0.1 * n      # and identical for the large majority of arguments
    assert specials == 1
    # the table-driven routine (arguments of either sign)
    assert worst_tab <= 1 and n_diff_tab < 0.1 * 3000000 and specials_tab == 1
