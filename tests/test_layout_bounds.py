"""Host-side check of the LDS index arithmetic the forward kernels share with the launch code
(paper_2511_13645_amd/csrc/fsa_layout.h): a plain C++ driver, built with the address and
undefined-behaviour sanitizers, sweeps every fanout pair, waves-per-root value and table
flavour and asserts that each index a kernel can form stays in bounds."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_every_lds_index_of_the_two_hop_forward_stays_in_bounds(tmp_path):
    exe = str(tmp_path / "layout_check")
    src = os.path.join(ROOT, "tests", "native", "layout_check.cpp")
    subprocess.run(["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                    "-static-libasan", "-o", exe, src], check=True)
    r = subprocess.run([exe], capture_output=True, text=True, timeout=600)
    sys.stdout.write(r.stdout)
    assert r.returncode == 0, r.stdout + r.stderr
    assert r.stdout.startswith("ok ")
