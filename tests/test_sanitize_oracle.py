"""Host sanitizer pass: the CPU oracle, compiled with the address and undefined-behaviour
sanitizers, replays a seeded fuzz of graphs, fanouts, table types and saved-ID arrays from a
plain C++ driver whose buffers have exactly the sizes the oracle's header states."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_is_clean_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "sanitize_driver")
    subprocess.run(["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                    "-static-libasan", "-o", exe, os.path.join(ROOT, "tests", "native", "sanitize_driver.cpp"),
                    os.path.join(ROOT, "oracle", "fsa_oracle.cpp")], check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, timeout=600, env=env)
    sys.stdout.write(r.stdout)
    assert r.returncode == 0, r.stdout + r.stderr[-4000:]
    assert r.stdout.strip().endswith("cases") and "ok" in r.stdout
