"""Host-side property test of the balanced-launch index arithmetic, under AddressSanitizer and UBSan.

The streaming kernel (share -> pieces) and the combine kernel (row -> first piece id, count) take
their integer arithmetic from one header, paper_2408_04093_amd/csrc/balanced_index.hpp; this test
compiles that header for the host together with tests/balanced_index_check.cpp and runs the checks
described there.  No GPU.
"""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_share_walk_and_row_lookup_agree_on_seeded_random_length_tables(tmp_path):
    exe = str(tmp_path / "balanced_index_check")
    src = os.path.join(ROOT, "tests", "balanced_index_check.cpp")
    subprocess.run(["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan",
                    "-Wall", "-Wextra", src, "-o", exe], check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0")
    r = subprocess.run([exe, "400"], capture_output=True, text=True, env=env, timeout=600)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-2000:]
    assert "cases hold" in r.stdout
