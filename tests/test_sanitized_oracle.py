"""The oracle's pins once more, against a build of oracle/ta_oracle.c with AddressSanitizer and UBSan.

The oracle allocates score arrays, walks chunk tables and merge lists; an out-of-range index there
would silently corrupt the checker every GPU test relies on.  The pins run in a child process that
has the ASan runtime preloaded (an instrumented shared object cannot be loaded otherwise); any report
aborts that process.  Host code only: no GPU, no GPU sanitizer.
"""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_pins_pass_under_asan_and_ubsan():
    sys.path.insert(0, ROOT)
    from oracle import build as oracle_build
    oracle_build.build(sanitize=True)
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True, check=True).stdout.strip()
    preload = ":".join(x for x in (asan, os.environ.get("LD_PRELOAD", "")) if x)   # ASan first, nothing dropped
    env = dict(os.environ, TA_ORACLE_SANITIZED="1", LD_PRELOAD=preload,
               ASAN_OPTIONS="detect_leaks=0:abort_on_error=1", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1",
               OMP_NUM_THREADS="4")
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                        "-p", "no:cacheprovider"], capture_output=True, text=True, env=env, cwd=ROOT, timeout=1200)
    tail = r.stdout[-3000:] + r.stderr[-3000:]
    assert r.returncode == 0, tail
    assert "passed" in r.stdout and "AddressSanitizer" not in tail and "runtime error" not in tail, tail
