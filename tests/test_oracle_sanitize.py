"""The CPU oracle under the host sanitizers: oracle/aqt_oracle.c and a small C driver that
calls every routine on ragged shapes with exactly sized buffers are built with
-fsanitize=address,undefined (runtime linked statically, errors fatal) and run once."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_runs_clean_under_address_and_undefined_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_sanitized")
    cmd = ["gcc", "-O1", "-g", "-ffp-contract=off", "-fopenmp", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-static-libasan", "-static-libubsan", "-Wall", "-Wextra",
           os.path.join(ROOT, "oracle", "aqt_oracle.c"), os.path.join(ROOT, "tests", "oracle_sanitize_driver.c"),
           "-o", exe, "-lm"]
    b = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert b.returncode == 0, b.stdout
    env = dict(os.environ, OMP_NUM_THREADS="4",
               ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=120)
    if r.returncode != 0 and "LeakSanitizer has encountered a fatal error" in r.stdout:
        # the leak checker needs ptrace, which some sandboxes deny; everything else still runs
        env["ASAN_OPTIONS"] = "detect_leaks=0"
        r = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=120)
    sys.stdout.write(r.stdout)
    assert r.returncode == 0, r.stdout
    assert "oracle sanitizer run ok" in r.stdout
