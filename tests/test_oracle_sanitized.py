"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only, no GPU).

`oracle/slim_oracle.c` and a small driver are compiled into one executable with -fsanitize=address,undefined and
run: a read or write outside a buffer, a signed overflow or a misaligned access in the oracle ends the run with a
report and a non-zero exit code.  An executable of its own, so that nothing has to be preloaded into Python.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)


def test_oracle_is_clean_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_sanitize_driver")
    cmd = ["gcc", "-O1", "-g", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
           "-fno-fast-math", "-ffp-contract=off", "-Wall", "-Wextra", "-o", exe,
           os.path.join(HERE, "host_models", "oracle_sanitize_driver.c"), os.path.join(ROOT, "oracle", "slim_oracle.c"), "-lm"]
    subprocess.run(cmd, check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1", OMP_NUM_THREADS="4")
    r = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300, env=env)
    assert r.returncode == 0 and "clean" in r.stdout, r.stdout[-4000:]
