"""AddressSanitizer + UndefinedBehaviorSanitizer over the CPU code (the oracle and the workload generators):
tests/sanitize_driver.cpp calls every entry point of both; here it is compiled together with their sources with
-fsanitize=address,undefined (no recovery: the first report aborts) and run once."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_and_generators_are_clean_under_asan_and_ubsan(tmp_path):
    exe = tmp_path / "sanitize_driver"
    cmd = ["g++", "-O1", "-g", "-std=c++17", "-pthread", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan",               # the runtime is part of the executable, whatever else is loaded first
           "-o", str(exe), os.path.join(ROOT, "tests", "sanitize_driver.cpp"),
           os.path.join(ROOT, "oracle", "bpe_oracle.cpp"), os.path.join(ROOT, "workloads", "gen.cpp")]
    subprocess.check_call(cmd)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=1:verify_asan_link_order=0",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    run = subprocess.run([str(exe)], env=env, capture_output=True, text=True, timeout=600)
    sys.stdout.write(run.stdout)
    sys.stderr.write(run.stderr[-4000:])
    assert run.returncode == 0, run.stderr[-2000:]
    assert run.stdout.startswith("sanitize_driver ok ")
