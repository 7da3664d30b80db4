"""The C oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only, no GPU):
a driver calls every entry point on heap buffers of exactly the documented sizes over small and
ragged shapes; any access outside a buffer or undefined operation aborts the run."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRCS = [os.path.join(ROOT, "oracle", "loco_ref.c"), os.path.join(ROOT, "oracle", "loco_ref_mt.c"),
        os.path.join(ROOT, "tests", "oracle_sanitizer_driver.c")]


def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_san")
    cmd = ["gcc", "-O1", "-g", "-ffp-contract=off", "-fno-fast-math", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-static-libasan", "-static-libubsan", "-Wall", "-Wextra", "-o", exe, *SRCS,
           "-lm", "-lpthread"]
    built = subprocess.run(cmd, capture_output=True, text=True)
    assert built.returncode == 0, built.stderr
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], capture_output=True, text=True, timeout=600, env=env)
    assert run.returncode == 0, (run.stdout[-2000:], run.stderr[-4000:])
    assert run.stdout.startswith("ok "), run.stdout[-500:]
    assert int(run.stdout.split()[1]) > 5000
