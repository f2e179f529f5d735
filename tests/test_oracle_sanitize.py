"""The C oracle under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only): the oracle and a small C
driver that calls every entry point (both dtypes, adapters, synthetic cache rows, the refused cases) are
compiled together with -fsanitize=address,undefined and run as a plain program; any report fails the run."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    exe = tmp_path / "orc_san"
    subprocess.check_call(["gcc", "-O1", "-g", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                           "-fno-omit-frame-pointer", "-o", str(exe), os.path.join(ROOT, "oracle", "sd_oracle.c"),
                           os.path.join(ROOT, "tests", "oracle_sanitize_driver.c"), "-lm"])
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0", OMP_NUM_THREADS="2")
    r = subprocess.run([str(exe)], capture_output=True, text=True, timeout=300, env=env)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-4000:]
    assert "sanitize driver ok" in r.stdout
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr
