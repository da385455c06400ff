"""The CPU oracle under AddressSanitizer + UndefinedBehaviorSanitizer: a small C driver calls every
exported routine on ragged inputs; the sanitizers abort on any invalid access or undefined operation."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_clean_under_address_and_undefined_sanitizers(tmp_path):
    exe = tmp_path / "oracle_san"
    subprocess.check_call(["gcc", "-O1", "-g", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                           "-fno-omit-frame-pointer", "-o", str(exe),
                           os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c"),
                           os.path.join(ROOT, "oracle", "pevlm_oracle.c"), "-lm"])
    env = dict(os.environ)
    env.update(ASAN_OPTIONS="detect_leaks=1:verify_asan_link_order=0", OMP_NUM_THREADS="4")
    r = subprocess.run([str(exe)], capture_output=True, text=True, env=env)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "oracle sanitizer driver ok" in r.stdout
