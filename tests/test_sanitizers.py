"""The host generator and both oracles under AddressSanitizer and UndefinedBehaviorSanitizer (host code only):
one program built from their sources (tests/sanitize/driver.cpp) runs them over generated batches, values near the
top of the 32-bit range included, and must end cleanly."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_generator_and_oracles_are_clean_under_asan_and_ubsan(tmp_path):
    exe = tmp_path / "san_driver"
    subprocess.run(["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                    "-pthread", "-o", str(exe), os.path.join(ROOT, "tests", "sanitize", "driver.cpp")], check=True)
    env = {**os.environ, "ASAN_OPTIONS": "verify_asan_link_order=0:detect_leaks=1"}
    r = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=600)
    assert r.returncode == 0 and r.stdout.strip() == "ok", (r.returncode, r.stdout[-500:], r.stderr[-2000:])
